// kv_append: scatter new bf16 K/V rows into their page slots.
// One thread moves 16 bytes; a row of one (token, kv head) is D*2/16 threads,
// so a wave writes whole contiguous rows.  Thread order: (token, head, piece),
// piece fastest, K and V by the same thread.
#include "kernels.h"

namespace sd {

template <int D>
__global__ __launch_bounds__(256) void append_kernel(AppendArgs a)
{
    constexpr int kPieces = D * 2 / 16;  // 16-byte pieces per row
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)a.T * a.Hkv * kPieces;
    if (gid >= total) return;
    const int piece = (int)(gid % kPieces);
    const int g = (int)((gid / kPieces) % a.Hkv);
    const int j = (int)(gid / ((int64_t)kPieces * a.Hkv));
    // without index arrays row j is the newest token of sequence j: position context_lens[j] - 1
    const int seq = a.seq_ids ? a.seq_ids[j] : j;
    const int pos = a.positions ? a.positions[j] : min(a.context_lens[j], a.max_context_len) - 1;
    if (pos < 0) return;
    const int64_t page = a.block_table[(int64_t)seq * a.max_blocks + pos / kPage];
    const int64_t dst = ((page * a.Hkv + g) * kPage + pos % kPage) * kPieces + piece;
    a.k_pages[dst] = a.k_new[gid];
    a.v_pages[dst] = a.v_new[gid];
}

hipError_t launch_append(const AppendArgs &a, int head_dim, hipStream_t stream)
{
    const int64_t total = (int64_t)a.T * a.Hkv * (head_dim * 2 / 16);
    if (total == 0) return hipSuccess;
    const unsigned grid = (unsigned)((total + 255) / 256);
    if (head_dim == 128)
        hipLaunchKernelGGL(append_kernel<128>, dim3(grid), dim3(256), 0, stream, a);
    else if (head_dim == 64)
        hipLaunchKernelGGL(append_kernel<64>, dim3(grid), dim3(256), 0, stream, a);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace sd

// ---------------------------------------------------------------------------
// Quantising append into fp8 e4m3fn pools (head_dim 128 or 64).
//
// Rows arrive as ranges of consecutive positions of one sequence.  One
// wave (four to a workgroup) owns one (range, page touched by the range, KV head, K or V) tile:
// lane l handles a quarter of a row, slot l/4, d = (D/4)*(l%4)..+D/4.
//   amax_new over the rows written into the tile        (wave max, exact)
//   the tile's scale stays if the range starts inside the page and
//   amax_new <= old_scale*448; otherwise scale = amax_new/448 (1 if 0) and the
//   codes of the slots before the range are re-encoded as dec*(old_scale/scale)
//   new codes = enc(x/scale): v_cvt_pk_fp8_f32 (round-to-nearest-even) after
//   clamping to +-448.
// A range that starts a page treats it as fresh and ignores its old scale.
// ---------------------------------------------------------------------------
namespace sd {

typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_lo(unsigned w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ __forceinline__ float clamp448(float y) { return fminf(fmaxf(y, -448.0f), 448.0f); }

// x / s for many x and one s, bit for bit what the division operator gives, at half its cost: the
// compiler expands a division into reciprocal, two refinements of it, two of the quotient and a
// fix-up of special cases, the first three of which depend on s alone.  Here they are done once per
// tile.  Outside the range of s in which the fix-up and the operand scaling have nothing to do (and
// for a zero, infinite or NaN s) the operator itself is used.  |x / s| <= 448 for every x of the
// tile, so the quotient cannot overflow; quotients below the smallest code round to zero whatever
// their last bits are.
struct Divisor {
    float s, r;
    bool plain;   // use the operator
};
__device__ __forceinline__ Divisor divisor(float s)
{
    Divisor d;
    d.s = s;
    const float r0 = __builtin_amdgcn_rcpf(s);
    d.r = __builtin_fmaf(__builtin_fmaf(-s, r0, 1.0f), r0, r0);
    d.plain = !(fabsf(s) >= 0x1p-60f && fabsf(s) <= 0x1p60f);
    return d;
}
__device__ __forceinline__ float quotient(float x, const Divisor &d)
{
    if (d.plain) return x / d.s;
    float q = x * d.r;
    q = __builtin_fmaf(__builtin_fmaf(-d.s, q, x), d.r, q);
    return __builtin_fmaf(__builtin_fmaf(-d.s, q, x), d.r, q);
}

// four floats -> four e4m3fn codes in one word (byte i = code of f[i])
__device__ __forceinline__ unsigned enc4(float a, float b, float c, float d)
{
    unsigned w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a), clamp448(b), w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(c), clamp448(d), w, true);
    return w;
}

template <int D>
__global__ __launch_bounds__(256) void append_fp8_kernel(AppendFp8Args a)
{
    constexpr int E = D / 4;    // elements one lane handles: a quarter of a row
    constexpr int NW = E / 8;   // 16-byte words of bf16 that is
    constexpr int NC = E / 16;  // and 16-byte words of codes
    const int lane = threadIdx.x & 63;
    // four independent waves per workgroup (no barrier below), one tile each
    const unsigned tile_id = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (tile_id >= a.num_tiles) return;
    const int which = tile_id & 1;                    // 0: K, 1: V
    const int g = (tile_id >> 1) % a.Hkv;
    const int pi = (tile_id >> 1) / a.Hkv % a.pages_per_range;
    const int r = (tile_id >> 1) / a.Hkv / a.pages_per_range;
    const int start = a.range_start[r], row0 = a.range_row0[r];
    const int end = start + (a.range_row0[r + 1] - row0);
    const int pg = start / kPage + pi;
    const int p0 = pg * kPage;
    if (p0 >= end) return;  // wave-uniform
    const int seq = a.range_seq[r];
    const int s0 = max(start - p0, 0), s1 = min(end - p0, kPage);
    const int64_t page = a.block_table[(int64_t)seq * a.max_blocks + pg];
    const int64_t tile_index = page * a.Hkv + g;
    uint4 *tile = reinterpret_cast<uint4 *>((which ? a.v_pages : a.k_pages) + tile_index * (kPage * D));
    float *scale_p = (which ? a.v_scales : a.k_scales) + tile_index;
    const uint4 *src = which ? a.v_new : a.k_new;

    // one wave per tile: lane -> slot lane/4, d = (D/4)*(lane%4) .. +D/4
    const int slot = lane >> 2, quarter = lane & 3;
    const bool is_new = slot >= s0 && slot < s1;
    float x[E];
#pragma unroll
    for (int i = 0; i < E; ++i) x[i] = 0.f;
    if (is_new) {
        const int64_t row = row0 + (p0 + slot - start);
        const uint4 *p = src + (row * a.Hkv + g) * (D / 8) + quarter * NW;
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            const uint4 w = p[j];
            x[8 * j + 0] = bf16_lo(w.x); x[8 * j + 1] = bf16_hi(w.x); x[8 * j + 2] = bf16_lo(w.y); x[8 * j + 3] = bf16_hi(w.y);
            x[8 * j + 4] = bf16_lo(w.z); x[8 * j + 5] = bf16_hi(w.z); x[8 * j + 6] = bf16_lo(w.w); x[8 * j + 7] = bf16_hi(w.w);
        }
    }
    float amax_new = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) amax_new = fmaxf(amax_new, fabsf(x[i]));
    for (int off = 32; off > 0; off >>= 1) amax_new = fmaxf(amax_new, __shfl_xor(amax_new, off, 64));

    const float old_scale = s0 > 0 ? *scale_p : 0.f;
    const float old_amax = old_scale * 448.0f;
    const bool keep = s0 > 0 && amax_new <= old_amax;
    const float scale = keep ? old_scale : (amax_new > 0.f ? amax_new / 448.0f : 1.0f);
    const float ratio = old_scale / scale;  // re-encoding factor, one per tile
    const Divisor by = divisor(scale);
    if (!keep) {
        if (slot < s0) {  // re-encode what the page already held
#pragma unroll
            for (int j = 0; j < NC; ++j) {
                const uint4 c = tile[slot * (D / 16) + quarter * NC + j];
                const unsigned in[4] = {c.x, c.y, c.z, c.w};
                unsigned o[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(in[w], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(in[w], true);
                    o[w] = enc4(lo[0] * ratio, lo[1] * ratio, hi[0] * ratio, hi[1] * ratio);
                }
                tile[slot * (D / 16) + quarter * NC + j] = uint4{o[0], o[1], o[2], o[3]};
            }
        }
        if (lane == 0) *scale_p = scale;  // every lane has read the old scale: one wave runs in lockstep
    }
    if (is_new) {
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            unsigned o[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const int e = 16 * j + 4 * w;
                o[w] = enc4(quotient(x[e], by), quotient(x[e + 1], by), quotient(x[e + 2], by), quotient(x[e + 3], by));
            }
            tile[slot * (D / 16) + quarter * NC + j] = uint4{o[0], o[1], o[2], o[3]};
        }
    }
}

// The decode step's form of the same operation: every range is a single row, so
// a tile is touched in one slot only and 4 lanes (a quarter of the row each) are enough
// for it.  Lane group u = (range, KV head, K or V); 16 groups per wave.  Same
// arithmetic, in the same order, as append_fp8_kernel.
template <int D>
__global__ __launch_bounds__(256) void append_fp8_row_kernel(AppendFp8Args a)
{
    constexpr int E = D / 4;    // elements one lane handles: a quarter of a row
    constexpr int NW = E / 8;   // 16-byte words of bf16 that is
    constexpr int NC = E / 16;  // and 16-byte words of codes
    const unsigned gid = blockIdx.x * 256u + threadIdx.x;
    const unsigned unit = gid >> 2;
    const int quarter = gid & 3;
    if (unit >= a.num_tiles) return;  // whole 4-lane groups leave together
    const int which = unit & 1;
    const int g = (unit >> 1) % a.Hkv;
    const int r = (unit >> 1) / a.Hkv;
    const int row0 = a.range_row0[r];
    if (a.range_row0[r + 1] - row0 <= 0) return;
    const int start = a.range_start[r], seq = a.range_seq[r];
    const int s0 = start % kPage;
    const int64_t page = a.block_table[(int64_t)seq * a.max_blocks + start / kPage];
    const int64_t tile_index = page * a.Hkv + g;
    uint4 *tile = reinterpret_cast<uint4 *>((which ? a.v_pages : a.k_pages) + tile_index * (kPage * D));
    float *scale_p = (which ? a.v_scales : a.k_scales) + tile_index;
    const uint4 *p = (which ? a.v_new : a.k_new) + ((int64_t)row0 * a.Hkv + g) * (D / 8) + quarter * NW;
    float x[E];
#pragma unroll
    for (int j = 0; j < NW; ++j) {
        const uint4 w = p[j];
        x[8 * j + 0] = bf16_lo(w.x); x[8 * j + 1] = bf16_hi(w.x); x[8 * j + 2] = bf16_lo(w.y); x[8 * j + 3] = bf16_hi(w.y);
        x[8 * j + 4] = bf16_lo(w.z); x[8 * j + 5] = bf16_hi(w.z); x[8 * j + 6] = bf16_lo(w.w); x[8 * j + 7] = bf16_hi(w.w);
    }
    float amax_new = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) amax_new = fmaxf(amax_new, fabsf(x[i]));
    amax_new = fmaxf(amax_new, __shfl_xor(amax_new, 1, 64));
    amax_new = fmaxf(amax_new, __shfl_xor(amax_new, 2, 64));

    const float old_scale = s0 > 0 ? *scale_p : 0.f;
    const float old_amax = old_scale * 448.0f;
    const bool keep = s0 > 0 && amax_new <= old_amax;
    const float scale = keep ? old_scale : (amax_new > 0.f ? amax_new / 448.0f : 1.0f);
    const float ratio = old_scale / scale;  // re-encoding factor, one per tile
    const Divisor by = divisor(scale);
    if (!keep) {
        // re-encode what the page already held: eight slots' loads in flight at a time
        for (int base = 0; base < s0; base += 8) {
            uint4 c[8][NC];
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < NC; ++j)
                    if (base + i < s0) c[i][j] = tile[(base + i) * (D / 16) + quarter * NC + j];
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < NC; ++j) {
                    if (base + i >= s0) continue;
                    const unsigned in[4] = {c[i][j].x, c[i][j].y, c[i][j].z, c[i][j].w};
                    unsigned o[4];
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(in[w], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(in[w], true);
                        o[w] = enc4(lo[0] * ratio, lo[1] * ratio, hi[0] * ratio, hi[1] * ratio);
                    }
                    tile[(base + i) * (D / 16) + quarter * NC + j] = uint4{o[0], o[1], o[2], o[3]};
                }
        }
        if (quarter == 0) *scale_p = scale;  // the group's four lanes read the old scale in the same instruction
    }
#pragma unroll
    for (int j = 0; j < NC; ++j) {
        unsigned o[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int e = 16 * j + 4 * w;
            o[w] = enc4(quotient(x[e], by), quotient(x[e + 1], by), quotient(x[e + 2], by), quotient(x[e + 3], by));
        }
        tile[s0 * (D / 16) + quarter * NC + j] = uint4{o[0], o[1], o[2], o[3]};
    }
}

hipError_t launch_append_fp8(const AppendFp8Args &a, int head_dim, hipStream_t stream)
{
    if (a.num_tiles == 0) return hipSuccess;
    const bool rows = a.pages_per_range == 1 && a.single_rows;
    const dim3 grid(rows ? (a.num_tiles + 63) / 64 : (a.num_tiles + 3) / 4);
    if (head_dim == 128) {
        if (rows) hipLaunchKernelGGL(append_fp8_row_kernel<128>, grid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL(append_fp8_kernel<128>, grid, dim3(256), 0, stream, a);
    } else if (head_dim == 64) {
        if (rows) hipLaunchKernelGGL(append_fp8_row_kernel<64>, grid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL(append_fp8_kernel<64>, grid, dim3(256), 0, stream, a);
    } else {
        return hipErrorNotSupported;
    }
    return hipGetLastError();
}

// Whole-page copies inside the pool: one workgroup per (pair, K or V); the page of
// all heads is contiguous, so this is a straight 16-byte-per-lane copy.  The first
// workgroup of a pair also copies the page's scales.
__global__ __launch_bounds__(256) void copy_pages_kernel(CopyPagesArgs a)
{
    const int pair = blockIdx.x >> 1, is_v = blockIdx.x & 1;
    const int src = a.src_pages[pair], dst = a.dst_pages[pair];
    if (src < 0 || dst < 0 || src >= a.num_pages || dst >= a.num_pages || src == dst) return;
    uint4 *pool = is_v ? a.v_pages : a.k_pages;
    const uint4 *from = pool + (int64_t)src * a.page_words;
    uint4 *to = pool + (int64_t)dst * a.page_words;
    for (int i = threadIdx.x; i < a.page_words; i += 256) to[i] = from[i];
    float *scales = is_v ? a.v_scales : a.k_scales;
    if (scales)
        for (int i = threadIdx.x; i < a.Hkv; i += 256) scales[(int64_t)dst * a.Hkv + i] = scales[(int64_t)src * a.Hkv + i];
}

hipError_t launch_copy_pages(const CopyPagesArgs &a, hipStream_t stream)
{
    if (a.N <= 0) return hipSuccess;
    hipLaunchKernelGGL(copy_pages_kernel, dim3(2u * (unsigned)a.N), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace sd
