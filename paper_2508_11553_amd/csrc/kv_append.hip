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
    const int seq = a.seq_ids[j], pos = a.positions[j];
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
// Quantising append into fp8 e4m3fn pools (head_dim 128).
//
// Rows arrive as ranges of consecutive positions of one sequence.  One
// workgroup owns one (range, page touched by the range, KV head, K or V) tile:
// thread t handles 8 elements, slot t/16, d = 8*(t%16)..+8.
//   amax_new over the rows written into the tile        (block max, exact)
//   the tile's scale stays if the range starts inside the page and
//   amax_new <= old_scale*448; otherwise scale = amax_new/448 (1 if 0) and the
//   codes of the slots before the range are re-encoded as (dec*old_scale)/scale
//   new codes = enc(x/scale): v_cvt_pk_fp8_f32 (round-to-nearest-even) after
//   clamping to +-448.
// A range that starts a page treats it as fresh and ignores its old scale.
// ---------------------------------------------------------------------------
namespace sd {

typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_lo(unsigned w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ __forceinline__ float clamp448(float y) { return fminf(fmaxf(y, -448.0f), 448.0f); }

// four floats -> four e4m3fn codes in one word (byte i = code of f[i])
__device__ __forceinline__ unsigned enc4(float a, float b, float c, float d)
{
    unsigned w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a), clamp448(b), w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(c), clamp448(d), w, true);
    return w;
}

__global__ __launch_bounds__(256) void append_fp8_kernel(AppendFp8Args a)
{
    constexpr int D = 128;
    __shared__ float s_max[4];
    const int tid = threadIdx.x;
    const int which = blockIdx.x & 1;                 // 0: K, 1: V
    const int g = (blockIdx.x >> 1) % a.Hkv;
    const int pi = (blockIdx.x >> 1) / a.Hkv % a.pages_per_range;
    const int r = (blockIdx.x >> 1) / a.Hkv / a.pages_per_range;
    const int seq = a.range_seq[r], start = a.range_start[r], row0 = a.range_row0[r];
    const int end = start + (a.range_row0[r + 1] - row0);
    const int pg = start / kPage + pi;
    const int p0 = pg * kPage;
    if (p0 >= end) return;  // workgroup-uniform
    const int s0 = max(start - p0, 0), s1 = min(end - p0, kPage);
    const int64_t page = a.block_table[(int64_t)seq * a.max_blocks + pg];
    const int64_t tile_index = page * a.Hkv + g;
    uint2 *tile = reinterpret_cast<uint2 *>((which ? a.v_pages : a.k_pages) + tile_index * (kPage * D));
    float *scale_p = (which ? a.v_scales : a.k_scales) + tile_index;
    const uint4 *src = which ? a.v_new : a.k_new;

    const int slot = tid >> 4, piece = tid & 15;
    const bool is_new = slot >= s0 && slot < s1;
    float x[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (is_new) {
        const int64_t row = row0 + (p0 + slot - start);
        const uint4 w = src[(row * a.Hkv + g) * (D / 8) + piece];
        x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
        x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
    }
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(x[i]));
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((tid & 63) == 0) s_max[tid >> 6] = m;
    __syncthreads();
    const float amax_new = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));

    const float old_scale = s0 > 0 ? *scale_p : 0.f;
    const float old_amax = old_scale * 448.0f;
    const bool keep = s0 > 0 && amax_new <= old_amax;
    const float scale = keep ? old_scale : (amax_new > 0.f ? amax_new / 448.0f : 1.0f);
    __syncthreads();  // every thread has read the old scale before it is replaced
    if (!keep) {
        if (slot < s0) {  // re-encode what the page already held
            const uint2 c = tile[slot * (D / 8) + piece];
            const f32x2 a0 = __builtin_amdgcn_cvt_pk_f32_fp8(c.x, false), a1 = __builtin_amdgcn_cvt_pk_f32_fp8(c.x, true);
            const f32x2 b0 = __builtin_amdgcn_cvt_pk_f32_fp8(c.y, false), b1 = __builtin_amdgcn_cvt_pk_f32_fp8(c.y, true);
            uint2 o;
            o.x = enc4((a0[0] * old_scale) / scale, (a0[1] * old_scale) / scale, (a1[0] * old_scale) / scale, (a1[1] * old_scale) / scale);
            o.y = enc4((b0[0] * old_scale) / scale, (b0[1] * old_scale) / scale, (b1[0] * old_scale) / scale, (b1[1] * old_scale) / scale);
            tile[slot * (D / 8) + piece] = o;
        }
        if (tid == 0) *scale_p = scale;
    }
    if (is_new) {
        uint2 o;
        o.x = enc4(x[0] / scale, x[1] / scale, x[2] / scale, x[3] / scale);
        o.y = enc4(x[4] / scale, x[5] / scale, x[6] / scale, x[7] / scale);
        tile[slot * (D / 8) + piece] = o;
    }
}

hipError_t launch_append_fp8(const AppendFp8Args &a, hipStream_t stream)
{
    const uint64_t grid = 2ull * (uint64_t)a.R * (uint64_t)a.pages_per_range * (uint64_t)a.Hkv;
    if (grid == 0) return hipSuccess;
    if (grid > 0x7fffffffull) return hipErrorNotSupported;
    hipLaunchKernelGGL(append_fp8_kernel, dim3((unsigned)grid), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace sd
