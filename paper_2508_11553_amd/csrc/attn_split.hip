// Split-K pass of paged decode attention for gfx950 (wave64, MFMA).
//
// One workgroup (4 waves) owns one (sequence b, KV head g, chunk c of
// `chunk_tokens` tokens).  All G query heads of the KV head ride in one MFMA
// tile, so every K/V byte of the chunk is fetched once.  Each wave walks the
// chunk in 32-token tiles (two pages), software-pipelined one tile ahead:
//
//   S^T[token][head] = K_tile[token][d] . Q^T[d][head]      mfma 16x16x32 bf16
//   online softmax over tokens (base 2; scale*log2e folded into the scores)
//   O^T[d][head]    += V^T[d][token] . P^T[token][head]      mfma 16x16x32 bf16
//
// Computing the transposed products makes the accumulator layout of the first
// MFMA (lane = head, registers = tokens) exactly the B-operand layout of the
// second one, so the weights never leave their lanes.  K tiles are loaded as
// a plain memory image (16 bytes per lane, fully coalesced) and turned into
// A-operand layout (lane = token) through a per-wave LDS scratch.  V rows are
// loaded as 8-byte pieces (16 lanes cover 128 contiguous bytes of a row) and
// transposed 4x4 inside each lane with byte permutes, because the second
// product contracts over tokens while memory is contiguous along d.
//
// The four waves' (max, sum, O) are merged through LDS and written as one
// partial per (b, head, chunk); the merge kernel finishes the softmax.
#include "kernels.h"

namespace sd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

#define SD_DEV __device__ __forceinline__

SD_DEV f32x4 mfma_bf16_k32(u32x4 a, u32x4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// (lo16 of x) | (lo16 of y) << 16, or the same with the high halves
SD_DEV unsigned pack_lo(unsigned x, unsigned y) { return __builtin_amdgcn_perm(y, x, 0x05040100u); }
SD_DEV unsigned pack_hi(unsigned x, unsigned y) { return __builtin_amdgcn_perm(y, x, 0x07060302u); }

// two floats -> packed bf16 pair, round-to-nearest-even (v_cvt_pk_bf16_f32)
SD_DEV unsigned cvt_pk_bf16(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 r;
    r[0] = (__bf16)lo;
    r[1] = (__bf16)hi;
    return __builtin_bit_cast(unsigned, r);
}

// K/V bytes are used once per launch: load them with the non-temporal hint so
// that they stream through the caches instead of displacing each other.
template <typename T>
SD_DEV T stream_load(const T *p) { return __builtin_nontemporal_load(p); }

// Reductions over the four lanes {n, n+16, n+32, n+48} that share a head.
// v_permlane16_swap exchanges rows 1<->0' and 3<->2' of its two operands and
// v_permlane32_swap the upper half of one with the lower half of the other;
// fed the same value twice they return (x, x from the partner row/half).
SD_DEV float head_max(float x)
{
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const float y = fmaxf(__builtin_bit_cast(float, a[0]), __builtin_bit_cast(float, a[1]));
    const unsigned w = __builtin_bit_cast(unsigned, y);
    const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
    return fmaxf(__builtin_bit_cast(float, b[0]), __builtin_bit_cast(float, b[1]));
}
SD_DEV float head_sum(float x)
{
    x += __shfl_xor(x, 16, 64);
    return x + __shfl_xor(x, 32, 64);
}

// Registers of one 32-token tile as they arrive from memory.
template <int D>
struct Tile {
    u32x4 k[2][D / 32];     // [page][j]: 16 bytes at byte offset 1024*j + 16*lane of the K tile
    u32x2 v[2][D / 64][4];  // [page][half][j]: V row 4*(lane>>4)+j, d = 64*half + 4*(lane&15) .. +4
};

template <int D>
SD_DEV void load_page_bf16(Tile<D> &r, int pg, const char *kp, const char *vp, int lane)
{
    const char *kl = kp + lane * 16;
#pragma unroll
    for (int j = 0; j < D / 32; ++j) r.k[pg][j] = stream_load(reinterpret_cast<const u32x4 *>(kl + j * 1024));
    const char *vl = vp + (lane >> 4) * 4 * (D * 2) + (lane & 15) * 8;
#pragma unroll
    for (int h = 0; h < D / 64; ++h)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            r.v[pg][h][j] = stream_load(reinterpret_cast<const u32x2 *>(vl + j * (D * 2) + h * 128));
}

template <int D>
struct WaveState {
    float m;                 // running max of this lane's head (same in the 4 lanes of a head)
    float l;                 // this lane's share of the weight sum
    f32x4 acc[D / 64][4];    // acc[h][i][r] = O[head lane&15][d = 64h + 16(lane>>4) + 4r + i]
};

// K tiles arrive as a plain image of memory (lane = 16 consecutive bytes), the
// only pattern in which a wave's load touches each cache line once.  The MFMA
// wants lane = token, so each K tile takes a round trip through this wave's
// own LDS scratch: written as it lies in memory, read back row-per-lane.
// 16-byte pieces of row r are stored at piece index (c ^ r) so that both the
// writes (16 lanes = one row) and the reads (16 lanes = one piece column of 16
// rows) spread over all banks.  Only the owning wave touches its scratch and
// LDS operations of one wave execute in order, so no barrier is needed; the
// fences keep the compiler from moving reads above writes.
template <int D>
SD_DEV void k_tile_to_operands(const Tile<D> &r, char *scratch, int lane, u32x4 (&ka)[D / 32], u32x4 (&kb)[D / 32])
{
    constexpr int kPieces = D / 8;            // 16-byte pieces per K row
    constexpr int kRowsPerLoad = 64 / kPieces;  // rows one 1024-byte load covers
    constexpr int kTile = kPage * D * 2;      // bytes of one (page, head) K tile
#pragma unroll
    for (int pg = 0; pg < 2; ++pg)
#pragma unroll
        for (int j = 0; j < D / 32; ++j) {
            const int row = j * kRowsPerLoad + lane / kPieces;
            const int piece = (lane % kPieces) ^ (row % kPieces);
            *reinterpret_cast<u32x4 *>(scratch + pg * kTile + row * (D * 2) + piece * 16) = r.k[pg][j];
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int t = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
        const int piece = (4 * s + kg) ^ (t % kPieces);
        ka[s] = *reinterpret_cast<const u32x4 *>(scratch + t * (D * 2) + piece * 16);
        kb[s] = *reinterpret_cast<const u32x4 *>(scratch + kTile + t * (D * 2) + piece * 16);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// One 32-token tile: tokens tok0 .. tok0+31, of which those < t_end are real.
template <int D>
SD_DEV void consume_tile(Tile<D> &r, const u32x4 (&qop)[D / 32], WaveState<D> &st,
                         float scale_log2e, int tok0, int t_end, int lane, char *scratch)
{
    const int qd = lane >> 4;
    f32x4 sa = {0, 0, 0, 0}, sb = {0, 0, 0, 0};
    {
        u32x4 ka[D / 32], kb[D / 32];  // K row (lane&15), d = 32*s + 8*(lane>>4) .. +8
        k_tile_to_operands<D>(r, scratch, lane, ka, kb);
#pragma unroll
        for (int s = 0; s < D / 32; ++s) {
            sa = mfma_bf16_k32(ka[s], qop[s], sa);
            sb = mfma_bf16_k32(kb[s], qop[s], sb);
        }
    }
    // lane holds, for head lane&15, tokens tok0 + 4qd + e (page A) and tok0 + 16 + 4qd + e (page B)
    float x[8];
    const bool ragged = tok0 + kTileTokens > t_end;  // wave-uniform
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[e] = sa[e] * scale_log2e;
        x[4 + e] = sb[e] * scale_log2e;
    }
    if (ragged) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (tok0 + 4 * qd + e >= t_end) x[e] = -INFINITY;
            if (tok0 + 16 + 4 * qd + e >= t_end) x[4 + e] = -INFINITY;
        }
    }
    float tmax = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    tmax = head_max(tmax);
    const float m_new = fmaxf(st.m, tmax);
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
    st.m = m_new;
    unsigned pw[4];
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(x[e] - m_new);
        const float p1 = __builtin_amdgcn_exp2f(x[e + 1] - m_new);
        const unsigned w = cvt_pk_bf16(p0, p1);
        pw[e >> 1] = w;
        // the sum runs over the rounded weights, the ones the product below uses
        psum += __builtin_bit_cast(float, w << 16) + __builtin_bit_cast(float, w & 0xffff0000u);
    }
    st.l = st.l * alpha + psum;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) st.acc[h][i] *= alpha;
    }
    const u32x4 pop = {pw[0], pw[1], pw[2], pw[3]};

    auto &v = r.v;
    if (ragged) {  // slots past the end may hold anything, NaN included: 0 * NaN must not happen
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (tok0 + 16 * pg + 4 * qd + j >= t_end) {
#pragma unroll
                    for (int h = 0; h < D / 64; ++h) v[pg][h][j] = u32x2{0, 0};
                }
    }
#pragma unroll
    for (int h = 0; h < D / 64; ++h) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int w = i >> 1;
            u32x4 a;
            if (i & 1) {
                a[0] = pack_hi(v[0][h][0][w], v[0][h][1][w]);
                a[1] = pack_hi(v[0][h][2][w], v[0][h][3][w]);
                a[2] = pack_hi(v[1][h][0][w], v[1][h][1][w]);
                a[3] = pack_hi(v[1][h][2][w], v[1][h][3][w]);
            } else {
                a[0] = pack_lo(v[0][h][0][w], v[0][h][1][w]);
                a[1] = pack_lo(v[0][h][2][w], v[0][h][3][w]);
                a[2] = pack_lo(v[1][h][0][w], v[1][h][1][w]);
                a[3] = pack_lo(v[1][h][2][w], v[1][h][3][w]);
            }
            st.acc[h][i] = mfma_bf16_k32(a, pop, st.acc[h][i]);
        }
    }
}

template <int D>
__global__ __launch_bounds__(kWaves * 64, 2) void split_bf16_kernel(SplitArgs a)
{
    constexpr int kRow = D + 4;  // padded LDS row: 16 heads x float4 stores hit 64 distinct banks
    __shared__ __attribute__((aligned(16))) float s_acc[kWaves][kMaxGroup][kRow];
    __shared__ __attribute__((aligned(16))) char s_k[kWaves][2 * kPage * D * 2];  // per-wave K transposition scratch
    __shared__ float s_m[kWaves][kMaxGroup];
    __shared__ float s_l[kWaves][kMaxGroup];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int item = blockIdx.x;  // (chunk, sequence, kv head), kv head fastest
    const int g = item % a.Hkv;
    const int b = (item / a.Hkv) % a.B;
    const int c = item / (a.Hkv * a.B);

    const int L = min(a.context_lens[b], a.max_context_len);
    const int t0 = c * a.chunk_tokens;
    if (t0 >= L) return;
    const int t1 = min(L, t0 + a.chunk_tokens);
    const int ntiles = (t1 - t0 + kTileTokens - 1) / kTileTokens;

    // Q^T operand: lane = head n, d = 32*step + 8*(lane>>4) .. +8; heads >= G are zero rows
    const int n = lane & 15;
    u32x4 qop[D / 32];
    {
        const uint16_t *qrow = a.q + ((int64_t)b * a.Hq + (int64_t)g * a.G + n) * D + (lane >> 4) * 8;
#pragma unroll
        for (int s = 0; s < D / 32; ++s)
            qop[s] = (n < a.G) ? *reinterpret_cast<const u32x4 *>(qrow + s * 32) : u32x4{0, 0, 0, 0};
    }

    WaveState<D> st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int h = 0; h < D / 64; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) st.acc[h][i] = f32x4{0, 0, 0, 0};

    const int32_t *bt = a.block_table + (int64_t)b * a.max_blocks + t0 / kPage;
    const int64_t tile_bytes = (int64_t)kPage * D * 2;
    const int64_t page_bytes = tile_bytes * a.Hkv;
    const char *kbase = static_cast<const char *>(a.k_pages) + g * tile_bytes;
    const char *vbase = static_cast<const char *>(a.v_pages) + g * tile_bytes;

    // This wave's tiles are wave, wave+4, ... : nt of them.  Loads for tile i+1 are
    // issued before tile i is consumed, and the page ids of tile i+2 are fetched
    // (scalar loads) one step earlier still.  Everything inside the loop is
    // unconditional so that the wait counters stay exact; a tile's missing
    // second page re-reads the first (its tokens are masked by position).
    const int nt = ntiles > wave ? (ntiles - wave + kWaves - 1) / kWaves : 0;
    const int last_page = (t1 - t0 + kPage - 1) / kPage - 1;
    auto page_ids = [&](int i, int &pa, int &pb) {
        const int ti = wave + kWaves * min(i, nt - 1);
        pa = bt[2 * ti];
        pb = bt[min(2 * ti + 1, last_page)];
    };
    auto issue = [&](Tile<D> &r, int pa, int pb) {
        load_page_bf16<D>(r, 0, kbase + pa * page_bytes, vbase + pa * page_bytes, lane);
        load_page_bf16<D>(r, 1, kbase + pb * page_bytes, vbase + pb * page_bytes, lane);
    };
    auto consume = [&](Tile<D> &r, int i) {
        consume_tile<D>(r, qop, st, a.scale_log2e, t0 + (wave + kWaves * i) * kTileTokens, t1, lane, s_k[wave]);
    };
    if (nt > 0) {
        Tile<D> ra, rb;
        int pa, pb;
        page_ids(0, pa, pb);
        issue(ra, pa, pb);
        page_ids(1, pa, pb);
        int i = 0;
        for (; i + 2 < nt; i += 2) {
            issue(rb, pa, pb);
            page_ids(i + 2, pa, pb);
            consume(ra, i);
            issue(ra, pa, pb);
            page_ids(i + 3, pa, pb);
            consume(rb, i + 1);
        }
        if (i + 1 < nt) {
            issue(rb, pa, pb);
            consume(ra, i);
            consume(rb, i + 1);
        } else {
            consume(ra, i);
        }
    }

    // the four lanes of a head hold disjoint shares of the weight sum
    st.l = head_sum(st.l);

    const int qd = lane >> 4;
    if (qd == 0) {
        s_m[wave][n] = st.m;
        s_l[wave][n] = st.l;
    }
#pragma unroll
    for (int h = 0; h < D / 64; ++h)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const f32x4 o = {st.acc[h][0][r], st.acc[h][1][r], st.acc[h][2][r], st.acc[h][3][r]};
            *reinterpret_cast<f32x4 *>(&s_acc[wave][n][64 * h + 16 * qd + 4 * r]) = o;
        }
    __syncthreads();

    // merge the four waves; wave 0 always saw at least one token, so the max is finite
    const int64_t row0 = (int64_t)b * a.Hq + (int64_t)g * a.G;
    for (int idx = tid; idx < a.G * D; idx += kWaves * 64) {
        const int hn = idx / D, dd = idx % D;
        float M = s_m[0][hn];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, s_m[w][hn]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float wt = __builtin_amdgcn_exp2f(s_m[w][hn] - M);
            num += wt * s_acc[w][hn][dd];
            den += wt * s_l[w][hn];
        }
        const int64_t slot = (row0 + hn) * a.S + c;
        a.ws_acc[slot * D + dd] = num;
        if (dd == 0) {
            a.ws_m[slot] = M;
            a.ws_l[slot] = den;
        }
    }
}

hipError_t launch_split(const SplitArgs &a, int head_dim, int kv_dtype, hipStream_t stream,
                        hipEvent_t start, hipEvent_t stop)
{
    const unsigned grid = (unsigned)a.S * (unsigned)a.B * (unsigned)a.Hkv;
    if (grid == 0) return hipSuccess;
    if (kv_dtype != 0) return hipErrorNotSupported;
    if (head_dim == 128)
        hipExtLaunchKernelGGL(split_bf16_kernel<128>, dim3(grid), dim3(kWaves * 64), 0, stream, start, stop, 0, a);
    else if (head_dim == 64)
        hipExtLaunchKernelGGL(split_bf16_kernel<64>, dim3(grid), dim3(kWaves * 64), 0, stream, start, stop, 0, a);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace sd
