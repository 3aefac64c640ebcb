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
// loaded in pieces of which 16 lanes cover 128 contiguous bytes of a row, and
// the token-major operand is formed inside each lane (byte permutes for bf16,
// the fp8->bf16 conversion itself for fp8), because the second product
// contracts over tokens while memory is contiguous along d.
//
// fp8 pools (OCP e4m3fn codes with one fp32 scale per page and head) are
// converted to bf16 in registers, which is exact; the K scale multiplies the
// page's scores and the V scale multiplies the page's weights.
//
// The four waves' (max, sum, O) are merged through LDS and written as one
// partial per (b, head, chunk); the merge kernel finishes the softmax.
#include "kernels.h"

namespace sd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
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
    bf16x2 r;
    r[0] = (__bf16)lo;
    r[1] = (__bf16)hi;
    return __builtin_bit_cast(unsigned, r);
}

// two e4m3fn codes (one 16-bit half of w) -> packed bf16 pair, exact.  The
// instruction applies only the power-of-two part of its scale operand; 1.0
// leaves the values as they are.
template <bool HI>
SD_DEV unsigned cvt_pk_bf16_fp8(unsigned w)
{
    return __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, HI));
}

// K/V bytes that one wave uses once per launch are loaded with the
// non-temporal hint, so that they stream through the caches instead of
// displacing each other (STREAM = true).  Bytes that the four waves of a
// workgroup all read (shared-prefix items) take ordinary loads: the first wave
// to ask brings a line in and the caches serve the other three.
template <bool STREAM, typename T>
SD_DEV T kv_load(const T *p)
{
    if (STREAM) return __builtin_nontemporal_load(p);
    return *p;
}

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

// Keeps the compiler from moving this wave's LDS reads above its LDS writes
// (and the other way round).  Only the owning wave touches its scratch and the
// LDS operations of one wave execute in order, so no workgroup barrier is needed.
SD_DEV void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int D>
struct WaveState {
    float m;             // running max of this lane's head (same in the 4 lanes of a head)
    float l;             // this lane's share of the weight sum
    f32x4 acc[D / 16];   // O^T accumulators; which d each one holds is the path's business
};

// Scores of one tile -> weights.  x holds, for head lane&15, the scaled scores
// of tokens tok0 + 4qd + e (e < 4, first page) and tok0 + 16 + 4qd + e - 4
// (second page).  Updates the running max and rescales the accumulators when
// some head's max moved.  Returns exp2(x - m) in p.
template <int D>
SD_DEV void online_softmax(float (&x)[8], float (&p)[8], WaveState<D> &st, bool ragged, int tok0, int t_end, int qd)
{
    if (ragged) {  // mask by position, never by content
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
#pragma unroll
    for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(x[e] - m_new);
    st.l *= alpha;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {
#pragma unroll
        for (int i = 0; i < D / 16; ++i) st.acc[i] *= alpha;
    }
}

// ---------------------------------------------------------------------------
// bf16 pools
// ---------------------------------------------------------------------------
template <int D>
struct Bf16Path {
    static constexpr int kDim = D;
    static constexpr int kTileBytes = kPage * D * 2;     // one (page, head) tile
    static constexpr int kScratchBytes = 2 * kTileBytes;  // K of one 32-token tile in LDS
    static constexpr int kVBytes = 2 * kTileBytes;        // V registers of one tile parked in LDS
    static constexpr int kPieces = D / 8;                 // 16-byte pieces per K row
    static constexpr int kRowsPerLoad = 64 / kPieces;     // K rows one 1024-byte load covers

    struct Tile {
        u32x4 k[2][D / 32];     // [page][j]: 16 bytes at byte offset 1024*j + 16*lane of the K tile
        u32x2 v[2][D / 64][4];  // [page][half][j]: V row 4*(lane>>4)+j, d = 64*half + 4*(lane&15) .. +4
    };

    // Q^T operand of step s: head lane&15, d = 32*s + 8*(lane>>4) .. +8
    SD_DEV static int q_offset(int s, int lane) { return 32 * s + 8 * (lane >> 4); }

    template <bool STREAM>
    SD_DEV static void load_page(Tile &r, int pg, const char *kp, const char *vp, const float *, const float *, int64_t, int lane)
    {
        const char *kl = kp + lane * 16;
#pragma unroll
        for (int j = 0; j < D / 32; ++j) r.k[pg][j] = kv_load<STREAM>(reinterpret_cast<const u32x4 *>(kl + j * 1024));
        const char *vl = vp + (lane >> 4) * 4 * (D * 2) + (lane & 15) * 8;
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                r.v[pg][h][j] = kv_load<STREAM>(reinterpret_cast<const u32x2 *>(vl + j * (D * 2) + h * 128));
    }

    // K tiles go through LDS: written as they lie in memory, read back one row
    // per lane.  Piece c of row r sits at piece index c ^ r so that the writes
    // (16 lanes = one row) and the reads (16 lanes = one piece column over 16
    // rows) both spread over all banks.
    SD_DEV static void k_store(const Tile &r, char *kslot, int lane)
    {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int j = 0; j < D / 32; ++j) {
                const int row = j * kRowsPerLoad + lane / kPieces;
                const int piece = (lane % kPieces) ^ (row % kPieces);
                *reinterpret_cast<u32x4 *>(kslot + pg * kTileBytes + row * (D * 2) + piece * 16) = r.k[pg][j];
            }
    }

    // K row (lane&15), d = 32*s + 8*(lane>>4) .. +8, of both pages
    SD_DEV static void k_fetch(const char *kslot, int lane, u32x4 (&ka)[D / 32], u32x4 (&kb)[D / 32])
    {
        const int t = lane & 15, kg = lane >> 4;
#pragma unroll
        for (int s = 0; s < D / 32; ++s) {
            const int piece = (4 * s + kg) ^ (t % kPieces);
            ka[s] = *reinterpret_cast<const u32x4 *>(kslot + t * (D * 2) + piece * 16);
            kb[s] = *reinterpret_cast<const u32x4 *>(kslot + kTileBytes + t * (D * 2) + piece * 16);
        }
    }

    // V registers (the same for every wave that consumes the tile) parked in LDS, lane-linear
    SD_DEV static void v_store(const Tile &r, char *vslot, int lane)
    {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int h = 0; h < D / 64; ++h)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const u32x4 w = {r.v[pg][h][2 * jj][0], r.v[pg][h][2 * jj][1], r.v[pg][h][2 * jj + 1][0],
                                     r.v[pg][h][2 * jj + 1][1]};
                    *reinterpret_cast<u32x4 *>(vslot + ((pg * (D / 64) + h) * 2 + jj) * 1024 + lane * 16) = w;
                }
    }
    SD_DEV static void v_fetch(Tile &r, const char *vslot, int lane)
    {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int h = 0; h < D / 64; ++h)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const u32x4 w = *reinterpret_cast<const u32x4 *>(vslot + ((pg * (D / 64) + h) * 2 + jj) * 1024 + lane * 16);
                    r.v[pg][h][2 * jj] = u32x2{w[0], w[1]};
                    r.v[pg][h][2 * jj + 1] = u32x2{w[2], w[3]};
                }
    }

    // Scores, online softmax and weighted V sum of one 32-token tile: tokens
    // tok0 .. tok0+31, of which those < t_end are real.  ka/kb: K operands of
    // the two pages; r.v: the V registers.
    SD_DEV static void attend(const u32x4 (&ka)[D / 32], const u32x4 (&kb)[D / 32], Tile &r,
                              const u32x4 (&qop)[D / 32], WaveState<D> &st, float scale_log2e, int tok0, int t_end,
                              int lane)
    {
        const int qd = lane >> 4;
        f32x4 sa = {0, 0, 0, 0}, sb = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < D / 32; ++s) {
            sa = mfma_bf16_k32(ka[s], qop[s], sa);
            sb = mfma_bf16_k32(kb[s], qop[s], sb);
        }
        const bool ragged = tok0 + kTileTokens > t_end;  // wave-uniform
        float x[8], p[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = sa[e] * scale_log2e;
            x[4 + e] = sb[e] * scale_log2e;
        }
        online_softmax<D>(x, p, st, ragged, tok0, t_end, qd);
        u32x4 pop;
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const unsigned w = cvt_pk_bf16(p[e], p[e + 1]);
            pop[e >> 1] = w;
            // the sum runs over the rounded weights, the ones the product below uses
            psum += __builtin_bit_cast(float, w << 16) + __builtin_bit_cast(float, w & 0xffff0000u);
        }
        st.l += psum;

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
        // acc[4h + i][r] = O[head lane&15][d = 64h + 16qd + 4r + i]
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
                st.acc[4 * h + i] = mfma_bf16_k32(a, pop, st.acc[4 * h + i]);
            }
        }
    }

    // this lane's accumulators -> row `dst` ([D] floats) of its head
    SD_DEV static void store_acc(const WaveState<D> &st, float *dst, int qd)
    {
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const f32x4 o = {st.acc[4 * h][r], st.acc[4 * h + 1][r], st.acc[4 * h + 2][r], st.acc[4 * h + 3][r]};
                *reinterpret_cast<f32x4 *>(dst + 64 * h + 16 * qd + 4 * r) = o;
            }
    }
};

// ---------------------------------------------------------------------------
// fp8 e4m3fn pools, head_dim 128: rows of 128 bytes, tiles of 2 KB
// ---------------------------------------------------------------------------
struct Fp8Path {
    static constexpr int D = 128;
    static constexpr int kDim = D;
    static constexpr int kTileBytes = kPage * D;
    static constexpr int kScratchBytes = 2 * kTileBytes;
    static constexpr int kVBytes = 2 * kTileBytes + 16;  // codes + the four page scales

    struct Tile {
        u32x4 k[2][2];  // [page][j]: 16 bytes at byte offset 1024*j + 16*lane of the K tile
        u32x2 v[2][4];  // [page][j]: V row 4*(lane>>4)+j, d = 8*(lane&15) .. +8
        float ks[2], vs[2];
    };

    // Step s of the first product uses the 8 codes at d = 16*(kg + 4*(s>>1)) + 8*(s&1)
    // of the lane's K row (kg = lane>>4): each lane converts two 16-byte pieces.
    SD_DEV static int q_offset(int s, int lane) { return 16 * ((lane >> 4) + 4 * (s >> 1)) + 8 * (s & 1); }

    template <bool STREAM>
    SD_DEV static void load_page(Tile &r, int pg, const char *kp, const char *vp, const float *ks, const float *vs, int64_t si, int lane)
    {
        const char *kl = kp + lane * 16;
        r.k[pg][0] = kv_load<STREAM>(reinterpret_cast<const u32x4 *>(kl));
        r.k[pg][1] = kv_load<STREAM>(reinterpret_cast<const u32x4 *>(kl + 1024));
        const char *vl = vp + (lane >> 4) * 4 * D + (lane & 15) * 8;
#pragma unroll
        for (int j = 0; j < 4; ++j) r.v[pg][j] = kv_load<STREAM>(reinterpret_cast<const u32x2 *>(vl + j * D));
        r.ks[pg] = ks[si];
        r.vs[pg] = vs[si];
    }

    // Rows are 128 bytes = 8 pieces; piece c of row r sits at c ^ (r >> 1), and
    // odd rows start half a bank cycle later, so 16 lanes never share a bank.
    SD_DEV static void k_store(const Tile &r, char *kslot, int lane)
    {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = 8 * j + (lane >> 3);
                const int piece = (lane & 7) ^ ((row >> 1) & 7);
                *reinterpret_cast<u32x4 *>(kslot + pg * kTileBytes + row * D + piece * 16) = r.k[pg][j];
            }
    }

    SD_DEV static void k_fetch(const char *kslot, int lane, u32x4 (&ka)[4], u32x4 (&kb)[4])
    {
        const int t = lane & 15, kg = lane >> 4;
        u32x4 raw[2][2];
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const int piece = (kg + 4 * hh) ^ ((t >> 1) & 7);
                raw[pg][hh] = *reinterpret_cast<const u32x4 *>(kslot + pg * kTileBytes + t * D + piece * 16);
            }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int hh = s >> 1, lo = 2 * (s & 1);
            ka[s] = u32x4{cvt_pk_bf16_fp8<false>(raw[0][hh][lo]), cvt_pk_bf16_fp8<true>(raw[0][hh][lo]),
                          cvt_pk_bf16_fp8<false>(raw[0][hh][lo + 1]), cvt_pk_bf16_fp8<true>(raw[0][hh][lo + 1])};
            kb[s] = u32x4{cvt_pk_bf16_fp8<false>(raw[1][hh][lo]), cvt_pk_bf16_fp8<true>(raw[1][hh][lo]),
                          cvt_pk_bf16_fp8<false>(raw[1][hh][lo + 1]), cvt_pk_bf16_fp8<true>(raw[1][hh][lo + 1])};
        }
    }

    // V registers and the four page scales parked in LDS (scales after the 4 KB of codes)
    SD_DEV static void v_store(const Tile &r, char *vslot, int lane)
    {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const u32x4 w = {r.v[pg][2 * jj][0], r.v[pg][2 * jj][1], r.v[pg][2 * jj + 1][0], r.v[pg][2 * jj + 1][1]};
                *reinterpret_cast<u32x4 *>(vslot + (pg * 2 + jj) * 1024 + lane * 16) = w;
            }
        if (lane == 0) *reinterpret_cast<f32x4 *>(vslot + 4096) = f32x4{r.ks[0], r.ks[1], r.vs[0], r.vs[1]};
    }
    SD_DEV static void v_fetch(Tile &r, const char *vslot, int lane)
    {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const u32x4 w = *reinterpret_cast<const u32x4 *>(vslot + (pg * 2 + jj) * 1024 + lane * 16);
                r.v[pg][2 * jj] = u32x2{w[0], w[1]};
                r.v[pg][2 * jj + 1] = u32x2{w[2], w[3]};
            }
        const f32x4 sc = *reinterpret_cast<const f32x4 *>(vslot + 4096);
        r.ks[0] = sc[0];
        r.ks[1] = sc[1];
        r.vs[0] = sc[2];
        r.vs[1] = sc[3];
    }

    SD_DEV static void attend(const u32x4 (&ka)[4], const u32x4 (&kb)[4], Tile &r, const u32x4 (&qop)[4],
                              WaveState<D> &st, float scale_log2e, int tok0, int t_end, int lane)
    {
        const int qd = lane >> 4;
        f32x4 sa = {0, 0, 0, 0}, sb = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            sa = mfma_bf16_k32(ka[s], qop[s], sa);
            sb = mfma_bf16_k32(kb[s], qop[s], sb);
        }
        const bool ragged = tok0 + kTileTokens > t_end;
        const float ca = scale_log2e * r.ks[0], cb = scale_log2e * r.ks[1];
        float x[8], p[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = sa[e] * ca;
            x[4 + e] = sb[e] * cb;
        }
        online_softmax<D>(x, p, st, ragged, tok0, t_end, qd);
        // the weight sum takes the unscaled weights; the product takes them times the page's V scale
        st.l += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
        u32x4 pop;
        pop[0] = cvt_pk_bf16(p[0] * r.vs[0], p[1] * r.vs[0]);
        pop[1] = cvt_pk_bf16(p[2] * r.vs[0], p[3] * r.vs[0]);
        pop[2] = cvt_pk_bf16(p[4] * r.vs[1], p[5] * r.vs[1]);
        pop[3] = cvt_pk_bf16(p[6] * r.vs[1], p[7] * r.vs[1]);

        auto &v = r.v;
        if (ragged) {
#pragma unroll
            for (int pg = 0; pg < 2; ++pg)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (tok0 + 16 * pg + 4 * qd + j >= t_end) v[pg][j] = u32x2{0, 0};
        }
        // acc[i][r] = O[head lane&15][d = 8*(4qd + r) + i]: codes i, i+1 of four tokens at a time;
        // converting to f32 and packing two tokens' values per register is the transposition.
#pragma unroll
        for (int w = 0; w < 2; ++w) {
#pragma unroll
            for (int hi = 0; hi < 2; ++hi) {
                f32x2 f[2][4];
#pragma unroll
                for (int pg = 0; pg < 2; ++pg)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        f[pg][j] = hi ? __builtin_amdgcn_cvt_pk_f32_fp8(v[pg][j][w], true)
                                      : __builtin_amdgcn_cvt_pk_f32_fp8(v[pg][j][w], false);
#pragma unroll
                for (int ii = 0; ii < 2; ++ii) {
                    const int i = 4 * w + 2 * hi + ii;
                    const u32x4 a = {cvt_pk_bf16(f[0][0][ii], f[0][1][ii]), cvt_pk_bf16(f[0][2][ii], f[0][3][ii]),
                                     cvt_pk_bf16(f[1][0][ii], f[1][1][ii]), cvt_pk_bf16(f[1][2][ii], f[1][3][ii])};
                    st.acc[i] = mfma_bf16_k32(a, pop, st.acc[i]);
                }
            }
        }
    }

    SD_DEV static void store_acc(const WaveState<D> &st, float *dst, int qd)
    {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const f32x4 lo = {st.acc[0][r], st.acc[1][r], st.acc[2][r], st.acc[3][r]};
            const f32x4 hi = {st.acc[4][r], st.acc[5][r], st.acc[6][r], st.acc[7][r]};
            *reinterpret_cast<f32x4 *>(dst + 32 * qd + 8 * r) = lo;
            *reinterpret_cast<f32x4 *>(dst + 32 * qd + 8 * r + 4) = hi;
        }
    }
};

// Streams the tiles first, first+stride, ... of the chunk [t0, t1) through this
// wave.  Loads for tile i+1 are issued before tile i is consumed, and the page
// ids of tile i+2 are fetched (scalar loads) one step earlier still.
// Everything inside the loop is unconditional so that the wait counters stay
// exact; a tile's missing second page re-reads the first (its tokens are
// masked by position).  `bt` points at the table entry of the chunk's first page.
template <class P, bool STREAM>
SD_DEV void stream_tiles(const SplitArgs &a, const int32_t *bt, int g, int t0, int t1, int first, int stride,
                         const u32x4 (&qop)[P::kDim / 32], WaveState<P::kDim> &st, char *scratch, int lane)
{
    const int ntiles = (t1 - t0 + kTileTokens - 1) / kTileTokens;
    const int nt = ntiles > first ? (ntiles - first + stride - 1) / stride : 0;
    if (nt <= 0) return;
    const int last_page = (t1 - t0 + kPage - 1) / kPage - 1;
    const int64_t page_bytes = (int64_t)P::kTileBytes * a.Hkv;
    const char *kbase = static_cast<const char *>(a.k_pages) + g * P::kTileBytes;
    const char *vbase = static_cast<const char *>(a.v_pages) + g * P::kTileBytes;
    auto page_ids = [&](int i, int &pa, int &pb) {
        const int ti = first + stride * min(i, nt - 1);
        pa = bt[2 * ti];
        pb = bt[min(2 * ti + 1, last_page)];
    };
    auto issue = [&](typename P::Tile &r, int pa, int pb) {
        P::template load_page<STREAM>(r, 0, kbase + pa * page_bytes, vbase + pa * page_bytes, a.k_scales, a.v_scales,
                     (int64_t)pa * a.Hkv + g, lane);
        P::template load_page<STREAM>(r, 1, kbase + pb * page_bytes, vbase + pb * page_bytes, a.k_scales, a.v_scales,
                     (int64_t)pb * a.Hkv + g, lane);
    };
    // K takes a round trip through this wave's own LDS scratch; only the owning
    // wave touches it, so wave-level fences suffice
    auto consume = [&](typename P::Tile &r, int i) {
        u32x4 ka[P::kDim / 32], kb[P::kDim / 32];
        P::k_store(r, scratch, lane);
        wave_lds_fence();
        P::k_fetch(scratch, lane, ka, kb);
        wave_lds_fence();
        P::attend(ka, kb, r, qop, st, a.scale_log2e, t0 + (first + stride * i) * kTileTokens, t1, lane);
    };
    typename P::Tile ra, rb;
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

// Tokens of sequence b that its group shares: whole pages, never more than the
// sequence has and never more than the host-side bound.
SD_DEV int shared_tokens(const SplitArgs &a, int b)
{
    const int L = min(a.context_lens[b], a.max_context_len);
    return max(0, min(min(a.shared_len[b], a.max_shared_len), L)) & ~(kPage - 1);
}

template <int D>
SD_DEV void reset(WaveState<D> &st)
{
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int i = 0; i < D / 16; ++i) st.acc[i] = f32x4{0, 0, 0, 0};
}

// LDS of one workgroup.  Plain items: per-wave K scratch plus the merge
// buffers.  Shared-prefix items: four tile slots (K image + parked V
// registers), one filled by each wave and read by all.
template <class P>
struct Lds {
    static constexpr int kRow = P::kDim + 4;  // padded: 16 rows x float4 stores hit 64 distinct banks
    static constexpr int kSlotBytes = P::kScratchBytes + ((P::kVBytes + 15) / 16) * 16;
    static constexpr int kPlainBytes = kWaves * P::kScratchBytes + kWaves * kMaxGroup * kRow * 4 + 2 * kWaves * kMaxGroup * 4;
    static constexpr int kSharedBytes = kWaves * kSlotBytes;
    static constexpr int kBytes = kPlainBytes > kSharedBytes ? kPlainBytes : kSharedBytes;
};

// Shared-prefix item: one workgroup owns one whole chunk of a group's shared
// prefix for one KV head and up to 64 query rows: wave w owns the 16 rows of
// column block w (G heads each of 16/G consecutive sequences of the group).
// The pages are the same for every member, so the first member's table row is
// read.  Per round each wave loads a different 32-token tile from HBM (one
// round prefetched ahead), parks it in its LDS slot, and after a barrier every
// wave attends all four tiles from LDS with its own rows: each byte leaves HBM
// once per workgroup and the four-fold reuse is paid in LDS bandwidth.  Every
// wave writes the partials of its own rows; nothing is merged across waves.
template <class P>
SD_DEV void shared_item(const SplitArgs &a, char *lds, int lane, int wave)
{
    constexpr int D = P::kDim;
    constexpr int kSlot = Lds<P>::kSlotBytes;
    const unsigned item = blockIdx.x;  // (chunk, group, block of 4 column blocks, kv head), kv head fastest
    const int g = item % a.Hkv;
    const int sub = (item / a.Hkv) % a.group_subs;
    const int grp = (item / (a.Hkv * a.group_subs)) % a.num_groups;
    const int c = item / (a.Hkv * a.group_subs * a.num_groups);
    const int gs = a.group_start[grp], ge = a.group_start[grp + 1];
    const int spw = a.G <= kMaxGroup / 2 ? kMaxGroup / a.G : 1;  // sequences per column block
    if (gs + sub * kWaves * spw >= ge) return;                    // workgroup-uniform
    const int shared = shared_tokens(a, gs);
    const int t0 = c * a.chunk_tokens;
    if (t0 >= shared) return;  // workgroup-uniform
    const int t1 = min(shared, t0 + a.chunk_tokens);  // the prefix's last chunk may be short

    const int seq0 = gs + (sub * kWaves + wave) * spw;
    const bool active = seq0 < ge;  // wave-uniform; idle waves still load their tile and meet the barriers
    const int n = lane & 15;
    const int row_seq = seq0 + n / a.G;
    const int64_t row = (int64_t)row_seq * a.Hq + g * a.G + n % a.G;
    const bool row_ok = active && n / a.G < spw && row_seq < ge;
    u32x4 qop[D / 32];
#pragma unroll
    for (int s = 0; s < D / 32; ++s)
        qop[s] = row_ok ? *reinterpret_cast<const u32x4 *>(a.q + row * D + P::q_offset(s, lane)) : u32x4{0, 0, 0, 0};
    WaveState<D> st;
    reset(st);

    const int32_t *bt = a.block_table + (int64_t)gs * a.max_blocks + t0 / kPage;
    const int64_t page_bytes = (int64_t)P::kTileBytes * a.Hkv;
    const char *kbase = static_cast<const char *>(a.k_pages) + g * P::kTileBytes;
    const char *vbase = static_cast<const char *>(a.v_pages) + g * P::kTileBytes;
    auto issue = [&](typename P::Tile &r, int pa, int pb) {
        P::template load_page<true>(r, 0, kbase + pa * page_bytes, vbase + pa * page_bytes, a.k_scales, a.v_scales,
                                    (int64_t)pa * a.Hkv + g, lane);
        P::template load_page<true>(r, 1, kbase + pb * page_bytes, vbase + pb * page_bytes, a.k_scales, a.v_scales,
                                    (int64_t)pb * a.Hkv + g, lane);
    };
    const int rounds = (t1 - t0 + kWaves * kTileTokens - 1) / (kWaves * kTileTokens);
    const int last_page = (t1 - t0) / kPage - 1;  // shared lengths are whole pages
    char *mine = lds + wave * kSlot;
    typename P::Tile r;
    // round 0: this wave's tile is tile `wave`; tiles past the end re-read the last page and are skipped below
    issue(r, bt[min(2 * wave, last_page)], bt[min(2 * wave + 1, last_page)]);
    for (int rd = 0; rd < rounds; ++rd) {
        const int tn = kWaves * min(rd + 1, rounds - 1) + wave;
        const int na = bt[min(2 * tn, last_page)], nb = bt[min(2 * tn + 1, last_page)];
        P::k_store(r, mine, lane);
        P::v_store(r, mine + P::kScratchBytes, lane);
        if (rd + 1 < rounds) issue(r, na, nb);
        __syncthreads();
        if (active) {
#pragma unroll 1
            for (int j = 0; j < kWaves; ++j) {
                if (t0 + (kWaves * rd + j) * kTileTokens >= t1) break;  // wave-uniform
                const char *slot = lds + j * kSlot;
                u32x4 ka[D / 32], kb[D / 32];
                typename P::Tile t;
                P::k_fetch(slot, lane, ka, kb);
                P::v_fetch(t, slot + P::kScratchBytes, lane);
                P::attend(ka, kb, t, qop, st, a.scale_log2e, t0 + (kWaves * rd + j) * kTileTokens, t1, lane);
            }
        }
        __syncthreads();
    }
    if (!active) return;
    st.l = head_sum(st.l);
    if (row_ok) {
        const int64_t slot = row * a.S + c;
        P::store_acc(st, a.ws_acc + slot * D, lane >> 4);
        if ((lane >> 4) == 0) {
            a.ws_m[slot] = st.m;
            a.ws_l[slot] = st.l;
        }
    }
}

// Plain item: one workgroup owns one (sequence b, KV head g, chunk c).  The
// rows of the MFMA tile are the G query heads of the KV head (rows >= G idle);
// the chunk may be ragged at the sequence's end; nobody else reads these K/V
// bytes, so they stream.  The four waves take every fourth 32-token tile,
// merge through LDS and write one partial per head.
template <class P>
__global__ __launch_bounds__(kWaves * 64, 2) void split_kernel(SplitArgs a)
{
    constexpr int D = P::kDim;
    constexpr int kRow = Lds<P>::kRow;
    __shared__ __attribute__((aligned(16))) char lds[Lds<P>::kBytes];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (blockIdx.x < a.group_items) {  // shared-prefix items come first in the grid
        shared_item<P>(a, lds, lane, wave);
        return;
    }
    char *s_k = lds + wave * P::kScratchBytes;
    float (*s_acc)[kMaxGroup][kRow] = reinterpret_cast<float (*)[kMaxGroup][kRow]>(lds + kWaves * P::kScratchBytes);
    float (*s_m)[kMaxGroup] = reinterpret_cast<float (*)[kMaxGroup]>(lds + kWaves * P::kScratchBytes + kWaves * kMaxGroup * kRow * 4);
    float (*s_l)[kMaxGroup] = s_m + kWaves;

    // (chunk counted from the sequence's end, sequence, kv head), kv head fastest.  The grid
    // walks the chunks of every sequence from the front, aligned at the END: its last rows
    // hold every sequence's last chunk, which is the short one, so the workgroups that run
    // while the machine drains are the small ones.
    const unsigned item = blockIdx.x - a.group_items;
    const int g = item % a.Hkv;
    const int b = (item / a.Hkv) % a.B;
    const int from_end = a.grid_chunks - 1 - (int)(item / (a.Hkv * a.B));

    const int L = min(a.context_lens[b], a.max_context_len);
    // slots of a shared prefix belong to the shared-prefix items; the others start where the prefix ends
    const int shared = a.shared_len ? shared_tokens(a, b) : 0;
    const int n_private = (L - shared + a.chunk_tokens - 1) / a.chunk_tokens;
    const int c_private = n_private - 1 - from_end;
    if (c_private < 0) return;
    const int c = shared_slots(shared, a.chunk_tokens) + c_private;  // slot of this chunk
    const int t0 = shared + c_private * a.chunk_tokens;
    const int t1 = min(L, t0 + a.chunk_tokens);

    // Q^T operand: lane&15 = head n; heads >= G are zero rows
    const int n = lane & 15;
    u32x4 qop[D / 32];
    {
        const uint16_t *qrow = a.q + ((int64_t)b * a.Hq + (int64_t)g * a.G + n) * D;
#pragma unroll
        for (int s = 0; s < D / 32; ++s)
            qop[s] = (n < a.G) ? *reinterpret_cast<const u32x4 *>(qrow + P::q_offset(s, lane)) : u32x4{0, 0, 0, 0};
    }

    WaveState<D> st;
    reset(st);
    const int32_t *bt = a.block_table + (int64_t)b * a.max_blocks + t0 / kPage;
    stream_tiles<P, true>(a, bt, g, t0, t1, wave, kWaves, qop, st, s_k, lane);

    // the four lanes of a head hold disjoint shares of the weight sum
    st.l = head_sum(st.l);

    const int qd = lane >> 4;
    if (qd == 0) {
        s_m[wave][n] = st.m;
        s_l[wave][n] = st.l;
    }
    P::store_acc(st, &s_acc[wave][n][0], qd);
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

// Plain launches go through hipLaunchKernelGGL (capturable into HIP graphs); only
// timed launches bind begin/end events with hipExtLaunchKernelGGL.
template <class P>
static void launch_one(const SplitArgs &a, dim3 g, dim3 b, hipStream_t stream, hipEvent_t start, hipEvent_t stop)
{
    if (start || stop)
        hipExtLaunchKernelGGL(split_kernel<P>, g, b, 0, stream, start, stop, 0, a);
    else
        hipLaunchKernelGGL(split_kernel<P>, g, b, 0, stream, a);
}

hipError_t launch_split(const SplitArgs &a, int head_dim, int kv_dtype, hipStream_t stream,
                        hipEvent_t start, hipEvent_t stop)
{
    const unsigned grid = a.group_items + (unsigned)a.grid_chunks * (unsigned)a.B * (unsigned)a.Hkv;
    if (grid == 0) return hipSuccess;
    const dim3 g(grid), b(kWaves * 64);
    if (kv_dtype == 0 && head_dim == 128)
        launch_one<Bf16Path<128>>(a, g, b, stream, start, stop);
    else if (kv_dtype == 0 && head_dim == 64)
        launch_one<Bf16Path<64>>(a, g, b, stream, start, stop);
    else if (kv_dtype == 1 && head_dim == 128)
        launch_one<Fp8Path>(a, g, b, stream, start, stop);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace sd
