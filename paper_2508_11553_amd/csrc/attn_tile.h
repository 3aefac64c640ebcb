// Tile-level building blocks shared by the attention kernels of libseamdecode
// (gfx950, wave64): MFMA wrappers, the online softmax of one 32-token tile, and
// the two storage paths (bf16 pools, fp8 e4m3fn pools) with their loads, LDS
// layouts and operand formation.
//
// Every kernel computes the transposed products of one 32-token tile,
//   S^T[token][row] = K[token][d] . Q^T[d][row]        mfma 16x16x32 bf16
//   O^T[d][row]    += V^T[d][token] . P^T[token][row]   mfma 16x16x32 bf16
// so that the accumulator layout of the first (lane = row, registers = tokens)
// is the B-operand layout of the second and the weights never leave their
// lanes.  A "row" is one query row: a query head in the decode pass, a (query
// token, head) pair in the causal pass.  There are two ways to run the step:
//
//   attend         the wave owns the tile: K operands from its LDS scratch, V^T
//                  operands formed in registers from the V rows it loaded
//   attend_parked  the tile sits in an LDS slot that several waves consume: the
//                  loading wave has parked the K image (k_store) and the
//                  ready-made V^T operands (v_park); NB column blocks of 16 rows
//                  share every operand read
#pragma once
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
// displacing each other (STREAM = true).  Bytes that other workgroups will ask
// for again soon (the causal pass) take ordinary loads.
template <bool STREAM, typename T>
SD_DEV T kv_load(const T *p)
{
    if (STREAM) return __builtin_nontemporal_load(p);
    return *p;
}

// What a decode or prefill kernel only reads and nothing running beside it writes (the block table,
// the fp8 scales) is read through the constant address space: that pins wave-uniform reads to scalar
// loads whatever else the kernel stores.  As vector loads they would queue behind the tile loads,
// and every wait for a page id or a scale would drain the tiles in flight.
typedef const __attribute__((address_space(4))) int32_t *ConstTable;
typedef const __attribute__((address_space(4))) float *ConstScales;

// The larger of two scores.  Scores are never NaN (a masked one is -inf), so the
// NaN-propagating maximum is the same value as fmaxf, and it is one v_maximum3_f32
// for up to three operands, where fmaxf first re-quiets every operand the compiler
// cannot prove canonical (an MFMA result, a permuted lane): a second instruction each.
SD_DEV float max_of(float a, float b) { return __builtin_elementwise_maximum(a, b); }
SD_DEV float max_of(float a, float b, float c) { return max_of(max_of(a, b), c); }

// Reductions over the four lanes {n, n+16, n+32, n+48} that share a row.
// v_permlane16_swap exchanges rows 1<->0' and 3<->2' of its two operands and
// v_permlane32_swap the upper half of one with the lower half of the other;
// fed the same value twice they return (x, x from the partner row/half).
// (The two results are copied out of the pair before they are reinterpreted: a bit cast applied
// directly to an element of the pair reads element 0 whichever element is named.)
SD_DEV float head_max(float x)
{
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned a0 = a[0], a1 = a[1];
    const float y = max_of(__builtin_bit_cast(float, a0), __builtin_bit_cast(float, a1));
    const unsigned w = __builtin_bit_cast(unsigned, y);
    const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
    const unsigned b0 = b[0], b1 = b[1];
    return max_of(__builtin_bit_cast(float, b0), __builtin_bit_cast(float, b1));
}
SD_DEV float head_sum(float x)
{
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned a0 = a[0], a1 = a[1];
    const float y = __builtin_bit_cast(float, a0) + __builtin_bit_cast(float, a1);
    const unsigned w = __builtin_bit_cast(unsigned, y);
    const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
    const unsigned b0 = b[0], b1 = b[1];
    return __builtin_bit_cast(float, b0) + __builtin_bit_cast(float, b1);
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

template <int D, int EXTRA = 0>
struct WaveState {
    static constexpr int kAcc = D / 16 + EXTRA;
    float m;             // running max of this lane's row, log2 domain (same in the 4 lanes of a row)
    float l;             // this lane's share of the weight sum
    f32x4 acc[kAcc];     // O^T accumulators; which d each one holds is the path's business
                         // (EXTRA = 1: one more that accumulates the weights themselves)
};

template <class State>
SD_DEV void reset(State &st)
{
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int i = 0; i < State::kAcc; ++i) st.acc[i] = f32x4{0, 0, 0, 0};
}

// Positional mask of one tile's scores.  x holds, for row lane&15, the scores
// of tokens tok0 + 4qd + e (e < 4, first page) and tok0 + 16 + 4qd + e - 4
// (second page).  Tokens >= row_end (this lane's row: the end of the sequence
// for a decode query, position + 1 for a causal one) become -inf: by position,
// never by content.
SD_DEV void mask_scores(float (&x)[8], int tok0, int row_end, int qd)
{
    const int visible = row_end - tok0 - 4 * qd;  // of this lane's tokens, counted from its first
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (e >= visible) x[e] = -INFINITY;
        if (16 + e >= visible) x[4 + e] = -INFINITY;
    }
}

SD_DEV float max8(const float (&x)[8])
{
    return max_of(max_of(x[0], x[1], x[2]), max_of(x[3], x[4], x[5]), max_of(x[6], x[7]));
}

// In the causal pass the reference m of a row's exponents may lag the row's largest score so far:
// weights above 1 lose nothing in fp32 or as bf16 (same relative rounding), and weight sum and
// weighted sum are relative to m whatever it is.  The row-wide maximum, a chain of a dozen
// dependent instructions with two lane exchanges, is taken there only when some lane's score has
// outgrown the reference: by kSlack over fp8 pools (checked before the weights are formed); over
// bf16 pools when a weight reaches 2 (seen from the weights themselves, see
// Bf16Path::attend_parked), the reference then moving to kLead above the row's maximum.  The
// decode kernels, which wait for memory, keep the exact maximum: a lagging reference made no
// difference to them.
constexpr float kSlack = 8.0f;  // log2 domain
constexpr float kLead = 7.0f;   // log2 domain: where a moved reference is put relative to the row's maximum (bf16 pools)

// The running max goes m_old -> m_new: everything accumulated so far shrinks by
// alpha = exp2(m_old - m_new).  When no row of the wave moved (the usual case once
// a few tiles are in) alpha is 1 in every lane, and neither the exponential nor the
// products are issued.
template <class State>
SD_DEV void advance_max(State &st, float m_new)
{
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(m_new != st.m) != 0, 0)) {
        const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
        st.l *= alpha;
#pragma unroll
        for (int i = 0; i < State::kAcc; ++i) st.acc[i] *= alpha;
        st.m = m_new;
    }
}

// Scaled scores x (log2 domain) of one tile -> weights p = exp2(x - m), with the
// running max and the accumulators brought up to date.
template <class State>
SD_DEV void online_softmax(const float (&x)[8], float (&p)[8], State &st)
{
    advance_max(st, max_of(st.m, head_max(max8(x))));
#pragma unroll
    for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(x[e] - st.m);
}

// The same with a reference that may lag the row's maximum by up to kSlack.
template <class State>
SD_DEV void online_softmax_lagging(const float (&x)[8], float (&p)[8], State &st)
{
    const float hi = max8(x);
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(hi > st.m + kSlack) != 0, 0)) advance_max(st, max_of(st.m, head_max(hi)));
#pragma unroll
    for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(x[e] - st.m);
}

// The same for raw scores and a positive scale c (log2 domain) folded into the
// exponent: p = exp2(s * c - m), one fused multiply-add per score; the max runs
// over the raw scores.
template <class State>
SD_DEV void online_softmax_folded(const float (&s)[8], float c, float (&p)[8], State &st)
{
    advance_max(st, max_of(st.m, head_max(max8(s)) * c));
#pragma unroll
    for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], c, -st.m));
}

// ---------------------------------------------------------------------------
// bf16 pools
// ---------------------------------------------------------------------------
template <int D>
struct Bf16Path {
    static constexpr int kDim = D;
    static constexpr int kTileBytes = kPage * D * 2;      // one (page, head) tile
    static constexpr int kScratchBytes = 2 * kTileBytes;  // K of one 32-token tile in LDS
    static constexpr int kOpsBytes = (D / 16) * 1024;     // the V^T operands of one tile in LDS
    static constexpr int kPieces = D / 8;                 // 16-byte pieces per K row
    static constexpr int kRowsPerLoad = 64 / kPieces;     // K rows one 1024-byte load covers
    typedef WaveState<D> State;
    typedef WaveState<D, 1> ParkedState;  // acc[D/16] sums the rounded weights through the MFMA

    struct Tile {
        u32x4 k[2][D / 32];     // [page][j]: 16 bytes at byte offset 1024*j + 16*lane of the K tile
        u32x2 v[2][D / 64][4];  // [page][half][j]: V row 4*(lane>>4)+j, d = 64*half + 4*(lane&15) .. +4
    };

    // Q^T operand of step s: row lane&15, d = 32*s + 8*(lane>>4) .. +8
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

    // One page of a tile on its own: the causal pass with 8 waves brings its tiles page by page.
    struct Page {
        u32x4 k[D / 32];     // as Tile, one page
        u32x2 v[D / 64][4];
    };
    template <bool STREAM>
    SD_DEV static void load_one(Page &r, const char *kp, const char *vp, const float *, const float *, int64_t, int lane)
    {
        const char *kl = kp + lane * 16;
#pragma unroll
        for (int j = 0; j < D / 32; ++j) r.k[j] = kv_load<STREAM>(reinterpret_cast<const u32x4 *>(kl + j * 1024));
        const char *vl = vp + (lane >> 4) * 4 * (D * 2) + (lane & 15) * 8;
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
#pragma unroll
            for (int j = 0; j < 4; ++j) r.v[h][j] = kv_load<STREAM>(reinterpret_cast<const u32x2 *>(vl + j * (D * 2) + h * 128));
    }
    // Page `half` (tokens tok0 .. tok0 + 15, those < t_end exist) of the tile parked in `slot`: its half
    // of the K image (as k_store) and of every V^T operand (as v_park: words 2 * half and 2 * half + 1).
    SD_DEV static void park_one(Page &r, char *slot, int half, int lane, int tok0, int t_end)
    {
        char *kdst = slot + half * kTileBytes;
#pragma unroll
        for (int j = 0; j < D / 32; ++j) {
            const int row = j * kRowsPerLoad + lane / kPieces;
            const int piece = (lane % kPieces) ^ (row % kPieces);
            *reinterpret_cast<u32x4 *>(kdst + row * (D * 2) + piece * 16) = r.k[j];
        }
        if (tok0 + kPage > t_end) {  // wave-uniform: V rows of tokens that do not exist may hold anything
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (tok0 + 4 * (lane >> 4) + j >= t_end) {
#pragma unroll
                    for (int h = 0; h < D / 64; ++h) r.v[h][j] = u32x2{0, 0};
                }
        }
        char *vdst = slot + kScratchBytes + lane * 16 + half * 8;
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int w = i >> 1;
                const u32x2 o = (i & 1) ? u32x2{pack_hi(r.v[h][0][w], r.v[h][1][w]), pack_hi(r.v[h][2][w], r.v[h][3][w])}
                                        : u32x2{pack_lo(r.v[h][0][w], r.v[h][1][w]), pack_lo(r.v[h][2][w], r.v[h][3][w])};
                *reinterpret_cast<u32x2 *>(vdst + (4 * h + i) * 1024) = o;
            }
    }

    // The newest token of a sequence handed over as rows instead of pool bytes (the decode step that
    // appends and attends in one go): row pieces in the lanes that would hold token 0 of a tile.
    static constexpr bool kAppendInPlace = true;
    static constexpr bool kDealByDie = false;   // the heads of a sequence share no lines worth keeping together
    struct NewRow {
        u32x4 k;            // lanes < kPieces: 16 bytes of the K row
        u32x2 v[D / 64];    // lanes < 16: V row, d = 64*half + 4*lane .. +4
    };
    SD_DEV static NewRow load_new_row(const uint16_t *k_row, const uint16_t *v_row, int lane)
    {
        NewRow x;
        x.k = lane < kPieces ? *reinterpret_cast<const u32x4 *>(k_row + lane * 8) : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
            x.v[h] = lane < 16 ? *reinterpret_cast<const u32x2 *>(v_row + 64 * h + 4 * lane) : u32x2{0, 0};
        return x;
    }
    SD_DEV static void store_new_row(const NewRow &x, uint16_t *k_row, uint16_t *v_row, int lane)
    {
        if (lane < kPieces) *reinterpret_cast<u32x4 *>(k_row + lane * 8) = x.k;
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
            if (lane < 16) *reinterpret_cast<u32x2 *>(v_row + 64 * h + 4 * lane) = x.v[h];
    }
    // a tile whose token 0 is the new row and whose other 31 tokens are zeros (masked by position anyway)
    SD_DEV static void new_row_tile(Tile &r, const NewRow &x)
    {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
#pragma unroll
            for (int j = 0; j < D / 32; ++j) r.k[pg][j] = u32x4{0, 0, 0, 0};
#pragma unroll
            for (int h = 0; h < D / 64; ++h)
#pragma unroll
                for (int j = 0; j < 4; ++j) r.v[pg][h][j] = u32x2{0, 0};
        }
        r.k[0][0] = x.k;
#pragma unroll
        for (int h = 0; h < D / 64; ++h) r.v[0][h][0] = x.v[h];
    }

    // XOR of everything a tile's loads brought in (read probe)
    SD_DEV static u32x4 fold(const Tile &r)
    {
        u32x4 f = {0, 0, 0, 0};
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
#pragma unroll
            for (int j = 0; j < D / 32; ++j) f ^= r.k[pg][j];
#pragma unroll
            for (int h = 0; h < D / 64; ++h)
#pragma unroll
                for (int j = 0; j < 4; ++j) f ^= u32x4{r.v[pg][h][j][0], r.v[pg][h][j][1], 0, 0};
        }
        return f;
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

    // V rows of tokens that do not exist (>= t_end) may hold anything, NaN
    // included; they are zeroed so that weight 0 times them is 0.
    SD_DEV static void v_sanitise(Tile &r, int tok0, int t_end, int qd)
    {
        if (tok0 + kTileTokens <= t_end) return;  // wave-uniform
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (tok0 + 16 * pg + 4 * qd + j >= t_end) {
#pragma unroll
                    for (int h = 0; h < D / 64; ++h) r.v[pg][h][j] = u32x2{0, 0};
                }
    }

    // V^T operand k = 4h + i of the second product, formed inside the lane with
    // byte permutes: it feeds acc[k][r] = O[row lane&15][d = 64h + 16qd + 4r + i].
    SD_DEV static u32x4 v_operand(const Tile &r, int h, int i)
    {
        const auto &v = r.v;
        const int w = i >> 1;
        if (i & 1)
            return u32x4{pack_hi(v[0][h][0][w], v[0][h][1][w]), pack_hi(v[0][h][2][w], v[0][h][3][w]),
                         pack_hi(v[1][h][0][w], v[1][h][1][w]), pack_hi(v[1][h][2][w], v[1][h][3][w])};
        return u32x4{pack_lo(v[0][h][0][w], v[0][h][1][w]), pack_lo(v[0][h][2][w], v[0][h][3][w]),
                     pack_lo(v[1][h][0][w], v[1][h][1][w]), pack_lo(v[1][h][2][w], v[1][h][3][w])};
    }

    // Scores, online softmax and weighted V sum of one 32-token tile (tokens
    // tok0 .. tok0+31, those < t_end exist) for the wave that loaded it.
    SD_DEV static void attend(const u32x4 (&ka)[D / 32], const u32x4 (&kb)[D / 32], Tile &r,
                              const u32x4 (&qop)[D / 32], State &st, float scale_log2e, int tok0, int t_end, int lane)
    {
        const int qd = lane >> 4;
        f32x4 sa = {0, 0, 0, 0}, sb = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < D / 32; ++s) {
            sa = mfma_bf16_k32(ka[s], qop[s], sa);
            sb = mfma_bf16_k32(kb[s], qop[s], sb);
        }
        float x[8], p[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = sa[e] * scale_log2e;
            x[4 + e] = sb[e] * scale_log2e;
        }
        if (tok0 + kTileTokens > t_end) mask_scores(x, tok0, t_end, qd);  // wave-uniform
        online_softmax(x, p, st);
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
        v_sanitise(r, tok0, t_end, qd);
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) st.acc[4 * h + i] = mfma_bf16_k32(v_operand(r, h, i), pop, st.acc[4 * h + i]);
    }

    // The loading wave's half of a shared tile: the V^T operands, one 16-byte
    // piece per lane and operand, ready for attend_parked.
    SD_DEV static void v_park(Tile &r, char *vslot, int lane, int tok0, int t_end)
    {
        v_sanitise(r, tok0, t_end, lane >> 4);
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *reinterpret_cast<u32x4 *>(vslot + (4 * h + i) * 1024 + lane * 16) = v_operand(r, h, i);
    }

    // The tile step for NB column blocks of 16 rows over a parked tile.  The row
    // of block b in this lane ends at row_end[b]; MASK says some row may end
    // inside the tile, and `tile_has_end` (wave-uniform) whether one does.  c = |scale| * log2(e) > 0 is folded into the
    // exponent.  The weight sum is one more accumulator fed an all-ones operand,
    // i.e. the sum of the rounded weights exactly.
    //
    // Order of issue.  A wave issues in program order, and a matrix instruction
    // holds the matrix pipe for 16 cycles of which its issue takes 4.  With several
    // blocks and no mask (the tiles below the diagonal: nearly all) the vector
    // arithmetic of block b's softmax is therefore written between the matrix
    // instructions of the group after it (the first product of block b + 1, or the
    // second product of block 0 after the last block), a few vector instructions per
    // matrix instruction, so that both pipes work at once within one wave.  Tiles
    // with a mask take the plain order (products, softmax, products).
    template <int NB, bool MASK>
    SD_DEV static void attend_parked(const u32x4 (&ka)[D / 32], const u32x4 (&kb)[D / 32], const char *vslot,
                                     const u32x4 (&qop)[NB][D / 32], ParkedState (&st)[NB], float c, int tok0,
                                     int lane, const int (&row_end)[NB], bool tile_has_end = true)
    {
        constexpr int S = D / 32, K = D / 16;
        constexpr bool kBeside = NB > 1 && !MASK;
        const int qd = lane >> 4;
        const u32x4 ones = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};  // bf16 1.0 pairs
        f32x4 sa[NB], sb[NB];
        u32x4 va[K], pop[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) sa[b] = sb[b] = f32x4{0, 0, 0, 0};
        auto first_product = [&](int b, int s) {
            sa[b] = mfma_bf16_k32(ka[s], qop[b][s], sa[b]);
            sb[b] = mfma_bf16_k32(kb[s], qop[b][s], sb[b]);
        };
        // step k of block b's second product; step K feeds the weight sum
        auto second_product = [&](int b, int k) {
            st[b].acc[k] = mfma_bf16_k32(k == K ? ones : va[k], pop[b], st[b].acc[k]);
        };
        // matrix instructions [i0, i1) of the group that runs beside block b's softmax
        auto beside = [&](int b, int i0, int i1) {
            if (!kBeside) return;
#pragma unroll
            for (int i = i0; i < i1; ++i) {
                if (b + 1 < NB) {
                    if (i < S) first_product(b + 1, i);
                } else {
                    if (i <= K) second_product(0, i == 0 ? K : i - 1);
                }
            }
        };
        constexpr int kBesideAll = K + 1;  // covers either kind of group
        auto fetch_v = [&]() {
#pragma unroll
            for (int k = 0; k < K; ++k) va[k] = *reinterpret_cast<const u32x4 *>(vslot + k * 1024 + lane * 16);
        };
#pragma unroll
        for (int b = 0; b < (kBeside ? 1 : NB); ++b)
#pragma unroll
            for (int s = 0; s < S; ++s) first_product(b, s);
        // plain order: the V^T operands are requested before the softmax arithmetic so that the LDS
        // latency passes behind it.  Beside-order: once the K operands are no longer needed (their
        // registers are reused), which still leaves a softmax between the request and the first use.
        if (!kBeside) fetch_v();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float x[8], p[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[e] = sa[b][e];
                x[4 + e] = sb[b][e];
            }
            if (MASK && tile_has_end) mask_scores(x, tok0, row_end[b], qd);
            auto weights = [&]() {
#pragma unroll
                for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[e], c, -st[b].m));
#pragma unroll
                for (int e = 0; e < 8; e += 2) pop[b][e >> 1] = cvt_pk_bf16(p[e], p[e + 1]);
            };
            if (kBeside) {
                // The weights are formed against the reference as it stands, beside the matrix
                // instructions of the next group; only then is it asked whether the reference has
                // fallen an octave or more behind (some weight >= 2: bit 14 of its bf16 pattern; inf and
                // NaN, which a reference of -inf gives, have it too).  If so the reference moves to the
                // row's maximum and the block's weights are formed again.
                beside(b, 0, kBesideAll);
                weights();
#pragma unroll
                for (int i = 0; i < K + 1; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one matrix instruction
                    __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);  // three vector instructions
                }
                const unsigned big = (pop[b][0] | pop[b][1] | pop[b][2] | pop[b][3]) & 0x40004000u;
                if (__builtin_expect(__builtin_amdgcn_ballot_w64(big != 0) != 0, 0)) {
                    // kLead above the row's maximum: its weights are then at most 2^-kLead (nothing is lost:
                    // bf16 has fp32's exponent range), and the row's scores can grow by kLead + 1 octaves
                    // before the reference has to move again
                    advance_max(st[b], max_of(st[b].m, head_max(max8(x)) * c + kLead));
                    weights();
                }
                if (b == NB - 2) {
                    __builtin_amdgcn_sched_barrier(0);
                    fetch_v();
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                advance_max(st[b], max_of(st[b].m, head_max(max8(x)) * c));
                weights();
            }
        }
        if (kBeside) {
            // what ran beside nothing: the second product of every block but the first
#pragma unroll
            for (int b = 1; b < NB; ++b)
#pragma unroll
                for (int k = 0; k <= K; ++k) second_product(b, k == 0 ? K : k - 1);
        } else {
#pragma unroll
            for (int b = 0; b < NB; ++b) second_product(b, K);
#pragma unroll
            for (int k = 0; k < K; ++k)
#pragma unroll
                for (int b = 0; b < NB; ++b) second_product(b, k);
        }
    }
    SD_DEV static float weight_sum(const ParkedState &st) { return st.acc[D / 16][0]; }

    // this lane's accumulators -> row `dst` ([D] floats)
    template <class S>
    SD_DEV static void store_acc(const S &st, float *dst, int qd)
    {
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const f32x4 o = {st.acc[4 * h][r], st.acc[4 * h + 1][r], st.acc[4 * h + 2][r], st.acc[4 * h + 3][r]};
                *reinterpret_cast<f32x4 *>(dst + 64 * h + 16 * qd + 4 * r) = o;
            }
    }
    // the inverse: row `src` as this lane's accumulators would hold it
    SD_DEV static void load_acc(f32x4 (&acc)[D / 16], const float *src, int qd)
    {
#pragma unroll
        for (int h = 0; h < D / 64; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const f32x4 o = *reinterpret_cast<const f32x4 *>(src + 64 * h + 16 * qd + 4 * r);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[4 * h + i][r] = o[i];
            }
    }
};

// ---------------------------------------------------------------------------
// fp8 e4m3fn pools, head_dim 128: rows of 128 bytes, tiles of 2 KB.  The codes
// are converted to bf16 in registers, which is exact; the K scale multiplies a
// page's scores and the V scale its weights.
// ---------------------------------------------------------------------------
struct Fp8Path {
    static constexpr int D = 128;
    static constexpr int kDim = D;
    static constexpr int kTileBytes = kPage * D;
    static constexpr int kScratchBytes = 2 * kTileBytes;
    static constexpr int kOpsBytes = 8 * 1024 + 16;  // eight bf16 V^T operands and the four page scales
    typedef WaveState<D> State;
    typedef WaveState<D> ParkedState;

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
        r.ks[pg] = ((ConstScales)ks)[si];
        r.vs[pg] = ((ConstScales)vs)[si];
    }

    // fp8 pools take new tokens through kv_append_fp8 (a page's scale may have to change)
    static constexpr bool kAppendInPlace = false;
    static constexpr bool kDealByDie = true;    // the scales of a page's heads lie in one line: one die takes all heads of a sequence
    struct NewRow {};
    SD_DEV static NewRow load_new_row(const uint16_t *, const uint16_t *, int) { return NewRow{}; }
    SD_DEV static void store_new_row(const NewRow &, uint16_t *, uint16_t *, int) {}
    SD_DEV static void new_row_tile(Tile &, const NewRow &) {}

    SD_DEV static u32x4 fold(const Tile &r)
    {
        u32x4 f = r.k[0][0] ^ r.k[0][1] ^ r.k[1][0] ^ r.k[1][1];
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f[0] ^= r.v[pg][j][0];
                f[1] ^= r.v[pg][j][1];
            }
        f[2] ^= __builtin_bit_cast(unsigned, r.ks[0]) ^ __builtin_bit_cast(unsigned, r.ks[1]);
        f[3] ^= __builtin_bit_cast(unsigned, r.vs[0]) ^ __builtin_bit_cast(unsigned, r.vs[1]);
        return f;
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

    SD_DEV static void v_sanitise(Tile &r, int tok0, int t_end, int qd)
    {
        if (tok0 + kTileTokens <= t_end) return;  // wave-uniform
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (tok0 + 16 * pg + 4 * qd + j >= t_end) r.v[pg][j] = u32x2{0, 0};
    }

    // The eight V^T operands, handed to `use(k, operand)`; operand k feeds
    // acc[k][r] = O[row lane&15][d = 8*(4qd + r) + k].  Codes k, k+1 of four tokens
    // at a time: converting to f32 and packing two tokens' values per register is
    // the transposition.
    template <class F>
    SD_DEV static void v_operands(const Tile &r, F use)
    {
        const auto &v = r.v;
#pragma unroll
        for (int w = 0; w < 2; ++w)
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
                for (int ii = 0; ii < 2; ++ii)
                    use(4 * w + 2 * hi + ii,
                        u32x4{cvt_pk_bf16(f[0][0][ii], f[0][1][ii]), cvt_pk_bf16(f[0][2][ii], f[0][3][ii]),
                              cvt_pk_bf16(f[1][0][ii], f[1][1][ii]), cvt_pk_bf16(f[1][2][ii], f[1][3][ii])});
            }
    }

    // Weights of one block -> P^T operand and weight sum.  The operand carries the page's V scale:
    // w = bf16(p * v_scale) multiplies the raw codes.  The sum runs over the weights the product
    // really uses, w / v_scale, so that the result is an exact convex combination of the dequantised
    // values (a page whose scale is 0 holds zeros only; its weights count unrounded).
    SD_DEV static u32x4 weight_operand(const float (&p)[8], float va, float vb, float &l)
    {
        const u32x4 w = {cvt_pk_bf16(p[0] * va, p[1] * va), cvt_pk_bf16(p[2] * va, p[3] * va),
                         cvt_pk_bf16(p[4] * vb, p[5] * vb), cvt_pk_bf16(p[6] * vb, p[7] * vb)};
        auto pair_sum = [](unsigned x) { return __builtin_bit_cast(float, x << 16) + __builtin_bit_cast(float, x & 0xffff0000u); };
        const float sa = pair_sum(w[0]) + pair_sum(w[1]), sb = pair_sum(w[2]) + pair_sum(w[3]);
        l += va != 0.f ? sa * __builtin_amdgcn_rcpf(va) : (p[0] + p[1]) + (p[2] + p[3]);
        l += vb != 0.f ? sb * __builtin_amdgcn_rcpf(vb) : (p[4] + p[5]) + (p[6] + p[7]);
        return w;
    }

    SD_DEV static void attend(const u32x4 (&ka)[4], const u32x4 (&kb)[4], Tile &r, const u32x4 (&qop)[4], State &st,
                              float scale_log2e, int tok0, int t_end, int lane)
    {
        const int qd = lane >> 4;
        f32x4 sa = {0, 0, 0, 0}, sb = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            sa = mfma_bf16_k32(ka[s], qop[s], sa);
            sb = mfma_bf16_k32(kb[s], qop[s], sb);
        }
        const float ca = scale_log2e * r.ks[0], cb = scale_log2e * r.ks[1];
        float x[8], p[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = sa[e] * ca;
            x[4 + e] = sb[e] * cb;
        }
        if (tok0 + kTileTokens > t_end) mask_scores(x, tok0, t_end, qd);  // wave-uniform
        online_softmax(x, p, st);
        const u32x4 pop = weight_operand(p, r.vs[0], r.vs[1], st.l);
        v_sanitise(r, tok0, t_end, qd);
        v_operands(r, [&](int k, u32x4 a) { st.acc[k] = mfma_bf16_k32(a, pop, st.acc[k]); });
    }

    SD_DEV static void v_park(Tile &r, char *vslot, int lane, int tok0, int t_end)
    {
        v_sanitise(r, tok0, t_end, lane >> 4);
        v_operands(r, [&](int k, u32x4 a) { *reinterpret_cast<u32x4 *>(vslot + k * 1024 + lane * 16) = a; });
        if (lane == 0) *reinterpret_cast<f32x4 *>(vslot + 8 * 1024) = f32x4{r.ks[0], r.ks[1], r.vs[0], r.vs[1]};
    }

    // as Bf16Path::attend_parked; the scores are scaled per page before the mask
    // (a page of zeros has scale 0), so nothing is folded here
    template <int NB, bool MASK>
    SD_DEV static void attend_parked(const u32x4 (&ka)[4], const u32x4 (&kb)[4], const char *vslot,
                                     const u32x4 (&qop)[NB][4], ParkedState (&st)[NB], float c, int tok0, int lane,
                                     const int (&row_end)[NB], bool tile_has_end = true)
    {
        const int qd = lane >> 4;
        const f32x4 sc = *reinterpret_cast<const f32x4 *>(vslot + 8 * 1024);  // k scales, v scales of the two pages
        f32x4 sa[NB], sb[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) sa[b] = sb[b] = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                sa[b] = mfma_bf16_k32(ka[s], qop[b][s], sa[b]);
                sb[b] = mfma_bf16_k32(kb[s], qop[b][s], sb[b]);
            }
        const float ca = c * sc[0], cb = c * sc[1];
        u32x4 pop[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float x[8], p[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[e] = sa[b][e] * ca;
                x[4 + e] = sb[b][e] * cb;
            }
            if (MASK && tile_has_end) mask_scores(x, tok0, row_end[b], qd);
            if (MASK)
                online_softmax(x, p, st[b]);
            else
                online_softmax_lagging(x, p, st[b]);
            pop[b] = weight_operand(p, sc[2], sc[3], st[b].l);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const u32x4 a = *reinterpret_cast<const u32x4 *>(vslot + k * 1024 + lane * 16);
#pragma unroll
            for (int b = 0; b < NB; ++b) st[b].acc[k] = mfma_bf16_k32(a, pop[b], st[b].acc[k]);
        }
    }
    SD_DEV static float weight_sum(const ParkedState &st) { return head_sum(st.l); }

    template <class S>
    SD_DEV static void store_acc(const S &st, float *dst, int qd)
    {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const f32x4 lo = {st.acc[0][r], st.acc[1][r], st.acc[2][r], st.acc[3][r]};
            const f32x4 hi = {st.acc[4][r], st.acc[5][r], st.acc[6][r], st.acc[7][r]};
            *reinterpret_cast<f32x4 *>(dst + 32 * qd + 8 * r) = lo;
            *reinterpret_cast<f32x4 *>(dst + 32 * qd + 8 * r + 4) = hi;
        }
    }
    SD_DEV static void load_acc(f32x4 (&acc)[8], const float *src, int qd)
    {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const f32x4 lo = *reinterpret_cast<const f32x4 *>(src + 32 * qd + 8 * r);
            const f32x4 hi = *reinterpret_cast<const f32x4 *>(src + 32 * qd + 8 * r + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[i][r] = lo[i];
                acc[4 + i][r] = hi[i];
            }
        }
    }
};

// ---------------------------------------------------------------------------
// fp8 e4m3fn pools, head_dim 64: rows of 64 bytes, tiles of 1 KB.  The codes
// are converted (exactly) into the register and LDS images the bf16 path of
// head_dim 64 works with, and that path's operand code does the rest; the page
// scales enter as in the 128-wide fp8 path (K scale on the scores, V scale on
// the weights, weight sum over the rounded weights divided by the scale).
// ---------------------------------------------------------------------------
struct Fp8Path64 {
    typedef Bf16Path<64> B;
    static constexpr int D = 64;
    static constexpr int kDim = D;
    static constexpr int kTileBytes = kPage * D;             // one (page, head) tile of codes
    static constexpr int kScratchBytes = B::kScratchBytes;   // K of one 32-token tile in LDS, as bf16
    static constexpr int kOpsBytes = B::kOpsBytes + 16;      // four bf16 V^T operands and the four page scales
    typedef WaveState<D> State;
    typedef WaveState<D> ParkedState;

    struct Tile {
        u32x4 k[2];        // [page]: 16 codes at byte offset 16*lane of the K tile: row lane>>2, d = 16*(lane&3) .. +16
        unsigned v[2][4];  // [page][j]: V row 4*(lane>>4)+j, d = 4*(lane&15) .. +4
        float ks[2], vs[2];
    };

    SD_DEV static int q_offset(int s, int lane) { return B::q_offset(s, lane); }

    template <bool STREAM>
    SD_DEV static void load_page(Tile &r, int pg, const char *kp, const char *vp, const float *ks, const float *vs, int64_t si, int lane)
    {
        r.k[pg] = kv_load<STREAM>(reinterpret_cast<const u32x4 *>(kp + lane * 16));
        const char *vl = vp + (lane >> 4) * 4 * D + (lane & 15) * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) r.v[pg][j] = kv_load<STREAM>(reinterpret_cast<const unsigned *>(vl + j * D));
        r.ks[pg] = ((ConstScales)ks)[si];
        r.vs[pg] = ((ConstScales)vs)[si];
    }

    static constexpr bool kAppendInPlace = false;
    static constexpr bool kDealByDie = true;
    struct NewRow {};
    SD_DEV static NewRow load_new_row(const uint16_t *, const uint16_t *, int) { return NewRow{}; }
    SD_DEV static void store_new_row(const NewRow &, uint16_t *, uint16_t *, int) {}
    SD_DEV static void new_row_tile(Tile &, const NewRow &) {}

    SD_DEV static u32x4 fold(const Tile &r)
    {
        u32x4 f = r.k[0] ^ r.k[1];
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int j = 0; j < 4; ++j) f[j] ^= r.v[pg][j];
        f[2] ^= __builtin_bit_cast(unsigned, r.ks[0]) ^ __builtin_bit_cast(unsigned, r.ks[1]);
        f[3] ^= __builtin_bit_cast(unsigned, r.vs[0]) ^ __builtin_bit_cast(unsigned, r.vs[1]);
        return f;
    }

    // four codes -> four bf16
    SD_DEV static u32x2 cvt4(unsigned w) { return u32x2{cvt_pk_bf16_fp8<false>(w), cvt_pk_bf16_fp8<true>(w)}; }

    // The lane's 16 codes are two 16-byte pieces of the bf16 row; they go where the bf16 path's k_store
    // would have put them, so that its k_fetch reads them back.
    SD_DEV static void k_store(const Tile &r, char *kslot, int lane)
    {
        const int row = lane >> 2;
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const u32x2 lo = cvt4(r.k[pg][2 * hh]), hi = cvt4(r.k[pg][2 * hh + 1]);
                const int piece = (2 * (lane & 3) + hh) ^ (row % B::kPieces);
                *reinterpret_cast<u32x4 *>(kslot + pg * B::kTileBytes + row * (D * 2) + piece * 16) = u32x4{lo[0], lo[1], hi[0], hi[1]};
            }
    }
    SD_DEV static void k_fetch(const char *kslot, int lane, u32x4 (&ka)[2], u32x4 (&kb)[2]) { B::k_fetch(kslot, lane, ka, kb); }

    // the V registers of the bf16 path (its K registers are not used)
    SD_DEV static void v_to_bf16(const Tile &r, typename B::Tile &t)
    {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int j = 0; j < 4; ++j) t.v[pg][0][j] = cvt4(r.v[pg][j]);
    }

    SD_DEV static void attend(const u32x4 (&ka)[2], const u32x4 (&kb)[2], Tile &r, const u32x4 (&qop)[2], State &st,
                              float scale_log2e, int tok0, int t_end, int lane)
    {
        const int qd = lane >> 4;
        f32x4 sa = {0, 0, 0, 0}, sb = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            sa = mfma_bf16_k32(ka[s], qop[s], sa);
            sb = mfma_bf16_k32(kb[s], qop[s], sb);
        }
        const float ca = scale_log2e * r.ks[0], cb = scale_log2e * r.ks[1];
        float x[8], p[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = sa[e] * ca;
            x[4 + e] = sb[e] * cb;
        }
        if (tok0 + kTileTokens > t_end) mask_scores(x, tok0, t_end, qd);  // wave-uniform
        online_softmax(x, p, st);
        const u32x4 pop = Fp8Path::weight_operand(p, r.vs[0], r.vs[1], st.l);
        typename B::Tile t;
        v_to_bf16(r, t);
        B::v_sanitise(t, tok0, t_end, qd);
#pragma unroll
        for (int i = 0; i < 4; ++i) st.acc[i] = mfma_bf16_k32(B::v_operand(t, 0, i), pop, st.acc[i]);
    }

    SD_DEV static void v_park(Tile &r, char *vslot, int lane, int tok0, int t_end)
    {
        typename B::Tile t;
        v_to_bf16(r, t);
        B::v_park(t, vslot, lane, tok0, t_end);
        if (lane == 0) *reinterpret_cast<f32x4 *>(vslot + B::kOpsBytes) = f32x4{r.ks[0], r.ks[1], r.vs[0], r.vs[1]};
    }

    // as Fp8Path::attend_parked, with the four operands of head_dim 64
    template <int NB, bool MASK>
    SD_DEV static void attend_parked(const u32x4 (&ka)[2], const u32x4 (&kb)[2], const char *vslot,
                                     const u32x4 (&qop)[NB][2], ParkedState (&st)[NB], float c, int tok0, int lane,
                                     const int (&row_end)[NB], bool tile_has_end = true)
    {
        const int qd = lane >> 4;
        const f32x4 sc = *reinterpret_cast<const f32x4 *>(vslot + B::kOpsBytes);  // k scales, v scales of the two pages
        f32x4 sa[NB], sb[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) sa[b] = sb[b] = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                sa[b] = mfma_bf16_k32(ka[s], qop[b][s], sa[b]);
                sb[b] = mfma_bf16_k32(kb[s], qop[b][s], sb[b]);
            }
        const float ca = c * sc[0], cb = c * sc[1];
        u32x4 pop[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float x[8], p[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[e] = sa[b][e] * ca;
                x[4 + e] = sb[b][e] * cb;
            }
            if (MASK && tile_has_end) mask_scores(x, tok0, row_end[b], qd);
            if (MASK)
                online_softmax(x, p, st[b]);
            else
                online_softmax_lagging(x, p, st[b]);
            pop[b] = Fp8Path::weight_operand(p, sc[2], sc[3], st[b].l);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const u32x4 a = *reinterpret_cast<const u32x4 *>(vslot + k * 1024 + lane * 16);
#pragma unroll
            for (int b = 0; b < NB; ++b) st[b].acc[k] = mfma_bf16_k32(a, pop[b], st[b].acc[k]);
        }
    }
    SD_DEV static float weight_sum(const ParkedState &st) { return head_sum(st.l); }

    template <class S>
    SD_DEV static void store_acc(const S &st, float *dst, int qd) { B::store_acc(st, dst, qd); }
    SD_DEV static void load_acc(f32x4 (&acc)[4], const float *src, int qd) { B::load_acc(acc, src, qd); }
};

// LDS of one workgroup of the split pass.  Plain items: per-wave K scratch plus
// the merge buffers.  Shared items (and the causal pass): four tile slots (K
// image + V^T operands), one filled by each wave and read by all.
template <class P>
struct Lds {
    static constexpr int kRow = P::kDim + 4;  // padded: 16 rows x float4 stores hit 64 distinct banks
    static constexpr int kSlotBytes = P::kScratchBytes + ((P::kOpsBytes + 15) / 16) * 16;
    static constexpr int kPlainBytes = kWaves * P::kScratchBytes + kWaves * kMaxGroup * kRow * 4 + 2 * kWaves * kMaxGroup * 4;
    static constexpr int kSharedBytes = kWaves * kSlotBytes;
    static constexpr int kBytes = kPlainBytes > kSharedBytes ? kPlainBytes : kSharedBytes;
};

// Walks the tiles first, first+stride, ... of the token range [t0, t1) of one
// sequence: loads for tile i+1 are issued before tile i is handed to
// `consume(tile, i)`, and the page ids of tile i+2 are fetched (scalar loads)
// one step earlier still.  Everything inside the loop is unconditional so that
// the wait counters stay exact; a tile's missing second page re-reads the first
// (its tokens are masked by position).  `bt` points at the table entry of the
// range's first page; t0 is a multiple of 32.  `a` supplies k_pages, v_pages,
// k_scales, v_scales and Hkv.
template <class P, bool STREAM, class Args, class Consume>
SD_DEV void walk_tiles(const Args &a, const int32_t *bt, int g, int t0, int t1, int first, int stride, int lane,
                       Consume consume)
{
    const int ntiles = (t1 - t0 + kTileTokens - 1) / kTileTokens;
    const int nt = ntiles > first ? (ntiles - first + stride - 1) / stride : 0;
    if (nt <= 0) return;
    const int last_page = (t1 - t0 + kPage - 1) / kPage - 1;
    const int64_t page_bytes = (int64_t)P::kTileBytes * a.Hkv;
    const char *kbase = static_cast<const char *>(a.k_pages) + g * P::kTileBytes;
    const char *vbase = static_cast<const char *>(a.v_pages) + g * P::kTileBytes;
    const ConstTable btc = (ConstTable)bt;
    auto page_ids = [&](int i, int &pa, int &pb) {
        const int ti = first + stride * min(i, nt - 1);
        pa = btc[2 * ti];
        pb = btc[min(2 * ti + 1, last_page)];
    };
    auto issue = [&](typename P::Tile &r, int pa, int pb) {
        P::template load_page<STREAM>(r, 0, kbase + pa * page_bytes, vbase + pa * page_bytes, a.k_scales, a.v_scales,
                     (int64_t)pa * a.Hkv + g, lane);
        P::template load_page<STREAM>(r, 1, kbase + pb * page_bytes, vbase + pb * page_bytes, a.k_scales, a.v_scales,
                     (int64_t)pb * a.Hkv + g, lane);
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

// The attention walk: every tile goes through the wave's own tile step.  K takes
// a round trip through this wave's LDS scratch; only the owning wave touches it,
// so wave-level fences suffice.
template <class P, bool STREAM, class Args>
SD_DEV void stream_tiles(const Args &a, const int32_t *bt, int g, int t0, int t1, int first, int stride,
                         const u32x4 (&qop)[P::kDim / 32], typename P::State &st, char *scratch, int lane)
{
    walk_tiles<P, STREAM>(a, bt, g, t0, t1, first, stride, lane, [&](typename P::Tile &r, int i) {
        u32x4 ka[P::kDim / 32], kb[P::kDim / 32];
        P::k_store(r, scratch, lane);
        wave_lds_fence();
        P::k_fetch(scratch, lane, ka, kb);
        wave_lds_fence();
        const int tok0 = t0 + (first + stride * i) * kTileTokens;
        P::attend(ka, kb, r, qop, st, a.scale_log2e, tok0, t1, lane);
    });
}

// The same walk with the same loads and no arithmetic beyond an XOR fold of what arrived.
template <class P, class Args>
SD_DEV void probe_tiles(const Args &a, const int32_t *bt, int g, int t0, int t1, u32x4 &fold, int lane)
{
    walk_tiles<P, true>(a, bt, g, t0, t1, 0, 1, lane, [&](typename P::Tile &r, int) { fold ^= P::fold(r); });
}

}  // namespace sd
