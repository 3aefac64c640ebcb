// Range pass of paged decode attention for gfx950 (wave64, MFMA): the decode
// step balanced over the machine whatever the mix of sequence lengths.
//
// Per (virtual) KV head the batch is laid out as one line of 32-token tiles,
// sequence after sequence (sequence b contributes ceil(L_b / 32) tiles).  The
// line is cut into `ranges` equal pieces and every wave of the grid walks one
// piece of one head, so all waves stream the same number of K/V bytes, start
// together and end together: no chunk size to choose and no tail in which a
// few long workgroups keep the machine waiting.  The grid is sized to the
// machine (two workgroups of four waves per compute unit), not to the batch.
//
// A wave's piece is a run of segments; a segment is the part of one sequence
// that lies inside the piece.  The wave carries the G query heads of its KV
// head through a segment with the online softmax (tile step: attn_tile.h) and
// then
//   - the segment is the whole sequence: normalises and writes `out` itself;
//   - otherwise: leaves (max, sum, weighted sum) in a partial slot.  A piece has
//     at most two such segments, its first and its last, so two slots per wave
//     suffice.
// The four waves of a workgroup walk neighbouring pieces; parts of one sequence
// that lie in neighbouring pieces of one workgroup are first added up through
// LDS (see handed_over), so a sequence leaves at most one part per workgroup.
// range_merge_kernel then combines the partials of every sequence that is still
// cut, in range order, and writes those rows of `out`; it finds the cuts from
// the tile offsets the range pass leaves in the workspace.
//
// Where the pieces fall depends on the lengths only (never on page placement),
// which keeps results independent of the physical layout.
//
// The same kernel with PROBE = true issues exactly the same loads and does no
// arithmetic on them beyond an XOR fold: its duration is what the memory system
// delivers for this walk.
#include "attn_tile.h"

namespace sd {

constexpr int kSeqsPerThread = kMaxRangeBatch / (kWaves * 64);

// LDS scratch of one wave: the K image of a tile, or a whole partial ([16][D] floats, then the rows'
// maxima and weight sums) on its way out or on its way to a neighbouring wave
template <class P>
constexpr int wave_lds_bytes()
{
    return (P::kScratchBytes > kMaxGroup * P::kDim * 4 ? P::kScratchBytes : kMaxGroup * P::kDim * 4) + 2 * kMaxGroup * 4;
}

// Slot of the partial that range r holds for a sequence whose tiles start at line position o0:
// the first segment of a range uses slot 0, a later one (it starts inside the range) slot 1.
SD_DEV int64_t partial_slot(int r, int gv, int Hv, int o0, int per)
{
    return ((int64_t)r * Hv + gv) * 2 + (o0 > r * per ? 1 : 0);
}

// Combines the partials that the ranges of `parts` hold for the `rows` query heads of one
// (sequence, head block) and writes columns [col0, col0 + DW) of the rows of `out` starting at
// row0.  One wave: the 64 lanes share the rows out (a row goes to 64 / R2 neighbouring lanes, R2 the
// power of two >= rows, each lane a run of DW * R2 / 64 >= 4 floats) and PB partials are fetched at
// a time, all loads in flight together, so up to PB partials cost one trip to memory.  Partials
// are folded in range order with a running maximum.
template <int PB, int NL_MAX>
SD_DEV void combine_parts(const RangeMergeArgs &a, const LiveParts &parts, int gv, int Hv, int o0, int per,
                          int rows, int64_t row0, int D, int col0, int DW, int lane)
{
    const int R2 = rows > 8 ? 16 : rows > 4 ? 8 : rows > 2 ? 4 : rows > 1 ? 2 : 1;
    const int lpr = min(64 / R2, DW / 4);   // lanes per row
    const int F = DW / lpr;                 // floats per lane
    const int NL = F / 4;                   // 16-byte loads per lane and partial (<= NL_MAX)
    const int mr = lane / lpr, c = lane - mr * lpr;
    if (mr >= rows) return;
    float M = -INFINITY, den = 0.f;
    f32x4 num[NL_MAX];
#pragma unroll
    for (int j = 0; j < NL_MAX; ++j) num[j] = f32x4{0, 0, 0, 0};
    for (int base = 0; base < parts.count; base += PB) {
        float m[PB], l[PB];
        f32x4 v[PB][NL_MAX];
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            const bool valid = base + p < parts.count;   // wave-uniform
            const int64_t ps = partial_slot(parts.range(valid ? base + p : 0), gv, Hv, o0, per);
            m[p] = valid ? a.ws_m[ps * kMaxGroup + mr] : -INFINITY;
            l[p] = valid ? a.ws_l[ps * kMaxGroup + mr] : 0.f;
            const f32x4 *src = reinterpret_cast<const f32x4 *>(a.ws_acc + (ps * a.rows_stride + mr) * D + col0 + c * F);
#pragma unroll
            for (int j = 0; j < NL_MAX; ++j) v[p][j] = valid && j < NL ? src[j] : f32x4{0, 0, 0, 0};
        }
        float Mn = M;
#pragma unroll
        for (int p = 0; p < PB; ++p) Mn = fmaxf(Mn, m[p]);
        const float shrink = __builtin_amdgcn_exp2f(M - Mn);  // first batch: exp2(-inf) = 0 on zeros
        M = Mn;
        den *= shrink;
#pragma unroll
        for (int j = 0; j < NL_MAX; ++j) num[j] *= shrink;
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            const float w = __builtin_amdgcn_exp2f(m[p] - M);
            den += w * l[p];
#pragma unroll
            for (int j = 0; j < NL_MAX; ++j) num[j] += w * v[p][j];
        }
    }
    float *dst = a.out + (row0 + mr) * D + col0 + c * F;
#pragma unroll
    for (int j = 0; j < NL_MAX; ++j)
        if (j < NL) *reinterpret_cast<f32x4 *>(dst + 4 * j) = num[j] / den;
}

// Two waves per SIMD, also for the probe, whose few registers would otherwise let the dispatcher
// pack the grid onto a part of the machine.
template <class P, bool PROBE>
__global__ __launch_bounds__(kWaves * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void range_kernel(RangeArgs a)
{
    constexpr int D = P::kDim;
    // per-wave K scratch, then the tile offsets of the B sequences (B + 1 words)
    extern __shared__ __attribute__((aligned(16))) char lds[];
    __shared__ int wave_total[kWaves];
    int *tile_off = reinterpret_cast<int *>(lds + kWaves * wave_lds_bytes<P>());

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int Hv = a.Hkv * a.HB;
    // head fastest over the grid: neighbouring workgroups (they run on different dies) walk the same
    // pages at the same pace, each reading its own head's tiles of them; where the heads share lines
    // (fp8 scales) one die takes all heads of a range block instead
    const unsigned item = P::kDealByDie ? xcd_deal(blockIdx.x, gridDim.x, Hv) : blockIdx.x;
    const int gv = item % Hv;
    const int rblock = item / Hv;
    const HeadBlock hb = head_block(gv, a.G, a.HB);

    // the newest token of every sequence comes as a row of k_new / v_new and goes into the pool from here
    const int fused = P::kAppendInPlace && !PROBE && a.k_new != nullptr;

    // ---- tile offsets: exclusive prefix sums of ceil(L_b / 32), by the whole workgroup
    int nt[kSeqsPerThread];
    int local = 0;
    const int per_thread = (a.B + kWaves * 64 - 1) / (kWaves * 64);
#pragma unroll
    for (int i = 0; i < kSeqsPerThread; ++i) {
        const int b = tid * per_thread + i;
        nt[i] = 0;
        if (i < per_thread && b < a.B)   // the pool's tokens: with an append in flight the newest one is not among them
            nt[i] = (max(0, min(a.context_lens[b], a.max_context_len) - fused) + kTileTokens - 1) / kTileTokens;
        local += nt[i];
    }
    int incl = local;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(incl, off, 64);
        if (lane >= off) incl += v;
    }
    if (lane == 63) wave_total[wave] = incl;
    __syncthreads();
    int run = incl - local;
    int T = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave) run += wave_total[w];
        T += wave_total[w];
    }
#pragma unroll
    for (int i = 0; i < kSeqsPerThread; ++i) {
        const int b = tid * per_thread + i;
        if (i < per_thread && b < a.B) tile_off[b] = run;
        run += nt[i];
    }
    if (tid == 0) tile_off[a.B] = T;
    __syncthreads();
    // the merge pass finds the cuts from these offsets
    if (!PROBE && blockIdx.x == 0)
        for (int i = tid; i <= a.B; i += kWaves * 64) a.tile_off[i] = tile_off[i];

    // ---- sequences without tiles; the workgroups of this head share them out.  Empty ones owe zero
    // rows; with an append in flight a sequence of one token is just that token: its V row is the
    // result, and the row still has to go into the pool.
    if (!PROBE) {
        const int nrb = gridDim.x / Hv;
        for (int b = rblock; b < a.B; b += nrb)
            if (tile_off[b + 1] == tile_off[b]) {
                const bool one = fused && min(a.context_lens[b], a.max_context_len) == 1;
                const uint16_t *vrow = one ? a.v_new + ((int64_t)b * a.Hkv + hb.g) * D : nullptr;
                for (int idx = tid; idx < hb.rows * D; idx += kWaves * 64)
                    a.out[((int64_t)b * a.Hq + hb.head0) * D + idx] =
                        one ? __builtin_bit_cast(float, (unsigned)vrow[idx % D] << 16) : 0.f;
                if (one && gv % a.HB == 0 && tid < D) {
                    const int64_t at = ((int64_t)a.block_table[(int64_t)b * a.max_blocks] * a.Hkv + hb.g) * (kPage * D) + tid;
                    a.k_pages_out[at] = a.k_new[((int64_t)b * a.Hkv + hb.g) * D + tid];
                    a.v_pages_out[at] = vrow[tid];
                }
            }
    }
    // no workgroup barrier below this line: from here on every wave is on its own

    // ---- this wave's piece of the line
    const int per = max((T + a.ranges - 1) / a.ranges, a.min_tiles);
    const int r = rblock * kWaves + wave;
    const int g0 = r * per;
    const int g1 = min(T, g0 + per);
    const bool has = g0 < g1;   // a wave past the end of the line only takes part in the hand-over's barrier
    if (PROBE && !has) return;
    int b_first = 0;
    if (has) {   // the sequence that holds tile g0: the last b with tile_off[b] <= g0
        int lo = 0, hi = a.B;  // tile_off[hi] = T > g0
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (__builtin_amdgcn_readfirstlane(tile_off[mid]) > g0) hi = mid; else lo = mid + 1;
        }
        b_first = lo - 1;
    }
    char *s_k = lds + wave * wave_lds_bytes<P>();
    const int n = lane & 15;

    // A segment: the tiles [lt0, lt1) of sequence b that lie in this wave's piece (all wave-uniform).
    struct Segment {
        int b, lt0, lt1, L, o0, o1;
        const int32_t *row;   // the sequence's block-table row
    };
    auto open_segment = [&](int b) {
        Segment sg;
        sg.b = b;
        sg.o0 = __builtin_amdgcn_readfirstlane(tile_off[b]);
        sg.o1 = __builtin_amdgcn_readfirstlane(tile_off[b + 1]);
        sg.lt0 = max(g0, sg.o0) - sg.o0;
        sg.lt1 = min(g1, sg.o1) - sg.o0;
        sg.L = max(0, min(a.context_lens[b], a.max_context_len) - fused);   // tokens in the pool
        sg.row = a.block_table + (int64_t)b * a.max_blocks;
        return sg;
    };
    u32x4 fold = {0, 0, 0, 0};
    u32x4 qop[D / 32];
    typename P::State st;
    // a finished segment: the whole sequence -> `out`; a part of one -> this wave's partial slot
    // (l: the rows' weight sums; the four lanes of a head hold disjoint shares of st.l)
    auto finish = [&](const auto &sg, float l, int lane) {
        const int n = lane & 15, qd = lane >> 4;
        if (sg.lt0 == 0 && sg.lt1 == sg.o1 - sg.o0) {
            if (n < hb.rows) {
#pragma unroll
                for (int k = 0; k < D / 16; ++k) st.acc[k] = st.acc[k] / l;
                P::store_acc(st, a.out + ((int64_t)sg.b * a.Hq + hb.head0 + n) * D, qd);
            }
            return;
        }
        // The partial goes out as whole lines: the rows pass through this wave's LDS scratch and leave
        // as the contiguous [rows][D] image, 16 bytes per lane and 1 KB per store instruction.
        const int64_t slot = partial_slot(r, gv, Hv, sg.o0, per);
        P::store_acc(st, reinterpret_cast<float *>(s_k) + n * D, qd);
        wave_lds_fence();
        char *dst = reinterpret_cast<char *>(a.ws_acc + slot * a.rows_stride * D);
        const int image_bytes = __builtin_amdgcn_readfirstlane(hb.rows * D * 4);
#pragma unroll
        for (int j = 0; j < kMaxGroup * D * 4 / 1024; ++j)
            if (j * 1024 + lane * 16 < image_bytes)
                *reinterpret_cast<u32x4 *>(dst + j * 1024 + lane * 16) = *reinterpret_cast<const u32x4 *>(s_k + j * 1024 + lane * 16);
        wave_lds_fence();
        if (lane < hb.rows) {   // lane n < 16 holds row n's max and weight sum (qd == 0)
            a.ws_m[slot * kMaxGroup + lane] = st.m;
            a.ws_l[slot * kMaxGroup + lane] = l;
        }
    };

    struct { int b, lt0, lt1, o0, o1; } last = {0, 0, 0, 0, 0};   // the piece's last segment is finished after the loop
    bool open = false;                                            // ... if there is one
    for (int b = b_first; has && b < a.B; ++b) {
        if (__builtin_amdgcn_readfirstlane(tile_off[b]) >= g1) break;
        if (__builtin_amdgcn_readfirstlane(tile_off[b + 1]) == __builtin_amdgcn_readfirstlane(tile_off[b])) continue;
        const Segment sg = open_segment(b);
        const int t0 = sg.lt0 * kTileTokens, t1 = min(sg.L, sg.lt1 * kTileTokens);
        const int32_t *bt = sg.row + t0 / kPage;
        if (PROBE) {
            probe_tiles<P>(a, bt, hb.g, t0, t1, fold, lane);
            continue;
        }
        // Q^T operand: lane&15 = head n of the block; rows past the block's heads are zero
        const int64_t row = (int64_t)b * a.Hq + hb.head0 + n;
#pragma unroll
        for (int s = 0; s < D / 32; ++s)
            qop[s] = n < hb.rows ? *reinterpret_cast<const u32x4 *>(a.q + row * D + P::q_offset(s, lane)) : u32x4{0, 0, 0, 0};
        reset(st);
        // the segment that ends its sequence also takes the newest token, which is not in the pool yet.  Its
        // rows are fetched after the walk (eight registers less to carry through it); four lanes touch their
        // lines now, so that the fetch finds them in the cache
        const bool newest = fused && sg.lt1 == sg.o1 - sg.o0;   // wave-uniform
        const int64_t new_at = ((int64_t)b * a.Hkv + hb.g) * D;
        unsigned touched = 0;
        if (newest && lane < 4 && (lane & 1) * 64 < D)
            touched = *reinterpret_cast<const unsigned *>((lane < 2 ? a.k_new : a.v_new) + new_at + (lane & 1) * 64);
        stream_tiles<P, true>(a, bt, hb.g, t0, t1, 0, 1, qop, st, s_k, lane);
        // What follows the walk forms its addresses from this copy of the lane number, i.e. here and not
        // ahead of the walk, where they would only occupy registers.  (Not volatile and no memory clobber:
        // either would make the block-table reads of the next segment vector loads; the dependence on the
        // walk's result keeps it in place.)
        int lane_after = lane;
        asm("" : "+v"(lane_after) : "v"(touched), "v"(st.m));
        if (newest) {
            const typename P::NewRow nr = P::load_new_row(a.k_new + new_at, a.v_new + new_at, lane_after);
            typename P::Tile t;
            P::new_row_tile(t, nr);
            u32x4 ka[D / 32], kb[D / 32];
            P::k_store(t, s_k, lane);
            wave_lds_fence();
            P::k_fetch(s_k, lane, ka, kb);
            wave_lds_fence();
            P::attend(ka, kb, t, qop, st, a.scale_log2e, sg.L, sg.L + 1, lane);   // one token, at position L - 1 of the sequence
            if (gv % a.HB == 0) {   // one of the head blocks of this KV head puts the rows into the pool
                const int64_t at = ((int64_t)sg.row[sg.L / kPage] * a.Hkv + hb.g) * (kPage * D) + (sg.L % kPage) * D;
                P::store_new_row(nr, a.k_pages_out + at, a.v_pages_out + at, lane_after);
            }
        }
        if (sg.o0 + sg.lt1 == g1) {
            last = {sg.b, sg.lt0, sg.lt1, sg.o0, sg.o1};
            open = true;
            break;
        }
        finish(sg, head_sum(st.l), lane_after);
    }
    if (PROBE) {
        unsigned f = fold[0] ^ fold[1] ^ fold[2] ^ fold[3];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) f ^= __shfl_xor(f, off, 64);
        if (lane == 0) a.sink[(int64_t)r * Hv + gv] = f;
        return;
    }
    // ---- hand-over inside the workgroup (see handed_over), then the last segment's result leaves.
    // (The lane number passes through an empty asm so that the addresses below are formed here and not
    // ahead of the walk, where they would only occupy registers.)
    __shared__ int s_link[kWaves][2];   // lt0 (< 0: the wave has no tiles) and lt1 of each wave's last segment
    int lane_now;   // the lane number once more, produced here so that nothing has to be kept for it
    asm("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_now) : "v"(open ? st.m : 0.f));
    const int n_now = lane_now & 15, qd_now = lane_now >> 4;
    float *image = reinterpret_cast<float *>(s_k);
    float l = open ? head_sum(st.l) : 0.f;
    const bool hands_over = open && wave > 0 && last.lt0 > 0;
    if (lane_now == 0) {
        s_link[wave][0] = open ? last.lt0 : -1;
        s_link[wave][1] = last.lt1;
    }
    if (hands_over) {
        P::store_acc(st, image + n_now * D, qd_now);
        if (qd_now == 0) {
            image[kMaxGroup * D + n_now] = st.m;
            image[kMaxGroup * D + kMaxGroup + n_now] = l;
        }
    }
    __syncthreads();
    if (open && !hands_over) {
        for (int w = wave + 1; w < kWaves && __builtin_amdgcn_readfirstlane(s_link[w][0]) > 0; ++w) {   // in range order
            const float *theirs = reinterpret_cast<const float *>(lds + w * wave_lds_bytes<P>());
            const float m2 = theirs[kMaxGroup * D + n_now], l2 = theirs[kMaxGroup * D + kMaxGroup + n_now];
            const float m_new = fmaxf(st.m, m2);
            const float c1 = __builtin_amdgcn_exp2f(st.m - m_new), c2 = __builtin_amdgcn_exp2f(m2 - m_new);
            f32x4 acc2[D / 16];
            P::load_acc(acc2, theirs + n_now * D, qd_now);
#pragma unroll
            for (int k = 0; k < D / 16; ++k) st.acc[k] = st.acc[k] * c1 + acc2[k] * c2;
            l = l * c1 + l2 * c2;
            st.m = m_new;
            last.lt1 = __builtin_amdgcn_readfirstlane(s_link[w][1]);
        }
        finish(last, l, lane_now);
    }
    // Which sequence the merge pass combines on behalf of this range: the one whose FIRST part lies here and
    // that does not end here.  Only a piece's last segment can be that (an earlier one that starts inside the
    // piece also ends inside it).
    const bool first_part = open && !hands_over && last.lt0 == 0 && last.lt1 < last.o1 - last.o0;
    if (lane_now == 0)
        a.merge_rec[(int64_t)r * Hv + gv] = first_part ? int4{last.b, last.o0, last.o1, T} : int4{-1, 0, 0, 0};
}

// Merge pass of the range design.  A sequence that one range held whole was written by the wave
// that walked it; a sequence that was cut is combined here.  One workgroup of two waves (each takes
// half of the columns) per item; an item is a (sequence, head block) when the batch has fewer
// sequences than the grid has ranges, else a (range, head block): the range pass leaves, per range,
// a record of the cut sequence whose first part lies there (at most one).
template <int D>
__global__ __launch_bounds__(128) void range_merge_kernel(RangeMergeArgs a)
{
    const int Hv = a.Hkv * a.HB;
    const int lane = threadIdx.x & 63, half = threadIdx.x >> 6;
    const int gv = blockIdx.x % Hv;
    int b, o0, o1, T;
    if (a.by_sequence) {
        b = blockIdx.x / Hv;
        o0 = a.tile_off[b], o1 = a.tile_off[b + 1], T = a.tile_off[a.B];
        if (o1 == o0) return;
    } else {
        const int4 rec = a.merge_rec[blockIdx.x];
        b = rec.x, o0 = rec.y, o1 = rec.z, T = rec.w;
        if (b < 0) return;
    }
    const int per = max((T + a.ranges - 1) / a.ranges, a.min_tiles);
    // parts that were handed over inside a workgroup are in their neighbour's; a sequence with a single part
    // left was written by the wave that held it
    const LiveParts parts = live_parts(o0, o1, T, per);
    if (parts.count == 1) return;
    const HeadBlock hb = head_block(gv, a.G, a.HB);
    const int64_t row0 = (int64_t)b * a.Hq + hb.head0;
    if (hb.rows > kMaxGroup / 2)
        combine_parts<8, D / 32>(a, parts, gv, Hv, o0, per, hb.rows, row0, D, half * (D / 2), D / 2, lane);
    else
        combine_parts<16, (D / 64 > 0 ? D / 64 : 1)>(a, parts, gv, Hv, o0, per, hb.rows, row0, D, half * (D / 2), D / 2, lane);
}

hipError_t launch_range_merge(const RangeMergeArgs &a, int head_dim, hipStream_t stream, hipEvent_t start, hipEvent_t stop)
{
    const unsigned grid = (unsigned)(a.by_sequence ? a.B : a.ranges) * (unsigned)(a.Hkv * a.HB);
    if (grid == 0 || a.B == 0) return hipSuccess;
    auto go = [&](auto kernel) {
        if (start || stop)
            hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(128), 0, stream, start, stop, 0, a);
        else
            hipLaunchKernelGGL(kernel, dim3(grid), dim3(128), 0, stream, a);
    };
    if (head_dim == 128)
        go(range_merge_kernel<128>);
    else if (head_dim == 64)
        go(range_merge_kernel<64>);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

template <class P, bool PROBE>
static void launch_range_one(const RangeArgs &a, unsigned grid, hipStream_t stream, hipEvent_t start, hipEvent_t stop)
{
    const size_t lds = (size_t)kWaves * wave_lds_bytes<P>() + ((size_t)a.B + 1) * 4;
    if (start || stop)
        hipExtLaunchKernelGGL((range_kernel<P, PROBE>), dim3(grid), dim3(kWaves * 64), lds, stream, start, stop, 0, a);
    else
        hipLaunchKernelGGL((range_kernel<P, PROBE>), dim3(grid), dim3(kWaves * 64), lds, stream, a);
}

hipError_t launch_range(const RangeArgs &a, int head_dim, int kv_dtype, unsigned grid, bool probe, hipStream_t stream,
                        hipEvent_t start, hipEvent_t stop)
{
    if (grid == 0 || a.B == 0) return hipSuccess;
    if (a.B > kMaxRangeBatch) return hipErrorNotSupported;
    if (kv_dtype == 0 && head_dim == 128)
        probe ? launch_range_one<Bf16Path<128>, true>(a, grid, stream, start, stop)
              : launch_range_one<Bf16Path<128>, false>(a, grid, stream, start, stop);
    else if (kv_dtype == 0 && head_dim == 64)
        probe ? launch_range_one<Bf16Path<64>, true>(a, grid, stream, start, stop)
              : launch_range_one<Bf16Path<64>, false>(a, grid, stream, start, stop);
    else if (kv_dtype == 1 && head_dim == 128)
        probe ? launch_range_one<Fp8Path, true>(a, grid, stream, start, stop)
              : launch_range_one<Fp8Path, false>(a, grid, stream, start, stop);
    else if (kv_dtype == 1 && head_dim == 64)
        probe ? launch_range_one<Fp8Path64, true>(a, grid, stream, start, stop)
              : launch_range_one<Fp8Path64, false>(a, grid, stream, start, stop);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace sd
