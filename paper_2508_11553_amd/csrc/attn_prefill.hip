// Causal attention of several query tokens per sequence over the paged cache
// (gfx950, wave64, MFMA): the re-computation of a stretch of a trajectory's own
// stored tokens when it resumes after an interruption.
//
// Sequence b brings n_b = q_start[b+1] - q_start[b] query tokens, its LAST n_b
// positions: query i sits at position pos = L - n_b + i and attends the tokens
// 0 .. pos.  A workgroup owns a block of consecutive query tokens of one
// sequence and one KV head; every wave owns 2 * (16 / G) of them as two column
// blocks of 16 rows (tokens times the G query heads of the KV head), which share
// every K operand fetched from LDS and every V^T operand.  The K/V tiles are
// the same for all waves: each is loaded from HBM/L2 once per workgroup, parked
// in LDS as the K image and the ready-made V^T operands, and attended by every
// wave with its own columns.  Each wave carries its rows through the whole
// range with the online softmax, so there is no split and no merge: the wave
// normalises and writes its rows itself.
//
// The causal limit is a per-lane token bound in the score mask; a wave stops
// once a tile starts at or past the last position any of its rows may see.
//
// Two kernels: prefill_kernel (workgroups of 4 waves, a whole tile per wave and
// round, two barriers per round; fp8 pools and head_dim 64) and
// prefill_wide_kernel (bf16 pools with head_dim 128: 8 waves, half a tile per
// wave and round, two LDS buffers, one barrier per round).
#include <type_traits>

#include "attn_tile.h"

namespace sd {

template <class P>
__global__ __launch_bounds__(kWaves * 64, 2) void prefill_kernel(PrefillArgs a)
{
    constexpr int D = P::kDim;
    constexpr int kSlot = Lds<P>::kSlotBytes;
    constexpr int NB = kPrefillBlocks;
    __shared__ __attribute__((aligned(16))) char lds[kWaves * kSlot];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Workgroup i runs on XCD i % 8, and each XCD has its own L2.  All query blocks of one
    // (sequence, kv head) read the same K/V, so they get consecutive slots of ONE XCD (query
    // block fastest, late positions = long ranges first): they run side by side, walk the
    // range at about the same pace, and all but the first find the tiles in that L2.
    const unsigned per_xcd = gridDim.x / kXcds;  // the grid is padded to a multiple of kXcds
    const unsigned item = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    const int Hv = a.Hkv * a.HB;
    if (item >= (unsigned)a.q_blocks * (unsigned)a.B * (unsigned)Hv) return;
    const int jb = a.q_blocks - 1 - (int)(item % a.q_blocks);
    const HeadBlock hb = head_block((item / a.q_blocks) % Hv, a.G, a.HB);
    const int g = hb.g;
    const int b = item / ((unsigned)a.q_blocks * Hv);
    const int tpb = units_per_block(a.G);  // query tokens per column block
    const int tpw = kPrefillBlocks * tpb;                        // and per wave

    // everything below up to the loop is workgroup-uniform
    const int qs = a.q_start[b];
    const int nq = min(a.q_start[b + 1] - qs, a.max_q_len);
    const int i0 = jb * kWaves * tpw;
    if (i0 >= nq) return;
    if (qs < 0 || (int64_t)qs + nq > a.total_q) return;  // rows outside q: nothing is read or written
    const int L = max(0, min(a.context_lens[b], a.max_context_len));
    const int base = L - nq;                                            // position of query 0 (may be negative)
    const int kv_end = max(0, base + min(nq, i0 + kWaves * tpw));       // tokens the block's last row sees

    // this wave's rows
    const int iw0 = i0 + wave * tpw;
    const int iw1 = min(iw0 + tpw, nq);
    const bool active = iw0 < nq && base + iw1 > 0;  // some row of the wave sees a token
    const int wave_max_end = base + iw1;            // its last row's limit
    const int wave_min_end = max(0, base + iw0) + 1;  // its first visible row's limit
    const int n = lane & 15;
    // row of column block c in this lane: query token, whether it exists, whether it sees a token
    // (recomputed where needed rather than kept in registers across the loop)
    auto locate = [&](int c, bool &in_range, bool &row_ok, int64_t &row) {
        const int i = iw0 + c * tpb + n / hb.rows;
        in_range = n / hb.rows < tpb && i < nq;
        row_ok = in_range && base + i >= 0;
        row = ((int64_t)qs + i) * a.Hq + hb.head0 + n % hb.rows;
        return i;
    };
    int row_end[NB];
    u32x4 qop[NB][D / 32];
    typename P::ParkedState st[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        bool in_range, row_ok;
        int64_t row;
        const int i = locate(c, in_range, row_ok, row);
        // rows that see nothing ride along with zero queries, masked only past the sequence's end
        row_end[c] = row_ok ? base + i + 1 : L;
#pragma unroll
        for (int s = 0; s < D / 32; ++s)
            qop[c][s] = row_ok ? (*reinterpret_cast<const u32x4 *>(a.q + row * D + P::q_offset(s, lane)) & a.q_keep) ^ a.q_flip
                               : u32x4{0, 0, 0, 0};
        reset(st[c]);
    }

    const int32_t *bt = a.block_table + (int64_t)b * a.max_blocks;
    const int64_t page_bytes = (int64_t)P::kTileBytes * a.Hkv;
    const char *kbase = static_cast<const char *>(a.k_pages) + g * P::kTileBytes;
    const char *vbase = static_cast<const char *>(a.v_pages) + g * P::kTileBytes;
    auto issue = [&](typename P::Tile &r, int pa, int pb) {
        P::template load_page<false>(r, 0, kbase + pa * page_bytes, vbase + pa * page_bytes, a.k_scales, a.v_scales,
                                     (int64_t)pa * a.Hkv + g, lane);
        P::template load_page<false>(r, 1, kbase + pb * page_bytes, vbase + pb * page_bytes, a.k_scales, a.v_scales,
                                     (int64_t)pb * a.Hkv + g, lane);
    };
    const int ntiles = (kv_end + kTileTokens - 1) / kTileTokens;
    const int rounds = (ntiles + kWaves - 1) / kWaves;
    const int last_page = (kv_end + kPage - 1) / kPage - 1;
    char *mine = lds + wave * kSlot;
    if (rounds > 0) {
        typename P::Tile r;
        // tiles past the end re-read the last page; nobody attends them
        issue(r, bt[min(2 * wave, last_page)], bt[min(2 * wave + 1, last_page)]);
        // page ids are read two rounds ahead of their tile: the read is waited for at this round's
        // barrier (with the LDS writes) and its result is used in the next round
        const int t1 = kWaves * min(1, rounds - 1) + wave;
        int na = bt[min(2 * t1, last_page)], nb = bt[min(2 * t1 + 1, last_page)];
        for (int rd = 0; rd < rounds; ++rd) {
            const int t2 = kWaves * min(rd + 2, rounds - 1) + wave;
            const int fa = bt[min(2 * t2, last_page)], fb = bt[min(2 * t2 + 1, last_page)];
            P::k_store(r, mine, lane);
            P::v_park(r, mine + P::kScratchBytes, lane, (kWaves * rd + wave) * kTileTokens, L);
            if (rd + 1 < rounds) issue(r, na, nb);
            na = fa;
            nb = fb;
            __syncthreads();
            if (active) {
                // the round's tiles below the diagonal of every row of the wave, then those on it
                auto step = [&](int j, auto masked) {
                    const int tok0 = (kWaves * rd + j) * kTileTokens;
                    const char *slot = lds + j * kSlot;
                    u32x4 ka[D / 32], kb[D / 32];
                    P::k_fetch(slot, lane, ka, kb);
                    P::template attend_parked<NB, decltype(masked)::value>(ka, kb, slot + P::kScratchBytes, qop, st, a.scale_log2e,
                                                                          tok0, lane, row_end);
                };
                const int t0 = kWaves * rd * kTileTokens;
                // tiles [0, j_plain) end at or before the first visible row's limit; tiles [j_plain, j_end) start before the last row's
                const int j_end = min(kWaves, (wave_max_end - t0 + kTileTokens - 1) / kTileTokens);
                const int j_plain = max(0, min(j_end, (wave_min_end - t0) / kTileTokens));
                int j = 0;
#pragma unroll 1
                for (; j < j_plain; ++j) step(j, std::false_type{});
#pragma unroll 1
                for (; j < j_end; ++j) step(j, std::true_type{});
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        const float l = P::weight_sum(st[c]);
        bool in_range, row_ok;
        int64_t row;
        locate(c, in_range, row_ok, row);
        if (!in_range) continue;
        // rows before the sequence's first token get zeros
        const float inv = row_ok ? 1.0f / l : 0.0f;
#pragma unroll
        for (int k = 0; k < D / 16; ++k) st[c].acc[k] = row_ok ? st[c].acc[k] * inv : f32x4{0, 0, 0, 0};
        P::store_acc(st[c], a.out + row * D, lane >> 4);
    }
}

// bf16 pools, head_dim 128: one workgroup of 8 waves per compute unit.  A round is four 32-token tiles, held in
// one of two LDS buffers; wave w brings page w & 1 of tile w >> 1 (half the registers of a whole
// tile), and because the next round's buffer is the one nobody reads, a wave parks what it loaded
// and asks for the page after that without waiting for anybody: one barrier per round, none
// between a write and the reads of the same round.  Twice the query tokens per workgroup also
// halve what travels from L2 to LDS per row.  The rest (rows of a wave, causal limits, tile step)
// is as above.
template <class P, int kW, int NB>
__global__ __launch_bounds__(kW * 64) void prefill_wide_kernel(PrefillArgs a)
{
    constexpr int D = P::kDim;
    constexpr int kTiles = 4;                 // tiles per round
    constexpr int kPages = 2 * kTiles / kW;   // pages a wave brings per round
    constexpr int kSlot = Lds<P>::kSlotBytes;
    constexpr int kBuf = kTiles * kSlot;
    static_assert(kW * NB == kPrefillWideWaves * kPrefillBlocks, "the host sizes the grid with this product");
    static_assert(kPages * kW == 2 * kTiles, "whole pages per wave");
    __shared__ __attribute__((aligned(16))) char lds[2 * kBuf];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned per_xcd = gridDim.x / kXcds;  // the grid is padded to a multiple of kXcds
    const unsigned item = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    const int Hv = a.Hkv * a.HB;
    if (item >= (unsigned)a.q_blocks * (unsigned)a.B * (unsigned)Hv) return;
    const int jb = a.q_blocks - 1 - (int)(item % a.q_blocks);
    const HeadBlock hb = head_block((item / a.q_blocks) % Hv, a.G, a.HB);
    const int g = hb.g;
    const int b = item / ((unsigned)a.q_blocks * Hv);
    const int tpb = units_per_block(a.G);  // query tokens per column block
    const int tpw = NB * tpb;              // and per wave

    // everything below up to the loop is workgroup-uniform
    const int qs = a.q_start[b];
    const int nq = min(a.q_start[b + 1] - qs, a.max_q_len);
    const int i0 = jb * kW * tpw;
    if (i0 >= nq) return;
    if (qs < 0 || (int64_t)qs + nq > a.total_q) return;  // rows outside q: nothing is read or written
    const int L = max(0, min(a.context_lens[b], a.max_context_len));
    const int base = L - nq;                                       // position of query 0 (may be negative)
    const int kv_end = max(0, base + min(nq, i0 + kW * tpw));      // tokens the block's last row sees

    const int iw0 = i0 + wave * tpw;
    const int iw1 = min(iw0 + tpw, nq);
    const bool active = iw0 < nq && base + iw1 > 0;  // some row of the wave sees a token
    const int wave_max_end = base + iw1;              // its last row's limit
    const int wave_min_end = max(0, base + iw0) + 1;  // its first visible row's limit
    const int n = lane & 15;
    auto locate = [&](int c, bool &in_range, bool &row_ok, int64_t &row) {
        const int i = iw0 + c * tpb + n / hb.rows;
        in_range = n / hb.rows < tpb && i < nq;
        row_ok = in_range && base + i >= 0;
        row = ((int64_t)qs + i) * a.Hq + hb.head0 + n % hb.rows;
        return i;
    };
    int row_end[NB];
    u32x4 qop[NB][D / 32];
    typename P::ParkedState st[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        bool in_range, row_ok;
        int64_t row;
        const int i = locate(c, in_range, row_ok, row);
        row_end[c] = row_ok ? base + i + 1 : L;
#pragma unroll
        for (int s = 0; s < D / 32; ++s)
            qop[c][s] = row_ok ? (*reinterpret_cast<const u32x4 *>(a.q + row * D + P::q_offset(s, lane)) & a.q_keep) ^ a.q_flip
                               : u32x4{0, 0, 0, 0};
        reset(st[c]);
    }

    const int32_t *bt = a.block_table + (int64_t)b * a.max_blocks;
    const int64_t page_bytes = (int64_t)P::kTileBytes * a.Hkv;
    const char *kbase = static_cast<const char *>(a.k_pages) + g * P::kTileBytes;
    const char *vbase = static_cast<const char *>(a.v_pages) + g * P::kTileBytes;
    typedef typename P::Page Page;
    // page i of this wave: tile and half of the round it belongs to
    auto tile_of = [&](int i) { return (wave * kPages + i) >> 1; };
    auto half_of = [&](int i) { return (wave * kPages + i) & 1; };
    auto issue = [&](Page &r, int page) {
        P::template load_one<false>(r, kbase + page * page_bytes, vbase + page * page_bytes, a.k_scales, a.v_scales,
                                    (int64_t)page * a.Hkv + g, lane);
    };
    // page i of round rd -> its half of its tile's slot in `buf`
    auto park = [&](Page &r, char *buf, int rd, int i) {
        const int my_tile = tile_of(i), my_page = half_of(i);
        P::park_one(r, buf + my_tile * kSlot, my_page, lane, (kTiles * rd + my_tile) * kTileTokens + my_page * kPage, L);
    };
    const int ntiles = (kv_end + kTileTokens - 1) / kTileTokens;
    const int rounds = (ntiles + kTiles - 1) / kTiles;
    const int last_page = (kv_end + kPage - 1) / kPage - 1;
    // page i this wave brings for round rd (pages past the end re-read the last one; nobody attends them)
    auto page_of = [&](int rd, int i) { return bt[min(2 * kTiles * min(rd, rounds - 1) + wave * kPages + i, last_page)]; };
    if (rounds > 0) {
        Page r[kPages];
        int next_page[kPages], after_next[kPages];  // read ahead of their use
#pragma unroll
        for (int i = 0; i < kPages; ++i) {
            issue(r[i], page_of(0, i));
            next_page[i] = page_of(1, i);
            after_next[i] = page_of(2, i);
        }
#pragma unroll
        for (int i = 0; i < kPages; ++i) {
            park(r[i], lds, 0, i);
            if (rounds > 1) issue(r[i], next_page[i]);
        }
        __syncthreads();
        for (int rd = 0; rd < rounds; ++rd) {
            const char *cur = lds + (rd & 1) * kBuf;
            // round rd + 1's page goes to the other buffer (last read in round rd - 1), round rd + 2's is requested
#pragma unroll
            for (int i = 0; i < kPages; ++i) {
                next_page[i] = after_next[i];
                after_next[i] = page_of(rd + 3, i);
                if (rd + 1 < rounds) {
                    park(r[i], lds + ((rd + 1) & 1) * kBuf, rd + 1, i);
                    if (rd + 2 < rounds) issue(r[i], next_page[i]);
                }
            }
            if (active) {
                auto step = [&](int j, auto masked) {
                    const int tok0 = (kTiles * rd + j) * kTileTokens;
                    const char *slot = cur + j * kSlot;
                    u32x4 ka[D / 32], kb[D / 32];
                    P::k_fetch(slot, lane, ka, kb);
                    P::template attend_parked<NB, decltype(masked)::value>(ka, kb, slot + P::kScratchBytes, qop, st, a.scale_log2e,
                                                                          tok0, lane, row_end);
                };
                const int t0 = kTiles * rd * kTileTokens;
                const int j_end = min(kTiles, (wave_max_end - t0 + kTileTokens - 1) / kTileTokens);
                const int j_plain = max(0, min(j_end, (wave_min_end - t0) / kTileTokens));
                int j = 0;
#pragma unroll 1
                for (; j < j_plain; ++j) step(j, std::false_type{});
#pragma unroll 1
                for (; j < j_end; ++j) step(j, std::true_type{});
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        const float l = P::weight_sum(st[c]);
        bool in_range, row_ok;
        int64_t row;
        locate(c, in_range, row_ok, row);
        if (!in_range) continue;
        const float inv = row_ok ? 1.0f / l : 0.0f;  // rows before the sequence's first token get zeros
#pragma unroll
        for (int k = 0; k < D / 16; ++k) st[c].acc[k] = row_ok ? st[c].acc[k] * inv : f32x4{0, 0, 0, 0};
        P::store_acc(st[c], a.out + row * D, lane >> 4);
    }
}

hipError_t launch_prefill(const PrefillArgs &a, int head_dim, int kv_dtype, hipStream_t stream, hipEvent_t start,
                          hipEvent_t stop)
{
    const unsigned items = (unsigned)a.q_blocks * (unsigned)a.B * (unsigned)(a.Hkv * a.HB);
    if (items == 0) return hipSuccess;
    const unsigned grid = (items + kXcds - 1) / kXcds * kXcds;
    const dim3 g(grid), b(prefill_waves(kv_dtype, head_dim) * 64);
    auto go = [&](auto kernel) {
        if (start || stop)
            hipExtLaunchKernelGGL(kernel, g, b, 0, stream, start, stop, 0, a);
        else
            hipLaunchKernelGGL(kernel, g, b, 0, stream, a);
    };
    if (kv_dtype == 0 && head_dim == 128)
        go(prefill_wide_kernel<Bf16Path<128>, kPrefillWideWaves, kPrefillBlocks>);
    else if (kv_dtype == 0 && head_dim == 64)
        go(prefill_kernel<Bf16Path<64>>);
    else if (kv_dtype == 1 && head_dim == 128)
        go(prefill_kernel<Fp8Path>);
    else if (kv_dtype == 1 && head_dim == 64)
        go(prefill_kernel<Fp8Path64>);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace sd
