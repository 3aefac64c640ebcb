// Internal declarations shared by the host entry points and the kernels of
// libseamdecode.  Not installed; the public interface is include/seamdecode.h.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace sd {

constexpr int kPage = 16;           // tokens per page
constexpr int kWaves = 4;           // waves per workgroup of the split pass
constexpr int kTileTokens = 32;     // tokens one wave consumes per iteration (two pages)
constexpr int kMaxGroup = 16;       // query heads per KV head that fit one MFMA tile
constexpr int kMaxHeadBlocks = 4;   // a KV head with more query heads is served as up to 4 blocks of 16

// A KV head with G > 16 query heads is split into HB = ceil(G / 16) "virtual" KV heads that read the
// same K/V tiles: virtual head gv = g * HB + hb owns the query heads g * G + 16 * hb .. (16 of them, the
// last block G - 16 * (HB - 1)).  With G <= 16 there is one block and gv == g.
struct HeadBlock {
    int g;       // KV head (addresses the pools)
    int head0;   // first query head of the block
    int rows;    // query heads in the block (<= 16)
};
__host__ __device__ inline int head_blocks(int G) { return (G + kMaxGroup - 1) / kMaxGroup; }
__host__ __device__ inline HeadBlock head_block(int gv, int G, int HB)
{
    const int g = gv / HB, hb = gv - g * HB;
    const int left = G - hb * kMaxGroup;
    return HeadBlock{g, g * G + hb * kMaxGroup, left < kMaxGroup ? left : kMaxGroup};
}
// Sequences (decode) or query tokens (causal pass) that share one 16-row column block.
__host__ __device__ inline int units_per_block(int G) { return G <= kMaxGroup / 2 ? kMaxGroup / G : 1; }
constexpr int kXcds = 8;            // accelerator dies, each with its own L2; workgroup i runs on die i % 8
// Deal of a grid's items to the dies.  Items i and i + 1 differ in the head (head fastest, `Hv` of
// them) and would run on different dies; lines that the heads of one sequence have in common (the
// scales of a page's heads lie in one line, so do its block-table entries) would then be fetched
// once per die.  Within every run of 8 * Hv items this hands the Hv items of one sequence to one
// die, one after the other; a ragged last run stays as it is.  A bijection of [0, n).
__device__ inline unsigned xcd_deal(unsigned i, unsigned n, unsigned Hv)
{
    const unsigned run = kXcds * Hv;
    const unsigned k = i / run, j = i - k * run;
    if ((k + 1) * run > n) return i;
    return k * run + (j % kXcds) * Hv + j / kXcds;
}
constexpr int kPrefillBlocks = 2;   // 16-row column blocks one wave of the causal pass carries
constexpr int kPrefillWideWaves = 8; // waves of a workgroup of the causal pass over bf16 pools with head_dim 128 (else kWaves)
// Waves per workgroup of the causal pass for a pool type (0 = bf16, 1 = fp8) and head size: the host sizes the grid with it.
// (At head_dim 64 three workgroups of 4 waves fit a compute unit and beat one of 8.)
__host__ __device__ inline int prefill_waves(int kv_dtype, int head_dim) { return kv_dtype == 0 && head_dim == 128 ? kPrefillWideWaves : kWaves; }

// Chunk slots of one output row.  Without a shared prefix, chunk c covers tokens
// [c*chunk, (c+1)*chunk).  With a shared prefix of `sh` tokens (a multiple of
// 16) the first ceil(sh/chunk) slots cover the prefix (the last one may be
// short) and the following ones cover [sh + j*chunk, ...), so that the prefix
// is cut at the same places for every member of a group.
__host__ __device__ inline int shared_slots(int sh, int chunk) { return (sh + chunk - 1) / chunk; }

// Arguments of the split-K pass (by value, lives in kernel-argument memory).
struct SplitArgs {
    const uint16_t *q;           // [B][Hq][D] bf16
    const void *k_pages;         // [num_pages][Hkv][16][D]
    const void *v_pages;
    const float *k_scales;       // [num_pages][Hkv] (fp8) or null
    const float *v_scales;
    const int32_t *block_table;  // [B][max_blocks]
    const int32_t *context_lens; // [B]
    float *ws_m;                 // [B][Hq][S]   running max, log2 domain
    float *ws_l;                 // [B][Hq][S]   sum of weights
    float *ws_acc;               // [B][Hq][S][D] weighted V sum
    float *out_direct;           // [B][Hq][D] or null: every sequence is one chunk, write the output instead of partials
    float scale_log2e;           // scale * log2(e)
    // the shared-prefix items fold a non-negative scale into their exponent: |scale| * log2(e), the sign as a
    // bit flip of the queries (0x80008000 when scale < 0), and zeroed queries with scale 1 when scale == 0
    float abs_scale_log2e;
    uint32_t q_flip, q_keep;
    int32_t B, Hq, Hkv, G;
    int32_t HB;                  // head blocks per KV head: ceil(G / 16)
    int32_t max_blocks, S, chunk_tokens, max_context_len;
    // shared-prefix groups (all zero / null when the call has none)
    const int32_t *group_start;  // [num_groups + 1] first sequence of each group
    const int32_t *shared_len;   // [B] tokens whose pages the sequence shares with its whole group
    int32_t num_groups, group_subs;  // group_subs: workgroups (4 x 16/G sequences each) that cover the largest group
    uint32_t group_items;        // grid entries that serve shared prefixes (they come first)
    int32_t max_shared_len;      // host-known bound on shared_len[]; larger values are clamped to it
    int32_t grid_chunks;         // chunk slots the plain part of the grid spans (S, or S-1 without groups)
};

// Hand-over inside a workgroup.  The four waves of a workgroup walk neighbouring pieces (ranges 4i ..
// 4i + 3).  When the LAST segment of a wave's piece began before the piece (then it is the piece's only
// segment and continues the last segment of the wave before), and the wave is not the workgroup's first,
// its result does not go to memory: it is handed through LDS to the wave before, which adds it to its own.
// Such a run of waves leaves one partial (in the slot of its first wave) or, when it holds the whole
// sequence, the finished rows.  Whether range r handed over its part of the sequence whose tiles are
// [o0, o1) of a line of T tiles follows from the geometry alone, so the merge pass needs no marker.
__host__ __device__ inline bool handed_over(int r, int o0, int o1, int T, int per)
{
    const int end = (r + 1) * per < T ? (r + 1) * per : T;
    return r % kWaves != 0 && o0 < r * per && o1 >= end;
}
// The ranges that still hold a part of a sequence spread over ranges r_first .. r_last: r_first, every
// workgroup's first range in between, and r_last unless it handed over.
struct LiveParts {
    int r_first, r_last, first_lead, leads, count;
    __host__ __device__ int range(int i) const { return i == 0 ? r_first : i <= leads ? first_lead + kWaves * (i - 1) : r_last; }
};
__host__ __device__ inline LiveParts live_parts(int o0, int o1, int T, int per)
{
    LiveParts p;
    p.r_first = o0 / per, p.r_last = (o1 - 1) / per;
    p.first_lead = (p.r_first / kWaves + 1) * kWaves;
    p.leads = p.r_last > p.first_lead ? (p.r_last - 1 - p.first_lead) / kWaves + 1 : 0;   // multiples of 4 inside (r_first, r_last)
    p.count = 1 + p.leads + (p.r_last > p.r_first && !handed_over(p.r_last, o0, o1, T, per) ? 1 : 0);
    return p;
}

// Arguments of the range pass (batches without shared prefixes).  Per (virtual) KV head the batch is one line of 32-token tiles (sequence after
// sequence); the line is cut into `ranges` equal ranges and each wave walks one of them.
constexpr int kMaxRangeBatch = 4096;  // sequences whose tile offsets fit the workgroup's LDS
struct RangeArgs {
    const uint16_t *q;
    const void *k_pages, *v_pages;
    const float *k_scales, *v_scales;
    const int32_t *block_table, *context_lens;
    float *out;                  // [B][Hq][D]
    // append and attend in one go (bf16 pools; all null otherwise): row b of k_new / v_new [B][Hkv][D] is the
    // newest token of sequence b, at position context_lens[b] - 1; it is attended from these rows and written
    // into the pool
    const uint16_t *k_new, *v_new;
    uint16_t *k_pages_out, *v_pages_out;
    int32_t *tile_off;           // [B + 1] written for the merge pass: tiles of the sequences before b
    int4 *merge_rec;             // [ranges][Hv] written for the merge pass: {b, tile_off[b], tile_off[b+1], T} of the cut
                                 // sequence whose first part the range holds, or b = -1
    float *ws_m, *ws_l;          // [slots][16]   a wave's partial rows: running max (log2 domain), weight sum
    float *ws_acc;               // [slots][rows_stride][D]   weighted V sums; slot = (range * Hv + head) * 2 + which
    uint32_t *sink;              // probe launches only: one word per wave
    float scale_log2e;           // scale * log2(e)
    int32_t B, Hq, Hkv, G, HB, max_blocks, max_context_len;
    int32_t ranges;              // ranges per virtual head: 4 x (grid / (Hkv * HB))
    int32_t min_tiles;           // a range holds at least this many tiles (unless the batch has fewer)
    int32_t rows_stride;         // rows per partial slot: min(G, 16)
};

struct RangeMergeArgs {
    const int32_t *tile_off;
    const int4 *merge_rec;
    const float *ws_m, *ws_l, *ws_acc;
    float *out;
    int32_t B, Hq, Hkv, G, HB, ranges, min_tiles, rows_stride;
    int32_t by_sequence;         // items are (sequence, head block) instead of (range, head block)
};

struct MergeArgs {
    const float *ws_m, *ws_l, *ws_acc;
    const int32_t *context_lens;
    float *out;                  // [B][Hq][D]
    int32_t B, Hq, S, chunk_tokens, max_context_len;
    const int32_t *shared_len;   // [B] or null, as in SplitArgs
    int32_t max_shared_len;
};

// Arguments of the causal multi-query pass.
struct PrefillArgs {
    const uint16_t *q;           // [total_q][Hq][D] bf16
    const int32_t *q_start;      // [B + 1] first query row of each sequence
    const void *k_pages, *v_pages;
    const float *k_scales, *v_scales;
    const int32_t *block_table, *context_lens;
    float *out;                  // [total_q][Hq][D]
    float scale_log2e;           // |scale| * log2(e); the sign of scale travels in q_flip
    uint32_t q_flip;             // 0x80008000 when scale < 0: every query element changes sign as it is loaded
    uint32_t q_keep;             // 0 when scale == 0 (all scores are zero: zero queries, scale 1), else all ones
    int32_t B, Hq, Hkv, G, HB, max_blocks, max_context_len;  // HB: head blocks per KV head, ceil(G / 16)
    int32_t total_q, max_q_len;  // rows of q; host-known bound on the rows of one sequence
    int32_t q_blocks;            // workgroups (prefill_waves x kPrefillBlocks x 16/G query tokens each) that cover max_q_len
};

struct AppendArgs {
    const uint4 *k_new, *v_new;  // [T][Hkv][D] bf16 viewed as 16-byte words
    const int32_t *seq_ids, *positions;   // [T], or both null: row j = sequence j's newest token (see context_lens)
    uint4 *k_pages, *v_pages;
    const int32_t *block_table;
    const int32_t *context_lens;          // used only without index arrays
    int32_t T, Hkv, max_blocks, max_context_len;
};

struct AppendFp8Args {
    const uint4 *k_new, *v_new;  // [T][Hkv][d] bf16 viewed as 16-byte words
    const int32_t *range_seq, *range_start, *range_row0;  // [R], [R], [R+1]
    uint8_t *k_pages, *v_pages;
    float *k_scales, *v_scales;
    const int32_t *block_table;
    int32_t R, Hkv, max_blocks, pages_per_range;
    uint32_t num_tiles;          // 2 * R * pages_per_range * Hkv (K and V tiles)
    int32_t single_rows;         // every range has at most one row (the decode step)
};

struct CopyPagesArgs {
    const int32_t *src_pages, *dst_pages;  // [N]
    uint4 *k_pages, *v_pages;              // pools viewed as 16-byte words
    float *k_scales, *v_scales;            // [num_pages][Hkv] or null
    int32_t N, Hkv, num_pages;
    int32_t page_words;                    // 16-byte words of one page over all heads
};

struct ValidateArgs {
    const int32_t *block_table, *context_lens;
    int32_t *report;             // [2]: bad table entries in use, bad lengths
    int32_t B, max_blocks, num_pages, max_context_len;
};

struct ValidateGroupsArgs {
    const int32_t *block_table, *context_lens, *group_start, *shared_len;
    int32_t *report;             // [4]
    int32_t B, max_blocks, max_context_len, num_groups, max_group_size, max_shared_len;
};

// Launchers: enqueue on `stream`, return the hipError_t of the launch.  When
// `start`/`stop` are given they are bound to the kernel's own begin and end
// timestamps (hipExtLaunchKernelGGL), so their elapsed time is the kernel's
// duration without launch latency.
hipError_t launch_split(const SplitArgs &a, int head_dim, int kv_dtype, hipStream_t stream,
                        hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
hipError_t launch_range(const RangeArgs &a, int head_dim, int kv_dtype, unsigned grid, bool probe, hipStream_t stream,
                        hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
hipError_t launch_range_merge(const RangeMergeArgs &a, int head_dim, hipStream_t stream,
                              hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
hipError_t launch_merge(const MergeArgs &a, int head_dim, hipStream_t stream,
                        hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
hipError_t launch_prefill(const PrefillArgs &a, int head_dim, int kv_dtype, hipStream_t stream,
                          hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
hipError_t launch_append(const AppendArgs &a, int head_dim, hipStream_t stream);
hipError_t launch_append_fp8(const AppendFp8Args &a, int head_dim, hipStream_t stream);
hipError_t launch_copy_pages(const CopyPagesArgs &a, hipStream_t stream);
hipError_t launch_validate(const ValidateArgs &a, hipStream_t stream);
hipError_t launch_validate_groups(const ValidateGroupsArgs &a, hipStream_t stream);

}  // namespace sd
