/*
 * libseamdecode -- paged decode attention for rollout on MI355X (gfx950).
 *
 * The paper's framework spends most of its run time in rollout, i.e. batched
 * autoregressive decoding inside the inference engine (System Overview, engine
 * layer; Pipeline Bubble Analysis).  Each decode step attends one new query token per sequence over that sequence's
 * KV cache.  Sequences have different lengths, are paused and resumed from
 * their stored tokens (Data Plane: Rollout Manager, Trajectory Manager) and
 * several trajectories of one session continue a common prefix (Trajectory
 * Manager: longest-prefix matching / prefix tree), so the cache is paged and
 * a block table maps each sequence's logical pages to physical pages that
 * may be shared between sequences.
 *
 * Conventions for every call below
 *   - All data pointers are DEVICE pointers owned by the caller and must be
 *     16-byte aligned.  The library never allocates, frees or retains device
 *     memory and never synchronises: a call validates its arguments on the
 *     host, enqueues its kernels on `stream` (a hipStream_t, NULL = default
 *     stream) and returns.
 *   - Return value: SD_OK (0) or a negative SD_E* code.  On a validation
 *     error nothing is enqueued and no output is written.
 *   - No global state (paged_decode_attention_static excepted, which owns one
 *     scratch array per GPU): calls from several host threads are independent.
 *     Calls that write the same output/workspace/pages must be ordered by the
 *     caller (same stream or events).
 *
 * Memory layouts (P = 16 tokens per page, d = head_dim, row-major, C order)
 *   q            bf16   [batch][num_q_heads][d]
 *   k_pages      bf16   [num_pages][num_kv_heads][16][d]     (SD_BF16)
 *                u8     [num_pages][num_kv_heads][16][d]     (SD_FP8_E4M3: OCP e4m3fn codes)
 *   v_pages      same shape and type as k_pages, separate pool
 *   k_scales     f32    [num_pages][num_kv_heads]            (fp8 only: value = code * scale)
 *   v_scales     f32    [num_pages][num_kv_heads]
 *   block_table  i32    [batch][max_blocks_per_seq]          physical page of logical page j
 *   context_lens i32    [batch]
 *   out          f32    [batch][num_q_heads][d]
 * Token t of sequence b is stored in page block_table[b][t / 16], slot t % 16.
 * Query head h uses KV head h / (num_q_heads / num_kv_heads).
 * Slots at positions >= context_lens[b] and table entries past the last
 * logical page are never read, whatever they contain.
 */
#ifndef SEAMDECODE_H
#define SEAMDECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SD_OK 0
#define SD_EINVAL (-1)       /* null or misaligned pointer, or a dimension out of range */
#define SD_EUNSUPPORTED (-2) /* valid request this build has no kernel for */
#define SD_EWORKSPACE (-3)   /* workspace smaller than sd_workspace_bytes() */
#define SD_EHIP (-4)         /* a HIP call failed; see sd_last_hip_error() */

struct sd_timer; /* see the measurement aids at the end */

#define SD_BF16 0
#define SD_FP8_E4M3 1

typedef struct {
    int32_t batch;              /* B >= 0 (0: the call is a no-op) */
    int32_t num_q_heads;        /* Hq */
    int32_t num_kv_heads;       /* Hkv; Hq % Hkv == 0 and Hq / Hkv <= 64 (above 16 the K/V of a head
                                   is read once per block of 16 query heads, mostly from cache) */
    int32_t head_dim;           /* 64 or 128 */
    int32_t page_size;          /* must be 16 */
    int32_t num_pages;          /* extent of the pools */
    int32_t max_blocks_per_seq; /* row stride of block_table */
    int32_t kv_dtype;           /* SD_BF16 or SD_FP8_E4M3 */
    int32_t max_context_len;    /* host-known upper bound on context_lens[]; lengths above it
                                   are treated as max_context_len; <= 16 * max_blocks_per_seq */
    int32_t chunk_tokens;       /* split-K chunk in tokens: 0 = library default, else a
                                   multiple of 128 in [128, 65536] */
} sd_shape;

/* Library version: major * 10000 + minor * 100 + patch. */
int sd_version(void);

/* Static, human-readable text for an SD_* code. */
const char *sd_strerror(int code);

/* hipError_t (as int) of the last failing HIP call made by this thread; 0 if none. */
int sd_last_hip_error(void);

/* The split-K chunk (tokens) the library uses for this shape; <= 0 is an SD_E* code.
   With shape->chunk_tokens == 0 it is chosen from the shape alone, taking sequences
   to average 55 % of max_context_len. */
int sd_chunk_tokens(const sd_shape *shape);

/* The chunk that balances the split pass for a batch whose sequences hold
   `total_tokens` distinct K/V tokens per KV head in all (the sum of context_lens,
   counting the tokens of a shared prefix once): a caller that tracks its
   trajectories' lengths on the host puts the result into shape->chunk_tokens.
   A multiple of 128; <= 0 is an SD_E* code. */
int sd_chunk_for_batch(const sd_shape *shape, int64_t total_tokens);

/*
 * Bytes of scratch paged_decode_attention needs for this shape (host-only
 * arithmetic).  Returns 0 for an invalid shape.
 */
size_t sd_workspace_bytes(const sd_shape *shape);

/*
 * kv_append -- write new tokens' K/V rows into their page slots.
 *
 * Advancing a rollout by one token, or resuming a paused trajectory from its
 * stored tokens (Data Plane: partial rollout resumes from previously produced
 * tokens), puts rows into the cache: row j of k_new/v_new belongs to sequence
 * seq_ids[j] at position positions[j] and is copied, for every KV head, to
 * page block_table[seq_ids[j]][positions[j] / 16], slot positions[j] % 16.
 *
 *   k_new, v_new   bf16 [T][num_kv_heads][d]   (device, read)
 *   seq_ids        i32  [T]                    (device, read) in [0, batch)
 *   positions      i32  [T]                    (device, read) in [0, 16*max_blocks_per_seq)
 *   k_pages,v_pages                            (device, written at the addressed slots only)
 *   block_table                                (device, read)
 * Only SD_BF16 pools are supported (SD_EUNSUPPORTED otherwise; see kv_append_fp8).  context_lens
 * is not touched: sequence state belongs to the caller.  Two rows that address
 * the same slot race.  T == 0 is a no-op.
 */
int kv_append(const sd_shape *shape, const void *k_new, const void *v_new,
              const int32_t *seq_ids, const int32_t *positions, int32_t T,
              void *k_pages, void *v_pages, const int32_t *block_table, void *stream);

/*
 * kv_append_fp8 -- quantising append into SD_FP8_E4M3 pools (head_dim 64 or 128).
 *
 * Resuming a paused trajectory from its stored tokens (Data Plane: partial
 * rollout) rewrites whole stretches of a sequence's cache, and a decode step
 * adds one token; with an fp8 cache the rows are quantised as they are
 * written.  Rows arrive as ranges: range r is the rows range_row0[r] ..
 * range_row0[r+1]-1 of k_new/v_new (bf16 [T][num_kv_heads][128], device) and
 * goes to positions range_start[r] .. of sequence range_seq[r].
 *
 * Per (page, KV head) tile a range touches, for K and V alike: the tile's
 * scale is absmax/448 over its valid tokens.  If the range starts inside the
 * page and its rows do not exceed the tile's current absmax (scale*448) the
 * scale and the codes already there stay; otherwise the scale becomes the new
 * rows' absmax/448 (1 if that is 0) and the codes before the range are
 * re-encoded as code*(old_scale/new_scale).  A range that starts a page treats
 * the page as fresh, whatever its old scale.  Codes are the nearest e4m3fn
 * value of x/scale (ties to even, saturating at +-448); all arithmetic fp32.
 *
 *   range_seq, range_start  i32 [num_ranges]      (device)
 *   range_row0              i32 [num_ranges + 1]  (device), ascending
 *   max_range_len           host-known bound on the rows of one range
 * Two ranges of one call that touch the same page race.  context_lens is not
 * touched.  Only SD_FP8_E4M3 shapes (SD_EUNSUPPORTED otherwise).
 */
int kv_append_fp8(const sd_shape *shape, const void *k_new, const void *v_new,
                  const int32_t *range_seq, const int32_t *range_start, const int32_t *range_row0,
                  int32_t num_ranges, int32_t max_range_len,
                  void *k_pages, void *v_pages, float *k_scales, float *v_scales,
                  const int32_t *block_table, void *stream);

/*
 * kv_copy_pages -- copy whole pages inside the pool.
 *
 * A session that branches where its last page is partly filled cannot share
 * that page: every branch will write its own next token into it.  Each new
 * branch gets a private copy (sessions branch into trajectories that continue a
 * common prefix, Data Plane; see sd_tree_fork).  For i < num_copies the K and V
 * tiles of all KV heads of page src_pages[i], and for SD_FP8_E4M3 its scales,
 * are copied to page dst_pages[i], bit for bit.
 *
 *   src_pages, dst_pages  i32 [num_copies] (device); a pair with an id outside
 *                         [0, num_pages) or with src == dst is skipped
 * A page that is the destination of one pair and the source or destination of
 * another pair of the same call races.
 */
int kv_copy_pages(const sd_shape *shape, const int32_t *src_pages, const int32_t *dst_pages,
                  int32_t num_copies, void *k_pages, void *v_pages, float *k_scales, float *v_scales,
                  void *stream);

/*
 * paged_decode_attention -- one decode step of attention for every sequence.
 *
 * The step rollout repeats for every generated token (System Overview,
 * inference-engine layer; Data Plane: trajectories of different lengths that are
 * paused, resumed and branched share one paged cache).
 *
 * For each sequence b with L = min(max(context_lens[b], 0), max_context_len)
 * tokens (a negative length counts as 0, a length above the bound as the bound)
 * and each query head h (g = h / G):
 *     s_t = scale * <q[b][h], K_t>,  p = softmax_t(s),  out[b][h] = sum_t p_t V_t
 * with K_t, V_t the rows of KV head g at logical position t (fp8: code times
 * the page's scale).  L == 0 gives a zero row.  Products are accumulated in
 * fp32 from bf16 operands; softmax weights are rounded to bf16 before the
 * weighted sum and normalised by the sum of the rounded weights (fp8 pools: the
 * weight is rounded after the page's V scale has been folded in, and the sum
 * runs over those rounded weights divided by the scale again).
 *
 * Runs two kernels (batches of up to 4096 sequences).  Range pass: per KV head
 * the batch's 32-token tiles form one line, sequence after sequence; the line
 * is cut into as many equal ranges as the device runs waves at once and each
 * wave streams one range, so every K/V page leaves HBM once per (sequence, KV
 * head) and all waves carry the same load whatever the mix of lengths.  A wave
 * that holds a whole sequence writes its `out` rows itself; of a sequence cut
 * across ranges each wave leaves (max, sum, weighted sum) in `workspace`.  Merge
 * pass: combines the parts of every cut sequence in range order (results are
 * reproducible bit for bit).  shape->chunk_tokens, when non-zero, is the least
 * number of tokens a range holds.  Larger batches take the chunked passes of
 * paged_decode_attention_prefix.  Results do not depend on the physical
 * placement of pages.
 *
 *   k_scales, v_scales  NULL for SD_BF16
 *   workspace           >= sd_workspace_bytes(shape) bytes, contents ignored on entry
 */
int paged_decode_attention(const sd_shape *shape, const void *q,
                           const void *k_pages, const void *v_pages,
                           const float *k_scales, const float *v_scales,
                           const int32_t *block_table, const int32_t *context_lens,
                           float scale, float *out,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * paged_decode_attention_append -- one decode step in one call: the newest
 * token of every sequence is written into the cache AND attended.
 *
 * Advancing a rollout by one token (Data Plane: trajectories advance token by
 * token between pauses) appends that token's K/V and attends over the sequence
 * including it.  Row b of k_new / v_new (bf16 [batch][num_kv_heads][d], device)
 * is the K/V of sequence b's newest token, whose position is
 * context_lens[b] - 1 (the lengths passed already count it).  The result is
 * that of kv_append(rows at those positions) followed by
 * paged_decode_attention, bit for bit in the pool; where the range pass runs,
 * the wave that walks a sequence's last tile takes the token from the rows and
 * writes it into its slot, so no separate append kernel is launched.
 * Sequences with context_lens <= 0 are left alone (zero rows in `out`).
 * SD_BF16 pools only (SD_EUNSUPPORTED otherwise: fp8 pools take new tokens
 * through kv_append_fp8).  Other arguments as for paged_decode_attention;
 * `timer` may be NULL.
 */
int paged_decode_attention_append(const sd_shape *shape, const void *q,
                                  const void *k_new, const void *v_new,
                                  void *k_pages, void *v_pages,
                                  const int32_t *block_table, const int32_t *context_lens,
                                  float scale, float *out,
                                  void *workspace, size_t workspace_bytes, void *stream,
                                  struct sd_timer *timer);

/*
 * paged_decode_attention_static -- paged_decode_attention without a workspace
 * argument, for callers that cannot allocate device memory: code running under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 *
 * The partial results of sequences that are cut across waves go to an array of
 * SD_STATIC_SCRATCH_BYTES bytes that is part of the library itself (every GPU
 * the library runs on holds its own copy until the process ends).  The call allocates and frees nothing; the
 * first call on a device looks the array's address up (current device = the
 * device of `stream`), so make that first call outside graph capture.  Same
 * kernels, same arithmetic and bit-identical results as paged_decode_attention
 * with the same shape.
 *
 * Returns SD_EWORKSPACE, before anything is enqueued, when the shape needs more
 * scratch than the array holds (sd_workspace_bytes(shape) >
 * SD_STATIC_SCRATCH_BYTES).
 * All calls on one GPU share the one array: calls that overlap in time on the
 * same GPU (different streams, different host threads) race; order them.
 */
#define SD_STATIC_SCRATCH_BYTES (48u << 20)
int paged_decode_attention_static(const sd_shape *shape, const void *q,
                                  const void *k_pages, const void *v_pages,
                                  const float *k_scales, const float *v_scales,
                                  const int32_t *block_table, const int32_t *context_lens,
                                  float scale, float *out, void *stream);

/*
 * paged_decode_attention_prefix -- the same result as paged_decode_attention
 * for batches in which groups of sequences share the physical pages of a
 * common prefix.
 *
 * One session may branch into several trajectories that continue a common
 * prefix (Trajectory Manager: a per-session prefix tree built by
 * longest-prefix matching), so the block-table rows of a group start with the
 * same physical pages.  This entry point reads such pages from HBM once per
 * group and KV head instead of once per sequence: the query rows of the
 * group's sequences are stacked into the dense tiles of the shared chunks.
 * Tokens past the shared prefix are handled as in paged_decode_attention and
 * the same merge pass produces `out`.
 *
 *   group_start   i32 [num_groups + 1] (device): group j is the sequences
 *                 group_start[j] .. group_start[j+1]-1; groups need not cover
 *                 the batch, sequences outside every group need shared_len 0
 *   shared_len    i32 [batch] (device): tokens (from position 0) whose pages the
 *                 sequence shares with every sequence of its group; equal within
 *                 a group, <= context_lens of each member, 0 for ungrouped
 *                 sequences; rounded down to whole pages.  These tokens are
 *                 read once per group, everything after them once per sequence.
 *   num_groups, max_group_size, max_shared_len: host-known; upper bounds on the
 *                 group sizes and on shared_len[] (max_shared_len <= max_context_len)
 *   timer         NULL or an sd_timer (see below)
 * The caller guarantees that block_table[b][j] is the same for all b of a
 * group for j < shared_len/16; the library reads the first member's row.
 * num_groups == 0 makes the call identical to paged_decode_attention.
 */
int paged_decode_attention_prefix(const sd_shape *shape, const void *q,
                                  const void *k_pages, const void *v_pages,
                                  const float *k_scales, const float *v_scales,
                                  const int32_t *block_table, const int32_t *context_lens,
                                  const int32_t *group_start, const int32_t *shared_len,
                                  int32_t num_groups, int32_t max_group_size, int32_t max_shared_len,
                                  float scale, float *out,
                                  void *workspace, size_t workspace_bytes, void *stream,
                                  struct sd_timer *timer);

/*
 * paged_prefill_attention -- causal attention of several query tokens per
 * sequence over the paged cache.
 *
 * Rollout is interrupted and resumed (partial rollout; the Trajectory Manager
 * re-sends a session's stored prefix to whichever instance continues it, Data
 * Plane), and a resumed trajectory re-computes attention for a stretch of its
 * own tokens whose K/V already sit in the cache.  Sequence b owns the query
 * rows q_start[b] .. q_start[b+1]-1 of q; with n_b of them and
 * L = min(context_lens[b], max_context_len), row i is the query of position
 * pos = L - n_b + i and attends the tokens 0 .. pos:
 *     out[row][h] = softmax_{t <= pos}(scale * <q[row][h], K_t>) . V
 * i.e. paged_decode_attention with context length pos + 1 (the arithmetic is
 * the same: bf16 operands, fp32 accumulation, bf16 weights normalised by their
 * own sum).  n_b == 1 for every b is the decode step.  Rows with pos < 0 (more
 * queries than tokens) get zero rows.  One kernel, no workspace.
 *
 *   q         bf16 [total_q][num_q_heads][head_dim]  (device)
 *   q_start   i32 [batch + 1] (device), ascending, q_start[batch] <= total_q; a
 *             sequence whose range leaves [0, total_q) is skipped
 *   max_q_len host-known bound on n_b; rows past it in a sequence are not computed
 *   out       f32 [total_q][num_q_heads][head_dim]   (device); rows no sequence owns are left as they are
 *   timer     NULL or an sd_timer; the kernel's time is reported as split_ms, merge_ms reads ~0
 */
int paged_prefill_attention(const sd_shape *shape, const void *q, const int32_t *q_start,
                            int32_t total_q, int32_t max_q_len,
                            const void *k_pages, const void *v_pages,
                            const float *k_scales, const float *v_scales,
                            const int32_t *block_table, const int32_t *context_lens,
                            float scale, float *out, void *stream, struct sd_timer *timer);

/*
 * Session prefix tree (host only; no device memory, no HIP calls).
 *
 * The Trajectory Manager keeps the trajectories of a session in a prefix tree
 * built by longest-prefix matching and tags every token with the model version
 * that produced it (Data Plane, Trajectory Manager paragraph).  sd_tree does
 * that bookkeeping at KV-page granularity: trajectories share the physical
 * page of a full 16-token page exactly when all their tokens and version tags
 * up to the end of that page are equal; a partly filled last page is private.
 * The tree owns the page ids 0 .. num_pages-1 of a pool (free list, reference
 * counts) and emits block-table rows and the group arrays of
 * paged_decode_attention_prefix.  Not thread-safe: one tree, one thread.
 *
 *   sd_tree_insert        stores tokens[n] (+ versions[n], NULL = all 0); returns
 *                         the trajectory id (>= 0), SD_EINVAL, or SD_EWORKSPACE when
 *                         the pool is out of pages.  *matched_tokens (optional) =
 *                         leading tokens whose pages already existed: K/V has to be
 *                         appended from that position on only.
 *   sd_tree_match         the same count without storing anything
 *   sd_tree_release       drops a trajectory; unreferenced pages return to the pool
 *   sd_tree_fork          a second trajectory with the same tokens (a session branching):
 *                         shares every full page; a partly filled last page gets a
 *                         fresh private page, reported as *copy_src -> *copy_dst (-1, -1
 *                         when there is none) for kv_copy_pages.  Returns the new id,
 *                         SD_EINVAL or SD_EWORKSPACE
 *   sd_tree_append        one more token (a decode step); *page / *slot (optional) = where
 *                         its K/V rows go.  Takes a page from the pool when the last one
 *                         was full (SD_EWORKSPACE if none).  A page that fills up becomes
 *                         shareable by later inserts unless an equal one already is
 *   sd_tree_block_table   writes min(pages, cap) page ids, returns the page count
 *   sd_tree_token_at      token id / model version stored at a position
 *   sd_tree_batch_groups  for trajectories in batch order: consecutive ones that
 *                         start with the same page form a group; fills
 *                         group_start_out[groups + 1] and shared_len_out[B] (16 x the
 *                         pages common to the whole group, 0 for groups of one);
 *                         returns the number of groups
 */
typedef struct sd_tree sd_tree;
sd_tree *sd_tree_create(int32_t num_pages);
void sd_tree_destroy(sd_tree *t);
int32_t sd_tree_pages_in_use(const sd_tree *t);
int32_t sd_tree_match(const sd_tree *t, const int32_t *tokens, const uint32_t *versions, int32_t n);
int32_t sd_tree_insert(sd_tree *t, const int32_t *tokens, const uint32_t *versions, int32_t n,
                       int32_t *matched_tokens);
int sd_tree_release(sd_tree *t, int32_t traj);
int32_t sd_tree_fork(sd_tree *t, int32_t traj, int32_t *copy_src, int32_t *copy_dst);
int sd_tree_append(sd_tree *t, int32_t traj, int32_t token, uint32_t version, int32_t *page, int32_t *slot);
int32_t sd_tree_length(const sd_tree *t, int32_t traj);
int32_t sd_tree_block_table(const sd_tree *t, int32_t traj, int32_t *pages_out, int32_t cap);
int sd_tree_token_at(const sd_tree *t, int32_t traj, int32_t pos, int32_t *token, uint32_t *version);
int32_t sd_tree_batch_groups(const sd_tree *t, const int32_t *trajs, int32_t B, int32_t *group_start_out,
                             int32_t *shared_len_out);

/*
 * sd_validate_tables -- optional check of a batch's tables before they are used.
 *
 * The attention and append kernels trust block_table: an entry that does not
 * name a page of the pool is an out-of-bounds access.  A caller that builds
 * tables from untrusted bookkeeping can run this first (two tiny launches on
 * `stream`): report[0] receives the number of entries a launch would
 * dereference -- pages 0 .. ceil(L/16)-1 of every sequence, L clamped to
 * [0, max_context_len] -- that lie outside [0, num_pages), report[1] the
 * number of sequences whose context_lens is outside [0, max_context_len].
 *
 *   report   i32 [2] (device), 16-byte aligned; read it back after the stream has run
 */
int sd_validate_tables(const sd_shape *shape, const int32_t *block_table, const int32_t *context_lens,
                       int32_t *report, void *stream);

/*
 * sd_validate_groups -- optional check of the group arrays of
 * paged_decode_attention_prefix, which trusts them: a group larger than
 * max_group_size, members that disagree on shared_len, or members whose shared
 * pages are not the first member's all give wrong output without any error.
 * Two tiny launches on `stream` fill report[4] (i32, device, 16-byte aligned):
 *   report[0]  groups that are empty, reach outside the batch or hold more than
 *              max_group_size sequences
 *   report[1]  sequences whose shared_len differs from their group's first
 *              member's, is negative, exceeds their context_lens or
 *              max_shared_len, or is non-zero although they are in no group
 *   report[2]  members whose first shared_len / 16 block-table entries are not
 *              those of the group's first member
 *   report[3]  0
 * All zero means the arrays are consistent.  Nothing else is read or written.
 */
int sd_validate_groups(const sd_shape *shape, const int32_t *block_table, const int32_t *context_lens,
                       const int32_t *group_start, const int32_t *shared_len, int32_t num_groups,
                       int32_t max_group_size, int32_t max_shared_len, int32_t *report, void *stream);

/*
 * Measurement aids (not part of the decode step).
 *
 * sd_timer owns HIP events (host objects; no device memory).  The _timed
 * variant of the attention call binds a begin and an end event to each of its
 * two kernel launches on `stream` (the kernels' own start/stop timestamps, so
 * launch latency is not included); sd_timer_read waits for them and returns
 * the per-call kernel durations.
 */
typedef struct sd_timer sd_timer;
sd_timer *sd_timer_create(int32_t max_calls);
void sd_timer_destroy(sd_timer *t);
void sd_timer_reset(sd_timer *t);
/* Fills up to `cap` entries of split_ms[] / merge_ms[] (host arrays); returns the
   number of recorded calls or an SD_E* code.  Synchronises on the recorded events. */
int sd_timer_read(sd_timer *t, float *split_ms, float *merge_ms, int32_t cap);

int paged_decode_attention_timed(const sd_shape *shape, const void *q,
                                 const void *k_pages, const void *v_pages,
                                 const float *k_scales, const float *v_scales,
                                 const int32_t *block_table, const int32_t *context_lens,
                                 float scale, float *out,
                                 void *workspace, size_t workspace_bytes, void *stream,
                                 sd_timer *timer);

/*
 * sd_range_parts -- where the range pass of paged_decode_attention leaves the
 * parts of one sequence (host only, no device access; for tests and for reading
 * a profile).  Per KV head the batch's 32-token tiles form one line of
 * `line_tiles` tiles, cut into ranges of `tiles_per_range` tiles (range r =
 * tiles [r * tiles_per_range, (r + 1) * tiles_per_range)); the four ranges 4i ..
 * 4i + 3 belong to one workgroup, whose waves add up neighbouring parts of one
 * sequence before anything is stored.  For the sequence that occupies tiles
 * [first_tile, end_tile) of the line, writes the ranges that still hold a part,
 * ascending, to `ranges` (host, at most max_ranges entries) and returns their
 * number; 1 means the range pass finished the sequence itself and the merge
 * pass skips it.  SD_EINVAL for an empty or out-of-line sequence, a range size
 * below 1, or a null `ranges` with max_ranges > 0.
 */
int sd_range_parts(int first_tile, int end_tile, int line_tiles, int tiles_per_range, int *ranges, int max_ranges);

/*
 * sd_probe_read -- the kernel of paged_decode_attention with the arithmetic
 * taken out: same grid, same ranges, same loads of every K and V byte (and fp8
 * scale) the decode step must read, folded with XOR; one word per wave goes to
 * `sink` (u32 [sd_probe_sink_words(shape)], device).  Its duration is what the
 * memory system delivers for this walk on the machine at hand, i.e. the ceiling
 * for the decode step.  Batches above 4096 sequences: SD_EUNSUPPORTED.
 */
size_t sd_probe_sink_words(const sd_shape *shape);
int sd_probe_read(const sd_shape *shape, const void *k_pages, const void *v_pages,
                  const float *k_scales, const float *v_scales,
                  const int32_t *block_table, const int32_t *context_lens,
                  uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SEAMDECODE_H */
