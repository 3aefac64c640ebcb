// Host side of libseamdecode: argument validation and kernel dispatch behind
// the C ABI declared in include/seamdecode.h.  No device allocation, no
// synchronisation (sd_timer_read excepted, which waits on its own events).
#include "../../include/seamdecode.h"
#include "kernels.h"

#include <algorithm>
#include <atomic>
#include <new>
#include <vector>

// Scratch of paged_decode_attention_static: one array per GPU, part of the library's code object, so it
// exists on a device from the moment the library is loaded there until the process ends.  In host
// code the array's name is only a handle, not a device address.
static __device__ __align__(256) unsigned char scratch[SD_STATIC_SCRATCH_BYTES];

namespace {

thread_local int tl_hip_error = 0;

int hip_fail(hipError_t e)
{
    tl_hip_error = (int)e;
    return SD_EHIP;
}

// Workgroups of 4 waves at 2 waves per SIMD that the largest device this library targets runs at once
// (256 compute units x 2).
constexpr int kMaxRangeWorkgroups = 512;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool bad_ptr(const void *p) { return p == nullptr || !aligned16(p); }

// Shape checks common to every entry point.
int check_shape(const sd_shape *s)
{
    if (!s) return SD_EINVAL;
    if (s->batch < 0 || s->num_q_heads <= 0 || s->num_kv_heads <= 0 || s->num_pages < 0 ||
        s->max_blocks_per_seq <= 0 || s->max_context_len < 0 || s->head_dim <= 0)
        return SD_EINVAL;
    if (s->page_size != sd::kPage) return SD_EINVAL;
    if (s->num_q_heads % s->num_kv_heads != 0) return SD_EINVAL;
    if ((int64_t)s->max_context_len > (int64_t)sd::kPage * s->max_blocks_per_seq) return SD_EINVAL;
    if (s->kv_dtype != SD_BF16 && s->kv_dtype != SD_FP8_E4M3) return SD_EINVAL;
    if (s->chunk_tokens != 0 &&
        (s->chunk_tokens < 128 || s->chunk_tokens > 65536 || s->chunk_tokens % 128 != 0))
        return SD_EINVAL;
    if (s->head_dim != 64 && s->head_dim != 128) return SD_EUNSUPPORTED;
    if (s->num_q_heads / s->num_kv_heads > sd::kMaxGroup * sd::kMaxHeadBlocks) return SD_EUNSUPPORTED;
    return SD_OK;
}

// Split-K chunk for a batch that holds `total_tokens` K/V tokens per KV head in all.
//
// The grid runs the chunks longest first (full chunks, then every sequence's short last one), so
// the pass ends when the last full-size workgroup ends: a chunk should take somewhat less than the
// whole pass would on a perfectly balanced machine, total / (256 CUs x 2 workgroups).  Longer
// chunks leave the machine waiting for single workgroups; shorter ones pay more partials,
// prologues and merge work.  Measured optimum on four workloads: 0.65-0.85 of that share, flat
// within +-20 %, so the target 0.75 x share is rounded to the nearest of 2^k and 3 * 2^(k-1).
// Bounds: a chunk costs one partial per query head, about 2 * G / (chunk * elem_bytes) of its K/V
// bytes, kept near 1 % from below; 8192 tokens from above.  A target that covers the longest
// sequence gives one chunk per sequence (then no merge pass runs at all).
int chunk_for(const sd_shape *s, int64_t total_tokens)
{
    const int G = s->num_q_heads / s->num_kv_heads;
    const int elem = s->kv_dtype == SD_BF16 ? 2 : 1;
    int lo = 512;
    while (lo * elem < 200 * G && lo < 4096) lo *= 2;
    const int64_t whole = std::max<int64_t>(128, ((int64_t)s->max_context_len + 127) / 128 * 128);
    // workgroup slots of the largest device this library targets (256 compute units x 2); the chunk is a host-only
    // function of the shape so that callers can size buffers without a device, hence no device query here
    const int64_t share = total_tokens * s->num_kv_heads / kMaxRangeWorkgroups;  // tokens per workgroup slot
    const double target = (double)std::max<int64_t>(share * 3 / 4, lo);
    int best = lo;
    for (int c = 512; c <= 8192; c += (c & (c - 1)) ? c / 3 : c / 2) {  // 512, 768, 1024, 1536, ... 8192
        if (c < lo) continue;
        const double rc = c > target ? c / target : target / c, rb = best > target ? best / target : target / best;
        if (rc < rb) best = c;
    }
    return (int)std::min<int64_t>(best, whole);
}

// Without a token count the chunk is a function of the shape alone (so that chunk boundaries
// depend only on logical positions): sequences are taken to average 55 % of the length bound.
int pick_chunk(const sd_shape *s)
{
    if (s->chunk_tokens) return s->chunk_tokens;
    return chunk_for(s, (int64_t)s->batch * s->max_context_len * 55 / 100);
}

// Chunk slots per output row: one more than the length bound needs, because a
// shared prefix that ends inside a chunk splits that chunk in two.
int num_chunks(const sd_shape *s, int chunk)
{
    return (s->max_context_len + chunk - 1) / chunk + 1;
}

struct WsLayout {
    size_t m_off, l_off, acc_off, total;
};

WsLayout ws_layout(const sd_shape *s, int S)
{
    const size_t rows = (size_t)s->batch * (size_t)s->num_q_heads * (size_t)S;
    WsLayout w;
    w.m_off = 0;
    w.l_off = (rows * 4 + 255) & ~(size_t)255;
    w.acc_off = w.l_off + ((rows * 4 + 255) & ~(size_t)255);
    w.total = w.acc_off + rows * (size_t)s->head_dim * 4;
    return w;
}

// The device address of `scratch` is asked for once per device, with that device current, and kept.
constexpr size_t kStaticScratchBytes = SD_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Address of the current device's scratch array.
int static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return SD_EUNSUPPORTED;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e == hipSuccess ? hipErrorInvalidSymbol : e);
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // every thread gets the same address
    }
    *ptr = p;
    return SD_OK;
}

// Workspace of the range pass (batches without shared prefixes): the sequences' tile offsets for
// the merge pass, then the waves' partial slots.

struct RangeLayout {
    int rblocks;                 // workgroups per virtual head
    size_t slots;                // partial slots: two per wave
    size_t seq_off, m_off, l_off, acc_off, total;
};

// `workgroups`: how many the device takes at once (2 per compute unit), at most kMaxRangeWorkgroups.
RangeLayout range_layout(const sd_shape *s, int workgroups)
{
    const int G = s->num_q_heads / s->num_kv_heads;
    const int Hv = s->num_kv_heads * sd::head_blocks(G);
    RangeLayout r;
    r.rblocks = std::max(1, std::min(workgroups, kMaxRangeWorkgroups) / Hv);
    r.slots = (size_t)2 * sd::kWaves * r.rblocks * Hv;
    r.seq_off = (((size_t)s->batch + 1) * 4 + 255) & ~(size_t)255;
    r.m_off = r.seq_off + ((r.slots / 2 * 16 + 255) & ~(size_t)255);
    r.l_off = r.m_off + r.slots * sd::kMaxGroup * 4;
    r.acc_off = r.l_off + r.slots * sd::kMaxGroup * 4;
    r.total = r.acc_off + r.slots * (size_t)std::min(G, sd::kMaxGroup) * (size_t)s->head_dim * 4;
    return r;
}

// The range pass serves every batch whose tile offsets fit a workgroup's LDS; larger batches take
// the chunked split + merge passes.
bool range_pass_fits(const sd_shape *s) { return s->batch <= sd::kMaxRangeBatch; }

// Workgroups the current device runs at once with two per compute unit; asked once per device.
std::atomic<int> g_workgroups[kMaxDevices];
int device_workgroups(int *out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return SD_EUNSUPPORTED;
    int w = g_workgroups[dev].load(std::memory_order_acquire);
    if (!w) {
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess || cus <= 0) return hip_fail(e == hipSuccess ? hipErrorInvalidDevice : e);
        w = 2 * cus;
        g_workgroups[dev].store(w, std::memory_order_release);
    }
    *out = w;
    return SD_OK;
}

}  // namespace

struct sd_timer {
    std::vector<hipEvent_t> ev;  // 4 per call: split begin/end, merge begin/end
    int32_t max_calls = 0, calls = 0;
};

extern "C" {

int sd_version(void) { return 100; }

const char *sd_strerror(int code)
{
    switch (code) {
    case SD_OK: return "success";
    case SD_EINVAL: return "invalid argument (null or misaligned pointer, or dimension out of range)";
    case SD_EUNSUPPORTED: return "shape or dtype not supported by this build";
    case SD_EWORKSPACE: return "workspace too small; see sd_workspace_bytes()";
    case SD_EHIP: return "a HIP call failed; see sd_last_hip_error()";
    default: return "unknown error code";
    }
}

int sd_last_hip_error(void) { return tl_hip_error; }

int sd_chunk_tokens(const sd_shape *shape)
{
    const int rc = check_shape(shape);
    if (rc) return rc;
    return pick_chunk(shape);
}

int sd_chunk_for_batch(const sd_shape *shape, int64_t total_tokens)
{
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (total_tokens < 0) return SD_EINVAL;
    return chunk_for(shape, total_tokens);
}

size_t sd_workspace_bytes(const sd_shape *shape)
{
    if (check_shape(shape)) return 0;
    const int chunk = pick_chunk(shape);
    size_t t = ws_layout(shape, num_chunks(shape, chunk)).total;
    // the range pass, sized for the largest grid it ever uses
    if (range_pass_fits(shape)) t = std::max(t, range_layout(shape, kMaxRangeWorkgroups).total);
    return t ? t : 256;
}

int kv_append(const sd_shape *shape, const void *k_new, const void *v_new,
              const int32_t *seq_ids, const int32_t *positions, int32_t T,
              void *k_pages, void *v_pages, const int32_t *block_table, void *stream)
{
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (T < 0) return SD_EINVAL;
    if (shape->kv_dtype != SD_BF16) return SD_EUNSUPPORTED;
    if (T == 0) return SD_OK;
    if (bad_ptr(k_new) || bad_ptr(v_new) || bad_ptr(seq_ids) || bad_ptr(positions) || bad_ptr(k_pages) ||
        bad_ptr(v_pages) || bad_ptr(block_table))
        return SD_EINVAL;
    sd::AppendArgs a;
    a.k_new = static_cast<const uint4 *>(k_new);
    a.v_new = static_cast<const uint4 *>(v_new);
    a.seq_ids = seq_ids;
    a.positions = positions;
    a.k_pages = static_cast<uint4 *>(k_pages);
    a.v_pages = static_cast<uint4 *>(v_pages);
    a.block_table = block_table;
    a.context_lens = nullptr;
    a.T = T;
    a.Hkv = shape->num_kv_heads;
    a.max_blocks = shape->max_blocks_per_seq;
    a.max_context_len = shape->max_context_len;
    const hipError_t e = sd::launch_append(a, shape->head_dim, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SD_OK : hip_fail(e);
}

int kv_append_fp8(const sd_shape *shape, const void *k_new, const void *v_new, const int32_t *range_seq,
                  const int32_t *range_start, const int32_t *range_row0, int32_t num_ranges,
                  int32_t max_range_len, void *k_pages, void *v_pages, float *k_scales, float *v_scales,
                  const int32_t *block_table, void *stream)
{
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (num_ranges < 0 || max_range_len < 0) return SD_EINVAL;
    if (shape->kv_dtype != SD_FP8_E4M3) return SD_EUNSUPPORTED;
    if (num_ranges == 0 || max_range_len == 0) return SD_OK;
    if (bad_ptr(k_new) || bad_ptr(v_new) || bad_ptr(range_seq) || bad_ptr(range_start) || bad_ptr(range_row0) ||
        bad_ptr(k_pages) || bad_ptr(v_pages) || bad_ptr(k_scales) || bad_ptr(v_scales) || bad_ptr(block_table))
        return SD_EINVAL;
    sd::AppendFp8Args a;
    a.k_new = static_cast<const uint4 *>(k_new);
    a.v_new = static_cast<const uint4 *>(v_new);
    a.range_seq = range_seq;
    a.range_start = range_start;
    a.range_row0 = range_row0;
    a.k_pages = static_cast<uint8_t *>(k_pages);
    a.v_pages = static_cast<uint8_t *>(v_pages);
    a.k_scales = k_scales;
    a.v_scales = v_scales;
    a.block_table = block_table;
    a.R = num_ranges;
    a.Hkv = shape->num_kv_heads;
    a.max_blocks = shape->max_blocks_per_seq;
    a.pages_per_range = (max_range_len + sd::kPage - 2) / sd::kPage + 1;  // a range may start inside a page
    const uint64_t tiles = 2ull * (uint64_t)num_ranges * (uint64_t)a.pages_per_range * (uint64_t)a.Hkv;
    if (tiles > 0x7fffffffull) return SD_EUNSUPPORTED;
    a.num_tiles = (uint32_t)tiles;
    a.single_rows = max_range_len == 1;
    const hipError_t e = sd::launch_append_fp8(a, shape->head_dim, static_cast<hipStream_t>(stream));
    if (e == hipErrorNotSupported) return SD_EUNSUPPORTED;
    return e == hipSuccess ? SD_OK : hip_fail(e);
}

int kv_copy_pages(const sd_shape *shape, const int32_t *src_pages, const int32_t *dst_pages, int32_t num_copies,
                  void *k_pages, void *v_pages, float *k_scales, float *v_scales, void *stream)
{
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (num_copies < 0 || num_copies > 0x3fffffff) return SD_EINVAL;
    if (num_copies == 0) return SD_OK;
    if (bad_ptr(src_pages) || bad_ptr(dst_pages) || bad_ptr(k_pages) || bad_ptr(v_pages)) return SD_EINVAL;
    const bool fp8 = shape->kv_dtype == SD_FP8_E4M3;
    if (fp8 && (bad_ptr(k_scales) || bad_ptr(v_scales))) return SD_EINVAL;
    sd::CopyPagesArgs a;
    a.src_pages = src_pages;
    a.dst_pages = dst_pages;
    a.k_pages = static_cast<uint4 *>(k_pages);
    a.v_pages = static_cast<uint4 *>(v_pages);
    a.k_scales = fp8 ? k_scales : nullptr;
    a.v_scales = fp8 ? v_scales : nullptr;
    a.N = num_copies;
    a.Hkv = shape->num_kv_heads;
    a.num_pages = shape->num_pages;
    a.page_words = shape->num_kv_heads * sd::kPage * shape->head_dim * (fp8 ? 1 : 2) / 16;
    const hipError_t e = sd::launch_copy_pages(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SD_OK : hip_fail(e);
}

}  // extern "C"

namespace {

// The decode step behind every attention entry point.  `own_scratch`: the workspace is the
// library's own per-device array (looked up here, after validation); only the bytes the launch
// really uses are checked against its size.
int attend_impl(const sd_shape *shape, const void *q, const void *k_pages, const void *v_pages,
                const float *k_scales, const float *v_scales, const int32_t *block_table,
                const int32_t *context_lens, const int32_t *group_start, const int32_t *shared_len,
                int32_t num_groups, int32_t max_group_size, int32_t max_shared_len, float scale, float *out,
                void *workspace, size_t workspace_bytes, void *stream, sd_timer *timer, bool own_scratch,
                const void *k_new = nullptr, const void *v_new = nullptr)
{
    const int rc = check_shape(shape);
    if (rc) return rc;
    if ((k_new || v_new) && (shape->kv_dtype != SD_BF16 || bad_ptr(k_new) || bad_ptr(v_new)))
        return shape->kv_dtype != SD_BF16 ? SD_EUNSUPPORTED : SD_EINVAL;
    if (num_groups < 0 || max_group_size < 0 || max_shared_len < 0 || max_shared_len > shape->max_context_len)
        return SD_EINVAL;
    if (shape->batch == 0) return SD_OK;
    if (bad_ptr(q) || bad_ptr(k_pages) || bad_ptr(v_pages) || bad_ptr(block_table) || bad_ptr(context_lens) ||
        bad_ptr(out) || (!own_scratch && bad_ptr(workspace)))
        return SD_EINVAL;
    if (shape->kv_dtype == SD_FP8_E4M3 && (bad_ptr(k_scales) || bad_ptr(v_scales))) return SD_EINVAL;
    if (num_groups > 0 && (bad_ptr(group_start) || bad_ptr(shared_len) || max_group_size < 1)) return SD_EINVAL;
    if (!(scale == scale)) return SD_EINVAL;
    const int chunk = pick_chunk(shape);
    const int S = num_chunks(shape, chunk);
    const WsLayout w = ws_layout(shape, S);
    const int shared_chunks = num_groups > 0 ? (max_shared_len + chunk - 1) / chunk : 0;
    // every sequence fits one chunk and nothing is shared: one workgroup per (sequence, KV head) is balanced
    // as it is; the split pass normalises and writes `out` itself, no partials, no merge pass
    const bool direct = !shared_chunks && shape->max_context_len <= chunk;
    // otherwise, when nothing is shared: the range pass and its merge pass
    const bool ranged = !shared_chunks && !direct && range_pass_fits(shape);
    if (timer && timer->calls >= timer->max_calls) return SD_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipEvent_t none[4] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t *ev = timer ? &timer->ev[(size_t)timer->calls * 4] : none;
    hipError_t e;

    if (ranged) {
        // workspace checks use the largest layout (what sd_workspace_bytes reports), whatever the device
        if (own_scratch ? range_layout(shape, kMaxRangeWorkgroups).total > kStaticScratchBytes
                        : workspace_bytes < sd_workspace_bytes(shape))
            return SD_EWORKSPACE;
        int workgroups = 0;
        int rc2 = device_workgroups(&workgroups);
        if (rc2) return rc2;
        if (own_scratch && (rc2 = static_scratch(&workspace))) return rc2;
        const RangeLayout rl = range_layout(shape, workgroups);
        char *ws = static_cast<char *>(workspace);
        sd::RangeArgs ra;
        ra.q = static_cast<const uint16_t *>(q);
        ra.k_pages = k_pages;
        ra.v_pages = v_pages;
        ra.k_scales = k_scales;
        ra.v_scales = v_scales;
        ra.block_table = block_table;
        ra.context_lens = context_lens;
        ra.out = out;
        ra.tile_off = reinterpret_cast<int32_t *>(ws);
        ra.merge_rec = reinterpret_cast<int4 *>(ws + rl.seq_off);
        ra.ws_m = reinterpret_cast<float *>(ws + rl.m_off);
        ra.ws_l = reinterpret_cast<float *>(ws + rl.l_off);
        ra.ws_acc = reinterpret_cast<float *>(ws + rl.acc_off);
        ra.sink = nullptr;
        ra.k_new = static_cast<const uint16_t *>(k_new);
        ra.v_new = static_cast<const uint16_t *>(v_new);
        ra.k_pages_out = k_new ? static_cast<uint16_t *>(const_cast<void *>(k_pages)) : nullptr;
        ra.v_pages_out = k_new ? static_cast<uint16_t *>(const_cast<void *>(v_pages)) : nullptr;
        ra.scale_log2e = scale * 1.4426950408889634f;
        ra.B = shape->batch;
        ra.Hq = shape->num_q_heads;
        ra.Hkv = shape->num_kv_heads;
        ra.G = shape->num_q_heads / shape->num_kv_heads;
        ra.HB = sd::head_blocks(ra.G);
        ra.max_blocks = shape->max_blocks_per_seq;
        ra.max_context_len = shape->max_context_len;
        ra.ranges = sd::kWaves * rl.rblocks;
        ra.min_tiles = std::max(1, shape->chunk_tokens / sd::kTileTokens);
        ra.rows_stride = std::min(ra.G, sd::kMaxGroup);
        const unsigned grid = (unsigned)rl.rblocks * (unsigned)(ra.Hkv * ra.HB);
        if ((e = sd::launch_range(ra, shape->head_dim, shape->kv_dtype, grid, false, st, ev[0], ev[1])) != hipSuccess)
            return e == hipErrorNotSupported ? SD_EUNSUPPORTED : hip_fail(e);
        sd::RangeMergeArgs rm;
        rm.tile_off = ra.tile_off;
        rm.merge_rec = ra.merge_rec;
        rm.by_sequence = ra.B <= ra.ranges;
        rm.ws_m = ra.ws_m;
        rm.ws_l = ra.ws_l;
        rm.ws_acc = ra.ws_acc;
        rm.out = out;
        rm.B = ra.B;
        rm.Hq = ra.Hq;
        rm.Hkv = ra.Hkv;
        rm.G = ra.G;
        rm.HB = ra.HB;
        rm.ranges = ra.ranges;
        rm.min_tiles = ra.min_tiles;
        rm.rows_stride = ra.rows_stride;
        if ((e = sd::launch_range_merge(rm, shape->head_dim, st, ev[2], ev[3])) != hipSuccess) return hip_fail(e);
        if (timer) timer->calls++;
        return SD_OK;
    }

    if (k_new) {   // these passes read the newest token from the pool: put it there first
        sd::AppendArgs ap;
        ap.k_new = static_cast<const uint4 *>(k_new);
        ap.v_new = static_cast<const uint4 *>(v_new);
        ap.seq_ids = ap.positions = nullptr;
        ap.k_pages = static_cast<uint4 *>(const_cast<void *>(k_pages));
        ap.v_pages = static_cast<uint4 *>(const_cast<void *>(v_pages));
        ap.block_table = block_table;
        ap.context_lens = context_lens;
        ap.T = shape->batch;
        ap.Hkv = shape->num_kv_heads;
        ap.max_blocks = shape->max_blocks_per_seq;
        ap.max_context_len = shape->max_context_len;
        if ((e = sd::launch_append(ap, shape->head_dim, st)) != hipSuccess) return hip_fail(e);
    }
    if (own_scratch) {
        if (!direct && w.total > kStaticScratchBytes) return SD_EWORKSPACE;
        const int src = static_scratch(&workspace);
        if (src) return src;
    } else if (workspace_bytes < sd_workspace_bytes(shape)) {
        return SD_EWORKSPACE;
    }
    char *ws = static_cast<char *>(workspace);
    sd::SplitArgs sa;
    sa.q = static_cast<const uint16_t *>(q);
    sa.k_pages = k_pages;
    sa.v_pages = v_pages;
    sa.k_scales = k_scales;
    sa.v_scales = v_scales;
    sa.block_table = block_table;
    sa.context_lens = context_lens;
    sa.ws_m = reinterpret_cast<float *>(ws + w.m_off);
    sa.ws_l = reinterpret_cast<float *>(ws + w.l_off);
    sa.ws_acc = reinterpret_cast<float *>(ws + w.acc_off);
    sa.scale_log2e = scale * 1.4426950408889634f;
    sa.abs_scale_log2e = scale == 0 ? 1.0f : (scale < 0 ? -scale : scale) * 1.4426950408889634f;
    sa.q_flip = scale < 0 ? 0x80008000u : 0u;
    sa.q_keep = scale == 0 ? 0u : 0xffffffffu;
    sa.B = shape->batch;
    sa.Hq = shape->num_q_heads;
    sa.Hkv = shape->num_kv_heads;
    sa.G = shape->num_q_heads / shape->num_kv_heads;
    sa.HB = sd::head_blocks(sa.G);
    sa.max_blocks = shape->max_blocks_per_seq;
    sa.S = S;
    sa.chunk_tokens = chunk;
    sa.max_context_len = shape->max_context_len;
    // shared-prefix items: whole chunks of each group's shared prefix, 4 waves x (16 / G) sequences per workgroup
    const int seqs_per_wg = sd::kWaves * sd::units_per_block(sa.G);
    sa.group_start = shared_chunks ? group_start : nullptr;
    sa.shared_len = shared_chunks ? shared_len : nullptr;
    sa.num_groups = shared_chunks ? num_groups : 0;
    sa.group_subs = shared_chunks ? (max_group_size + seqs_per_wg - 1) / seqs_per_wg : 0;
    const uint64_t group_items = (uint64_t)shared_chunks * (uint64_t)sa.num_groups * (uint64_t)sa.group_subs *
                                 (uint64_t)(sa.Hkv * sa.HB);
    sa.grid_chunks = shared_chunks ? S : S - 1;  // the extra slot exists only where a shared prefix splits a chunk
    const uint64_t plain_items = (uint64_t)sa.grid_chunks * (uint64_t)shape->batch * (uint64_t)(sa.Hkv * sa.HB);
    if (group_items + plain_items > 0x7fffffffull) return SD_EUNSUPPORTED;
    sa.group_items = (uint32_t)group_items;
    sa.max_shared_len = max_shared_len;
    sa.out_direct = direct ? out : nullptr;

    sd::MergeArgs ma;
    ma.ws_m = sa.ws_m;
    ma.ws_l = sa.ws_l;
    ma.ws_acc = sa.ws_acc;
    ma.context_lens = context_lens;
    ma.out = out;
    ma.B = shape->batch;
    ma.Hq = shape->num_q_heads;
    ma.S = S;
    ma.chunk_tokens = chunk;
    ma.max_context_len = shape->max_context_len;
    ma.shared_len = sa.shared_len;
    ma.max_shared_len = max_shared_len;

    if ((e = sd::launch_split(sa, shape->head_dim, shape->kv_dtype, st, ev[0], ev[1])) != hipSuccess)
        return e == hipErrorNotSupported ? SD_EUNSUPPORTED : hip_fail(e);
    if (direct) {
        // no merge pass; the timer's second event pair brackets nothing
        if (timer && ((e = hipEventRecord(ev[2], st)) != hipSuccess || (e = hipEventRecord(ev[3], st)) != hipSuccess))
            return hip_fail(e);
    } else if ((e = sd::launch_merge(ma, shape->head_dim, st, ev[2], ev[3])) != hipSuccess) {
        return hip_fail(e);
    }
    if (timer) timer->calls++;
    return SD_OK;
}

}  // namespace

extern "C" {

int paged_decode_attention_prefix(const sd_shape *shape, const void *q, const void *k_pages,
                                  const void *v_pages, const float *k_scales, const float *v_scales,
                                  const int32_t *block_table, const int32_t *context_lens,
                                  const int32_t *group_start, const int32_t *shared_len, int32_t num_groups,
                                  int32_t max_group_size, int32_t max_shared_len, float scale, float *out,
                                  void *workspace, size_t workspace_bytes, void *stream, sd_timer *timer)
{
    return attend_impl(shape, q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens, group_start,
                       shared_len, num_groups, max_group_size, max_shared_len, scale, out, workspace,
                       workspace_bytes, stream, timer, false);
}

int paged_decode_attention_append(const sd_shape *shape, const void *q, const void *k_new, const void *v_new,
                                  void *k_pages, void *v_pages, const int32_t *block_table,
                                  const int32_t *context_lens, float scale, float *out, void *workspace,
                                  size_t workspace_bytes, void *stream, sd_timer *timer)
{
    if (bad_ptr(k_new) || bad_ptr(v_new)) return check_shape(shape) ? check_shape(shape) : SD_EINVAL;
    return attend_impl(shape, q, k_pages, v_pages, nullptr, nullptr, block_table, context_lens, nullptr, nullptr, 0, 0,
                       0, scale, out, workspace, workspace_bytes, stream, timer, false, k_new, v_new);
}

int paged_decode_attention_static(const sd_shape *shape, const void *q, const void *k_pages, const void *v_pages,
                                  const float *k_scales, const float *v_scales, const int32_t *block_table,
                                  const int32_t *context_lens, float scale, float *out, void *stream)
{
    return attend_impl(shape, q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens, nullptr, nullptr,
                       0, 0, 0, scale, out, nullptr, 0, stream, nullptr, true);
}

int paged_decode_attention_timed(const sd_shape *shape, const void *q, const void *k_pages,
                                 const void *v_pages, const float *k_scales, const float *v_scales,
                                 const int32_t *block_table, const int32_t *context_lens, float scale,
                                 float *out, void *workspace, size_t workspace_bytes, void *stream,
                                 sd_timer *timer)
{
    return paged_decode_attention_prefix(shape, q, k_pages, v_pages, k_scales, v_scales, block_table,
                                         context_lens, nullptr, nullptr, 0, 0, 0, scale, out, workspace,
                                         workspace_bytes, stream, timer);
}

int paged_decode_attention(const sd_shape *shape, const void *q, const void *k_pages, const void *v_pages,
                           const float *k_scales, const float *v_scales, const int32_t *block_table,
                           const int32_t *context_lens, float scale, float *out, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    return paged_decode_attention_prefix(shape, q, k_pages, v_pages, k_scales, v_scales, block_table,
                                         context_lens, nullptr, nullptr, 0, 0, 0, scale, out, workspace,
                                         workspace_bytes, stream, nullptr);
}

int paged_prefill_attention(const sd_shape *shape, const void *q, const int32_t *q_start, int32_t total_q,
                            int32_t max_q_len, const void *k_pages, const void *v_pages, const float *k_scales,
                            const float *v_scales, const int32_t *block_table, const int32_t *context_lens,
                            float scale, float *out, void *stream, sd_timer *timer)
{
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (total_q < 0 || max_q_len < 0) return SD_EINVAL;
    if (shape->batch == 0 || total_q == 0 || max_q_len == 0) return SD_OK;
    if (bad_ptr(q) || bad_ptr(q_start) || bad_ptr(k_pages) || bad_ptr(v_pages) || bad_ptr(block_table) ||
        bad_ptr(context_lens) || bad_ptr(out))
        return SD_EINVAL;
    if (shape->kv_dtype == SD_FP8_E4M3 && (bad_ptr(k_scales) || bad_ptr(v_scales))) return SD_EINVAL;
    if (!(scale == scale)) return SD_EINVAL;
    if (timer && timer->calls >= timer->max_calls) return SD_EINVAL;
    sd::PrefillArgs a;
    a.q = static_cast<const uint16_t *>(q);
    a.q_start = q_start;
    a.k_pages = k_pages;
    a.v_pages = v_pages;
    a.k_scales = k_scales;
    a.v_scales = v_scales;
    a.block_table = block_table;
    a.context_lens = context_lens;
    a.out = out;
    // the kernel folds a non-negative scale into its exponent; a negative one is the same problem with -q
    a.scale_log2e = (scale < 0 ? -scale : scale) * 1.4426950408889634f;
    a.q_flip = scale < 0 ? 0x80008000u : 0u;
    a.q_keep = scale == 0 ? 0u : 0xffffffffu;
    if (scale == 0) a.scale_log2e = 1.0f;  // zero queries give the same all-zero scores without 0 * inf in the mask
    a.B = shape->batch;
    a.Hq = shape->num_q_heads;
    a.Hkv = shape->num_kv_heads;
    a.G = shape->num_q_heads / shape->num_kv_heads;
    a.HB = sd::head_blocks(a.G);
    a.max_blocks = shape->max_blocks_per_seq;
    a.max_context_len = shape->max_context_len;
    a.total_q = total_q;
    a.max_q_len = max_q_len < total_q ? max_q_len : total_q;
    const int tokens_per_wg = sd::prefill_waves(shape->kv_dtype, shape->head_dim) * sd::kPrefillBlocks * sd::units_per_block(a.G);
    a.q_blocks = (a.max_q_len + tokens_per_wg - 1) / tokens_per_wg;
    if ((uint64_t)a.q_blocks * (uint64_t)a.B * (uint64_t)(a.Hkv * a.HB) > 0x7ffffff0ull) return SD_EUNSUPPORTED;
    hipEvent_t none[2] = {nullptr, nullptr};
    hipEvent_t *ev = timer ? &timer->ev[(size_t)timer->calls * 4] : none;
    const hipError_t e = sd::launch_prefill(a, shape->head_dim, shape->kv_dtype, static_cast<hipStream_t>(stream), ev[0], ev[1]);
    if (e != hipSuccess) return e == hipErrorNotSupported ? SD_EUNSUPPORTED : hip_fail(e);
    if (timer) {
        // the timer keeps four events per call; this call has one kernel, so the second pair brackets nothing
        hipError_t r = hipEventRecord(ev[2], static_cast<hipStream_t>(stream));
        if (r == hipSuccess) r = hipEventRecord(ev[3], static_cast<hipStream_t>(stream));
        if (r != hipSuccess) return hip_fail(r);
        timer->calls++;
    }
    return SD_OK;
}

sd_timer *sd_timer_create(int32_t max_calls)
{
    if (max_calls <= 0) return nullptr;
    sd_timer *t = new (std::nothrow) sd_timer;
    if (!t) return nullptr;
    t->max_calls = max_calls;
    t->ev.resize((size_t)max_calls * 4, nullptr);
    for (auto &e : t->ev) {
        const hipError_t rc = hipEventCreate(&e);
        if (rc != hipSuccess) {
            tl_hip_error = (int)rc;
            sd_timer_destroy(t);
            return nullptr;
        }
    }
    return t;
}

void sd_timer_destroy(sd_timer *t)
{
    if (!t) return;
    for (auto e : t->ev)
        if (e) (void)hipEventDestroy(e);
    delete t;
}

void sd_timer_reset(sd_timer *t)
{
    if (t) t->calls = 0;
}

int sd_timer_read(sd_timer *t, float *split_ms, float *merge_ms, int32_t cap)
{
    if (!t || !split_ms || !merge_ms || cap < 0) return SD_EINVAL;
    const int n = t->calls < cap ? t->calls : cap;
    for (int i = 0; i < n; ++i) {
        hipEvent_t *ev = &t->ev[(size_t)i * 4];
        hipError_t e = hipEventSynchronize(ev[3]);
        if (e == hipSuccess) e = hipEventElapsedTime(&split_ms[i], ev[0], ev[1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&merge_ms[i], ev[2], ev[3]);
        if (e != hipSuccess) return hip_fail(e);
    }
    return n;
}

int sd_validate_tables(const sd_shape *shape, const int32_t *block_table, const int32_t *context_lens,
                       int32_t *report, void *stream)
{
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (bad_ptr(report)) return SD_EINVAL;
    if (shape->batch > 0 && (bad_ptr(block_table) || bad_ptr(context_lens))) return SD_EINVAL;
    sd::ValidateArgs a;
    a.block_table = block_table;
    a.context_lens = context_lens;
    a.report = report;
    a.B = shape->batch;
    a.max_blocks = shape->max_blocks_per_seq;
    a.num_pages = shape->num_pages;
    a.max_context_len = shape->max_context_len;
    const hipError_t e = sd::launch_validate(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SD_OK : hip_fail(e);
}

int sd_validate_groups(const sd_shape *shape, const int32_t *block_table, const int32_t *context_lens,
                       const int32_t *group_start, const int32_t *shared_len, int32_t num_groups,
                       int32_t max_group_size, int32_t max_shared_len, int32_t *report, void *stream)
{
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (num_groups < 0 || max_group_size < 0 || max_shared_len < 0 || max_shared_len > shape->max_context_len)
        return SD_EINVAL;
    if (bad_ptr(report)) return SD_EINVAL;
    if (shape->batch > 0 && (bad_ptr(block_table) || bad_ptr(context_lens) || bad_ptr(shared_len))) return SD_EINVAL;
    if (num_groups > 0 && bad_ptr(group_start)) return SD_EINVAL;
    sd::ValidateGroupsArgs a;
    a.block_table = block_table;
    a.context_lens = context_lens;
    a.group_start = group_start;
    a.shared_len = shared_len;
    a.report = report;
    a.B = shape->batch;
    a.max_blocks = shape->max_blocks_per_seq;
    a.max_context_len = shape->max_context_len;
    a.num_groups = num_groups;
    a.max_group_size = max_group_size;
    a.max_shared_len = max_shared_len;
    const hipError_t e = sd::launch_validate_groups(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SD_OK : hip_fail(e);
}

int sd_range_parts(int first_tile, int end_tile, int line_tiles, int tiles_per_range, int *ranges, int max_ranges)
{
    if (first_tile < 0 || end_tile <= first_tile || end_tile > line_tiles || tiles_per_range <= 0 || max_ranges < 0 ||
        (max_ranges > 0 && !ranges))
        return SD_EINVAL;
    const sd::LiveParts parts = sd::live_parts(first_tile, end_tile, line_tiles, tiles_per_range);
    for (int i = 0; i < parts.count && i < max_ranges; ++i) ranges[i] = parts.range(i);
    return parts.count;
}

size_t sd_probe_sink_words(const sd_shape *shape)
{
    if (check_shape(shape) || !range_pass_fits(shape)) return 0;
    return range_layout(shape, kMaxRangeWorkgroups).slots / 2;  // one word per wave
}

int sd_probe_read(const sd_shape *shape, const void *k_pages, const void *v_pages, const float *k_scales,
                  const float *v_scales, const int32_t *block_table, const int32_t *context_lens, uint32_t *sink,
                  void *stream)
{
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (!range_pass_fits(shape)) return SD_EUNSUPPORTED;
    if (shape->batch == 0) return SD_OK;
    if (bad_ptr(k_pages) || bad_ptr(v_pages) || bad_ptr(block_table) || bad_ptr(context_lens) || bad_ptr(sink))
        return SD_EINVAL;
    if (shape->kv_dtype == SD_FP8_E4M3 && (bad_ptr(k_scales) || bad_ptr(v_scales))) return SD_EINVAL;
    int workgroups = 0;
    const int rc2 = device_workgroups(&workgroups);
    if (rc2) return rc2;
    const RangeLayout rl = range_layout(shape, workgroups);
    sd::RangeArgs ra = {};
    ra.k_pages = k_pages;
    ra.v_pages = v_pages;
    ra.k_scales = k_scales;
    ra.v_scales = v_scales;
    ra.block_table = block_table;
    ra.context_lens = context_lens;
    ra.sink = sink;
    ra.B = shape->batch;
    ra.Hq = shape->num_q_heads;
    ra.Hkv = shape->num_kv_heads;
    ra.G = shape->num_q_heads / shape->num_kv_heads;
    ra.HB = sd::head_blocks(ra.G);
    ra.max_blocks = shape->max_blocks_per_seq;
    ra.max_context_len = shape->max_context_len;
    ra.ranges = sd::kWaves * rl.rblocks;
    ra.min_tiles = std::max(1, shape->chunk_tokens / sd::kTileTokens);
    ra.rows_stride = std::min(ra.G, sd::kMaxGroup);
    const unsigned grid = (unsigned)rl.rblocks * (unsigned)(ra.Hkv * ra.HB);
    const hipError_t e = sd::launch_range(ra, shape->head_dim, shape->kv_dtype, grid, true, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SD_OK : hip_fail(e);
}

}  // extern "C"
