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
// partial per (b, head, chunk); the merge kernel finishes the softmax.  When the
// host knows that every sequence is a single chunk, the workgroup writes the
// normalised output itself and no merge pass runs.
#include "attn_tile.h"

namespace sd {

// Tokens of sequence b that its group shares: whole pages, never more than the
// sequence has and never more than the host-side bound.
SD_DEV int shared_tokens(const SplitArgs &a, int b)
{
    const int L = max(0, min(a.context_lens[b], a.max_context_len));
    return max(0, min(min(a.shared_len[b], a.max_shared_len), L)) & ~(kPage - 1);
}

// Shared-prefix item: one workgroup owns one whole chunk of a group's shared
// prefix for one KV head and up to 64 query rows: wave w owns the 16 rows of
// column block w (G heads each of 16/G consecutive sequences of the group).
// The pages are the same for every member, so the first member's table row is
// read.  Per round each wave loads a different 32-token tile from HBM (one
// round prefetched ahead), parks its K image and the ready-made V^T operands
// in its LDS slot, and after a barrier every wave attends all four tiles from
// LDS with its own rows: each byte leaves HBM once per workgroup and the
// four-fold reuse is paid in LDS bandwidth.  These items fold |scale| into the
// exponent and take the sign of the scale through the queries (q_flip, q_keep).
// Every wave writes the partials of its own rows; nothing is merged across waves.
template <class P>
SD_DEV void shared_item(const SplitArgs &a, char *lds, int lane, int wave)
{
    constexpr int D = P::kDim;
    constexpr int kSlot = Lds<P>::kSlotBytes;
    const unsigned item = blockIdx.x;  // (chunk, group, block of 4 column blocks, head block), head block fastest
    const int Hv = a.Hkv * a.HB;
    const HeadBlock hb = head_block(item % Hv, a.G, a.HB);
    const int g = hb.g;
    const int sub = (item / Hv) % a.group_subs;
    const int grp = (item / (Hv * a.group_subs)) % a.num_groups;
    const int c = item / (Hv * a.group_subs * a.num_groups);
    const int gs = a.group_start[grp], ge = a.group_start[grp + 1];
    const int spw = units_per_block(a.G);  // sequences per column block
    if (gs + sub * kWaves * spw >= ge) return;                    // workgroup-uniform
    const int shared = shared_tokens(a, gs);
    const int t0 = c * a.chunk_tokens;
    if (t0 >= shared) return;  // workgroup-uniform
    const int t1 = min(shared, t0 + a.chunk_tokens);  // the prefix's last chunk may be short

    const int seq0 = gs + (sub * kWaves + wave) * spw;
    const bool active = seq0 < ge;  // wave-uniform; idle waves still load their tile and meet the barriers
    const int n = lane & 15;
    const int row_seq = seq0 + n / hb.rows;
    const int64_t row = (int64_t)row_seq * a.Hq + hb.head0 + n % hb.rows;
    const bool row_ok = active && n / hb.rows < spw && row_seq < ge;
    u32x4 qop[D / 32];
#pragma unroll
    for (int s = 0; s < D / 32; ++s)
        qop[s] = row_ok ? (*reinterpret_cast<const u32x4 *>(a.q + row * D + P::q_offset(s, lane)) & a.q_keep) ^ a.q_flip
                        : u32x4{0, 0, 0, 0};
    typename P::ParkedState st;
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
        P::v_park(r, mine + P::kScratchBytes, lane, t0 + (kWaves * rd + wave) * kTileTokens, t1);
        if (rd + 1 < rounds) issue(r, na, nb);
        __syncthreads();
        if (active) {
            const int ends[1] = {t1};
#pragma unroll 1
            for (int j = 0; j < kWaves; ++j) {
                const int tok0 = t0 + (kWaves * rd + j) * kTileTokens;
                if (tok0 >= t1) break;  // wave-uniform
                const char *slot = lds + j * kSlot;
                u32x4 ka[D / 32], kb[D / 32];
                P::k_fetch(slot, lane, ka, kb);
                auto &q1 = reinterpret_cast<const u32x4 (&)[1][D / 32]>(qop);
                auto &st1 = reinterpret_cast<typename P::ParkedState (&)[1]>(st);
                P::template attend_parked<1, true>(ka, kb, slot + P::kScratchBytes, q1, st1, a.abs_scale_log2e, tok0, lane, ends,
                                                   tok0 + kTileTokens > t1);  // the shared stretch ends inside the tile
            }
        }
        __syncthreads();
    }
    if (!active) return;
    const float l = P::weight_sum(st);
    if (row_ok) {
        const int64_t slot = row * a.S + c;
        P::store_acc(st, a.ws_acc + slot * D, lane >> 4);
        if ((lane >> 4) == 0) {
            a.ws_m[slot] = st.m;
            a.ws_l[slot] = l;
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
    const int Hv = a.Hkv * a.HB;
    const unsigned item = P::kDealByDie ? xcd_deal(blockIdx.x - a.group_items, gridDim.x - a.group_items, Hv) : blockIdx.x - a.group_items;
    const HeadBlock hb = head_block(item % Hv, a.G, a.HB);
    const int g = hb.g;
    const int b = (item / Hv) % a.B;
    const int from_end = a.grid_chunks - 1 - (int)(item / (Hv * a.B));

    const int L = max(0, min(a.context_lens[b], a.max_context_len));
    // slots of a shared prefix belong to the shared-prefix items; the others start where the prefix ends
    const int shared = a.shared_len ? shared_tokens(a, b) : 0;
    const int n_private = (L - shared + a.chunk_tokens - 1) / a.chunk_tokens;
    const int c_private = n_private - 1 - from_end;
    if (c_private < 0) {
        // single-chunk mode: an empty sequence still owes its zero rows
        if (a.out_direct && L == 0 && from_end == 0)
            for (int idx = tid; idx < hb.rows * D; idx += kWaves * 64)
                a.out_direct[((int64_t)b * a.Hq + hb.head0) * D + idx] = 0.f;
        return;
    }
    const int c = shared_slots(shared, a.chunk_tokens) + c_private;  // slot of this chunk
    const int t0 = shared + c_private * a.chunk_tokens;
    const int t1 = min(L, t0 + a.chunk_tokens);

    // Q^T operand: lane&15 = head n of the block; rows past the block's heads are zero
    const int n = lane & 15;
    u32x4 qop[D / 32];
    {
        const uint16_t *qrow = a.q + ((int64_t)b * a.Hq + hb.head0 + n) * D;
#pragma unroll
        for (int s = 0; s < D / 32; ++s)
            qop[s] = (n < hb.rows) ? *reinterpret_cast<const u32x4 *>(qrow + P::q_offset(s, lane)) : u32x4{0, 0, 0, 0};
    }

    typename P::State st;
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
    const int64_t row0 = (int64_t)b * a.Hq + hb.head0;
    for (int idx = tid; idx < hb.rows * D; idx += kWaves * 64) {
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
        if (a.out_direct) {  // the only chunk of its sequence: this is the result
            a.out_direct[(row0 + hn) * D + dd] = num / den;
            continue;
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
    const unsigned grid = a.group_items + (unsigned)a.grid_chunks * (unsigned)a.B * (unsigned)(a.Hkv * a.HB);
    if (grid == 0) return hipSuccess;
    const dim3 g(grid), b(kWaves * 64);
    if (kv_dtype == 0 && head_dim == 128)
        launch_one<Bf16Path<128>>(a, g, b, stream, start, stop);
    else if (kv_dtype == 0 && head_dim == 64)
        launch_one<Bf16Path<64>>(a, g, b, stream, start, stop);
    else if (kv_dtype == 1 && head_dim == 128)
        launch_one<Fp8Path>(a, g, b, stream, start, stop);
    else if (kv_dtype == 1 && head_dim == 64)
        launch_one<Fp8Path64>(a, g, b, stream, start, stop);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace sd
