// Read-only probe: walks the block table exactly like the split pass (same
// grid, same chunking, one workgroup per (chunk, sequence, kv head), each wave
// taking every fourth 32-token tile, one tile prefetched ahead) and loads
// every K and V byte of its chunk with coalesced 16-byte non-temporal loads,
// folding them with XOR.  No arithmetic, no LDS: its duration is what the
// memory system delivers for this access pattern (tiles of `tile_bytes`
// contiguous bytes at random page addresses), i.e. the ceiling for the split
// pass on the machine at hand.
#include "kernels.h"

namespace sd {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <int NL>  // 1024-byte loads per (page, head) tile and pool
__global__ __launch_bounds__(kWaves * 64, 2) void probe_kernel(ProbeArgs a)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int item = blockIdx.x;
    const int g = item % a.Hkv;
    const int b = (item / a.Hkv) % a.B;
    const int c = item / (a.Hkv * a.B);
    const int L = max(0, min(a.context_lens[b], a.max_context_len));
    const int t0 = c * a.chunk_tokens;
    if (t0 >= L) return;
    const int t1 = min(L, t0 + a.chunk_tokens);
    const int ntiles = (t1 - t0 + kTileTokens - 1) / kTileTokens;
    const int last_page = (t1 - t0 + kPage - 1) / kPage - 1;
    const int32_t *bt = a.block_table + (int64_t)b * a.max_blocks + t0 / kPage;
    const int64_t tile_bytes = a.tile_bytes;
    const int64_t page_bytes = tile_bytes * a.Hkv;
    const char *k = static_cast<const char *>(a.k_pages) + g * tile_bytes + lane * 16;
    const char *v = static_cast<const char *>(a.v_pages) + g * tile_bytes + lane * 16;

    struct Tile {
        u32x4 w[2][2][NL];  // [page][K or V][load]
    };
    const int nt = ntiles > wave ? (ntiles - wave + kWaves - 1) / kWaves : 0;
    auto page_ids = [&](int i, int &pa, int &pb) {
        const int ti = wave + kWaves * min(i, nt - 1);
        pa = bt[2 * ti];
        pb = bt[min(2 * ti + 1, last_page)];
    };
    auto issue = [&](Tile &r, int pa, int pb) {
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            r.w[0][0][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(k + pa * page_bytes + j * 1024));
            r.w[0][1][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(v + pa * page_bytes + j * 1024));
            r.w[1][0][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(k + pb * page_bytes + j * 1024));
            r.w[1][1][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(v + pb * page_bytes + j * 1024));
        }
    };
    u32x4 acc = {0, 0, 0, 0};
    auto consume = [&](const Tile &r) {
#pragma unroll
        for (int j = 0; j < NL; ++j) acc ^= r.w[0][0][j] ^ r.w[0][1][j] ^ r.w[1][0][j] ^ r.w[1][1][j];
    };
    if (nt > 0) {
        Tile ra, rb;
        int pa, pb;
        page_ids(0, pa, pb);
        issue(ra, pa, pb);
        page_ids(1, pa, pb);
        int i = 0;
        for (; i + 2 < nt; i += 2) {
            issue(rb, pa, pb);
            page_ids(i + 2, pa, pb);
            consume(ra);
            issue(ra, pa, pb);
            page_ids(i + 3, pa, pb);
            consume(rb);
        }
        if (i + 1 < nt) {
            issue(rb, pa, pb);
            consume(ra);
            consume(rb);
        } else {
            consume(ra);
        }
    }
    unsigned f = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    for (int off = 32; off > 0; off >>= 1) f ^= __shfl_xor(f, off, 64);
    __shared__ unsigned s[kWaves];
    if (lane == 0) s[wave] = f;
    __syncthreads();
    if (tid == 0) a.sink[item] = s[0] ^ s[1] ^ s[2] ^ s[3];
}

hipError_t launch_probe(const ProbeArgs &a, hipStream_t stream)
{
    const unsigned grid = (unsigned)a.S * (unsigned)a.B * (unsigned)a.Hkv;
    if (grid == 0) return hipSuccess;
    switch (a.tile_bytes) {
    case 4096: hipLaunchKernelGGL(probe_kernel<4>, dim3(grid), dim3(kWaves * 64), 0, stream, a); break;
    case 2048: hipLaunchKernelGGL(probe_kernel<2>, dim3(grid), dim3(kWaves * 64), 0, stream, a); break;
    case 1024: hipLaunchKernelGGL(probe_kernel<1>, dim3(grid), dim3(kWaves * 64), 0, stream, a); break;
    default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

// Table check for callers that want one before trusting a new block table: counts the entries a
// launch would dereference (pages 0 .. ceil(L / 16) - 1 of every sequence) that do not name a page of
// the pool, and the sequences whose length is outside [0, max_context_len].
__global__ void validate_clear_kernel(int32_t *report)
{
    report[0] = 0;
    report[1] = 0;
}

__global__ __launch_bounds__(256) void validate_kernel(ValidateArgs a)
{
    const int b = blockIdx.x;
    const int L = a.context_lens[b];
    if (threadIdx.x == 0 && (L < 0 || L > a.max_context_len)) atomicAdd(&a.report[1], 1);
    const int used = (min(max(L, 0), a.max_context_len) + kPage - 1) / kPage;
    int bad = 0;
    for (int j = threadIdx.x; j < used; j += 256) {
        const int p = a.block_table[(int64_t)b * a.max_blocks + j];
        bad += p < 0 || p >= a.num_pages;
    }
    if (bad) atomicAdd(&a.report[0], bad);
}

hipError_t launch_validate(const ValidateArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(validate_clear_kernel, dim3(1), dim3(1), 0, stream, a.report);
    if (a.B > 0) hipLaunchKernelGGL(validate_kernel, dim3(a.B), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace sd
