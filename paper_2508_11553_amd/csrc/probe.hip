// Read-only probe: walks the block table exactly like the split pass (same
// grid, same chunking, one workgroup per (chunk, sequence, kv head)) and loads
// every K and V byte of its chunk with 16-byte non-temporal loads, folding them
// with XOR.
// It measures what the memory system delivers for this access pattern: tiles
// of `tile_bytes` contiguous bytes at random page addresses.
#include "kernels.h"

namespace sd {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kWaves * 64, 2) void probe_kernel(ProbeArgs a)
{
    const int tid = threadIdx.x;
    const int item = blockIdx.x;
    const int g = item % a.Hkv;
    const int b = (item / a.Hkv) % a.B;
    const int c = item / (a.Hkv * a.B);
    const int L = min(a.context_lens[b], a.max_context_len);
    const int t0 = c * a.chunk_tokens;
    if (t0 >= L) return;
    const int t1 = min(L, t0 + a.chunk_tokens);
    const int npages = (t1 - t0 + kPage - 1) / kPage;
    const int32_t *bt = a.block_table + (int64_t)b * a.max_blocks + t0 / kPage;
    const int words = a.tile_bytes / 16;              // 16-byte words per tile (128 or 256 or 64)
    const int64_t page_words = (int64_t)words * a.Hkv;
    const u32x4 *k = static_cast<const u32x4 *>(a.k_pages) + (int64_t)g * words;
    const u32x4 *v = static_cast<const u32x4 *>(a.v_pages) + (int64_t)g * words;
    // a tile is `words` 16-byte words; 256 threads cover 256/words tiles per step
    const int per_step = (kWaves * 64) / words;
    const int sub = tid / words, w = tid % words;
    u32x4 acc = {0, 0, 0, 0};
#pragma unroll 4
    for (int p = sub; p < npages; p += per_step) {
        const int64_t page = bt[p];
        const u32x4 x = __builtin_nontemporal_load(k + page * page_words + w);
        const u32x4 y = __builtin_nontemporal_load(v + page * page_words + w);
        acc ^= x ^ y;
    }
    unsigned f = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    for (int off = 32; off > 0; off >>= 1) f ^= __shfl_xor(f, off, 64);
    __shared__ unsigned s[kWaves];
    if ((tid & 63) == 0) s[tid >> 6] = f;
    __syncthreads();
    if (tid == 0) a.sink[item] = s[0] ^ s[1] ^ s[2] ^ s[3];
}

hipError_t launch_probe(const ProbeArgs &a, hipStream_t stream)
{
    const unsigned grid = (unsigned)a.S * (unsigned)a.B * (unsigned)a.Hkv;
    if (grid == 0) return hipSuccess;
    hipLaunchKernelGGL(probe_kernel, dim3(grid), dim3(kWaves * 64), 0, stream, a);
    return hipGetLastError();
}

}  // namespace sd
