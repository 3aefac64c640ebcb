// kv_append: scatter new bf16 K/V rows into their page slots.
// One thread moves 16 bytes; a row of one (token, kv head) is D*2/16 threads,
// so a wave writes whole contiguous rows.  Thread order: (token, head, piece),
// piece fastest, K and V by the same thread.
#include "kernels.h"

namespace sd {

template <int D>
__global__ __launch_bounds__(256) void append_kernel(AppendArgs a)
{
    constexpr int kPieces = D * 2 / 16;  // 16-byte pieces per row
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)a.T * a.Hkv * kPieces;
    if (gid >= total) return;
    const int piece = (int)(gid % kPieces);
    const int g = (int)((gid / kPieces) % a.Hkv);
    const int j = (int)(gid / ((int64_t)kPieces * a.Hkv));
    const int seq = a.seq_ids[j], pos = a.positions[j];
    const int64_t page = a.block_table[(int64_t)seq * a.max_blocks + pos / kPage];
    const int64_t dst = ((page * a.Hkv + g) * kPage + pos % kPage) * kPieces + piece;
    a.k_pages[dst] = a.k_new[gid];
    a.v_pages[dst] = a.v_new[gid];
}

hipError_t launch_append(const AppendArgs &a, int head_dim, hipStream_t stream)
{
    const int64_t total = (int64_t)a.T * a.Hkv * (head_dim * 2 / 16);
    if (total == 0) return hipSuccess;
    const unsigned grid = (unsigned)((total + 255) / 256);
    if (head_dim == 128)
        hipLaunchKernelGGL(append_kernel<128>, dim3(grid), dim3(256), 0, stream, a);
    else if (head_dim == 64)
        hipLaunchKernelGGL(append_kernel<64>, dim3(grid), dim3(256), 0, stream, a);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace sd
