// Merge pass: combines the per-chunk partials of the split pass into the
// attention output.  For row (b, h) with n non-empty chunks:
//   M = max_s m_s;  out = sum_s 2^(m_s-M) acc_s / sum_s 2^(m_s-M) l_s
// in fixed chunk order (m is kept in the base-2 domain by the split pass).
// A row's slots are those of its shared prefix followed by those of the rest.
// One workgroup per row, one thread per output element.
#include "kernels.h"

namespace sd {

template <int D>
__global__ __launch_bounds__(D) void merge_kernel(MergeArgs a)
{
    const int row = blockIdx.x;  // b * Hq + h
    const int b = row / a.Hq;
    const int d = threadIdx.x;
    const int L = max(0, min(a.context_lens[b], a.max_context_len));
    const int sh = a.shared_len ? max(0, min(min(a.shared_len[b], a.max_shared_len), L)) & ~(kPage - 1) : 0;
    const int n = shared_slots(sh, a.chunk_tokens) + (L - sh + a.chunk_tokens - 1) / a.chunk_tokens;
    float *o = a.out + (int64_t)row * D;
    if (n <= 0) {
        o[d] = 0.f;
        return;
    }
    const float *m = a.ws_m + (int64_t)row * a.S;
    const float *l = a.ws_l + (int64_t)row * a.S;
    const float *acc = a.ws_acc + (int64_t)row * a.S * D;
    float M = m[0];
    for (int s = 1; s < n; ++s) M = fmaxf(M, m[s]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < n; ++s) {
        const float w = __builtin_amdgcn_exp2f(m[s] - M);
        num += w * acc[(int64_t)s * D + d];
        den += w * l[s];
    }
    o[d] = num / den;
}

hipError_t launch_merge(const MergeArgs &a, int head_dim, hipStream_t stream, hipEvent_t start, hipEvent_t stop)
{
    const unsigned grid = (unsigned)a.B * (unsigned)a.Hq;
    if (grid == 0) return hipSuccess;
    if (head_dim == 128)
        if (start || stop) hipExtLaunchKernelGGL(merge_kernel<128>, dim3(grid), dim3(128), 0, stream, start, stop, 0, a);
        else hipLaunchKernelGGL(merge_kernel<128>, dim3(grid), dim3(128), 0, stream, a);
    else if (head_dim == 64)
        if (start || stop) hipExtLaunchKernelGGL(merge_kernel<64>, dim3(grid), dim3(64), 0, stream, start, stop, 0, a);
        else hipLaunchKernelGGL(merge_kernel<64>, dim3(grid), dim3(64), 0, stream, a);
    else
        return hipErrorNotSupported;
    return hipGetLastError();
}

}  // namespace sd
