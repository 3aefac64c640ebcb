// Merge pass: combines the per-chunk partials of the split pass into the
// attention output.  For row (b, h) with n non-empty chunks:
//   M = max_s m_s;  out = sum_s 2^(m_s-M) acc_s / sum_s 2^(m_s-M) l_s
// in fixed chunk order, four chunks at a time under a running maximum (m is kept in the base-2
// domain by the split pass).
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
    // four slots at a time, all their loads in flight together (a row rarely has more); folded in slot
    // order with a running maximum
    float M = -INFINITY, num = 0.f, den = 0.f;
    for (int base = 0; base < n; base += 4) {
        float ms[4], ls[4], as[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const bool valid = base + p < n;   // workgroup-uniform
            ms[p] = valid ? m[base + p] : -INFINITY;
            ls[p] = valid ? l[base + p] : 0.f;
            as[p] = valid ? acc[(int64_t)(base + p) * D + d] : 0.f;
        }
        const float M_new = fmaxf(fmaxf(M, fmaxf(ms[0], ms[1])), fmaxf(ms[2], ms[3]));
        const float shrink = __builtin_amdgcn_exp2f(M - M_new);   // first batch: exp2(-inf) = 0 on zeros
        M = M_new;
        num *= shrink;
        den *= shrink;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const float w = __builtin_amdgcn_exp2f(ms[p] - M);   // 0 for the slots that are not there
            num += w * as[p];
            den += w * ls[p];
        }
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
