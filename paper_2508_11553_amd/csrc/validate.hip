// Table check (sd_validate_tables).
#include "kernels.h"

namespace sd {

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
