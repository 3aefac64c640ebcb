// Table and group checks (sd_validate_tables, sd_validate_groups).
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

// Group check for paged_decode_attention_prefix.  report[0]: groups that are empty, reach outside the
// batch or have more members than max_group_size; [1]: sequences whose shared_len disagrees with what
// the kernels assume (differs from the group's first member, is negative, exceeds the member's length
// or max_shared_len, or is non-zero outside every group); [2]: members whose first shared_len / 16
// table entries are not the first member's; [3]: unused (0).
__global__ void validate_groups_clear_kernel(int32_t *report)
{
    report[0] = report[1] = report[2] = report[3] = 0;
}

__global__ __launch_bounds__(256) void validate_groups_kernel(ValidateGroupsArgs a)
{
    const int j = blockIdx.x;
    if (j == a.num_groups) {   // the sequences outside every group (the groups tile [group_start[0], group_start[num_groups]))
        const int lo = a.num_groups ? a.group_start[0] : a.B, hi = a.num_groups ? a.group_start[a.num_groups] : a.B;
        int bad = 0;
        for (int b = threadIdx.x; b < a.B; b += 256) bad += (b < lo || b >= hi) && a.shared_len[b] != 0;
        if (bad) atomicAdd(&a.report[1], bad);
        return;
    }
    const int gs = a.group_start[j], ge = a.group_start[j + 1];
    if (gs < 0 || ge > a.B || ge <= gs || ge - gs > a.max_group_size) {
        if (threadIdx.x == 0) atomicAdd(&a.report[0], 1);
        if (gs < 0 || ge > a.B || ge <= gs) return;   // nothing inside can be indexed safely
    }
    const int sh0 = a.shared_len[gs];
    const int pages = max(0, min(min(sh0, a.max_shared_len), a.max_context_len)) / kPage;
    for (int b = gs + (threadIdx.x >> 6); b < ge; b += 4) {   // one wave per member
        const int lane = threadIdx.x & 63;
        const int sh = a.shared_len[b], L = a.context_lens[b];
        if (lane == 0 && (sh != sh0 || sh < 0 || sh > L || sh > a.max_shared_len)) atomicAdd(&a.report[1], 1);
        int differs = 0;
        for (int p = lane; p < pages; p += 64)
            differs |= a.block_table[(int64_t)b * a.max_blocks + p] != a.block_table[(int64_t)gs * a.max_blocks + p];
        if (__builtin_amdgcn_ballot_w64(differs != 0) && lane == 0) atomicAdd(&a.report[2], 1);
    }
}

hipError_t launch_validate_groups(const ValidateGroupsArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(validate_groups_clear_kernel, dim3(1), dim3(1), 0, stream, a.report);
    hipLaunchKernelGGL(validate_groups_kernel, dim3(a.num_groups + 1), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_validate(const ValidateArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(validate_clear_kernel, dim3(1), dim3(1), 0, stream, a.report);
    if (a.B > 0) hipLaunchKernelGGL(validate_kernel, dim3(a.B), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace sd
