// Ancestor masks of draft trees (paper Section 3.1: a draft tree holds several candidate
// tokens per position; a node may look at itself and its ancestors only).
// One wavefront per tree, one lane per node: lane i walks its parent chain.
#include "vs_internal.h"

namespace vs {

__global__ __launch_bounds__(kWave) void tree_mask_kernel(const int32_t* __restrict__ parent,
                                                          int32_t T, uint64_t* __restrict__ mask,
                                                          int32_t* __restrict__ depth,
                                                          int32_t* __restrict__ status) {
    __shared__ int32_t sp[VS_MAX_TREE];
    const int b = blockIdx.x;
    const int i = threadIdx.x;
    int32_t p = -1;
    bool bad_root = false, bad_parent = false;
    if (i < T) {
        p = parent[(int64_t)b * T + i];
        if (i == 0) bad_root = (p != -1);
        else bad_parent = (p < 0 || p >= i);
        sp[i] = p;
    }
    __syncthreads();
    const bool any_bad_root = __any(bad_root);
    const bool any_bad_parent = __any(bad_parent);
    const int32_t code = any_bad_root ? VS_STATUS_BAD_ROOT
                                      : (any_bad_parent ? VS_STATUS_BAD_PARENT : VS_STATUS_OK);
    if (i == 0 && status) status[b] = code;
    if (i >= T) return;
    uint64_t m = 0;
    int32_t dep = 0;
    if (code == VS_STATUS_OK) {
        // parent[j] < j for every j, so the walk ends at the root in at most i hops
        int32_t j = i;
        m = 1ull << j;
        while (j > 0) {
            j = sp[j];
            m |= 1ull << j;
            ++dep;
        }
    }
    mask[(int64_t)b * T + i] = m;
    depth[(int64_t)b * T + i] = dep;
}

hipError_t launch_tree_mask(const int32_t* parent, int32_t B, int32_t T, uint64_t* mask,
                            int32_t* depth, int32_t* status, hipStream_t s) {
    hipLaunchKernelGGL(tree_mask_kernel, dim3(B), dim3(kWave), 0, s, parent, T, mask, depth, status);
    return hipGetLastError();
}

} // namespace vs
