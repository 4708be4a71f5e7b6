// Reference device traversal: nodes and features straight from global memory.
//
// One thread owns one statement row and walks every tree of its family's model
// (Section 4.2 of the paper: the family's cost model estimates each candidate); the row
// score is bias + leaf values added in tree order.  Handles any model the ABI accepts and
// both feature layouts; it is the path for models that the LDS-staged kernels do not take.
#include "fs_internal.h"

namespace fs {

__device__ __forceinline__ int find_family_by_block(const FamDesc *descs, int n, int block,
                                                    int32_t FamDesc::*first)
{
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (descs[mid].*first <= block)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

__global__ void __launch_bounds__(kTravRowsPerBlock)
traverse_global_kernel(const FamDesc *__restrict__ descs, int n_families)
{
    const int f = find_family_by_block(descs, n_families, blockIdx.x, &FamDesc::trav_block0);
    const FamDesc d = descs[f];
    const int r = (blockIdx.x - d.trav_block0) * kTravRowsPerBlock + threadIdx.x;
    if (r >= d.n_rows)
        return;
    const float *x;
    int64_t stride;
    if (d.layout == FS_COLBLOCK64) {
        x = d.features + (int64_t)(r >> 6) * d.n_features * 64 + (r & 63);
        stride = 64;
    } else {
        x = d.features + (int64_t)r * d.n_features;
        stride = 1;
    }
    float acc = d.bias;
    for (int t = 0; t < d.n_trees; ++t) {
        const int root = d.tree_off[t];
        int n = root;
        GNode nd = d.nodes[n];
        while (nd.y >= 0) {
            const float v = x[(int64_t)nd.y * stride];
            n = (v < __int_as_float(nd.x)) ? nd.z : nd.w;
            nd = d.nodes[n];
        }
        acc = acc + __int_as_float(nd.x);
        if (d.leaf_idx)
            d.leaf_idx[(int64_t)r * d.n_trees + t] = (uint16_t)(n - root);
    }
    d.row_score[r] = acc;
}

int launch_traverse_global(const FamDesc *d_desc, int n_families, int total_blocks,
                           hipStream_t stream)
{
    hipLaunchKernelGGL(traverse_global_kernel, dim3(total_blocks), dim3(kTravRowsPerBlock), 0,
                       stream, d_desc, n_families);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "traverse_global_kernel launch");
    return FS_OK;
}

}  // namespace fs
