// Row-major -> 64-row column-blocked re-tiling of a feature matrix.
//
// A block takes 64 rows x up to 128 columns: it reads row segments with consecutive lanes
// on consecutive columns, parks them in LDS with one float of padding per row, and writes
// each column's 64 row values as one contiguous 256-byte run.
#include "fs_internal.h"

namespace fs {

constexpr int kPackCols = 128;

__global__ void __launch_bounds__(256)
pack_colblock64_kernel(const float *__restrict__ in, int n_rows, int n_features,
                       float *__restrict__ out)
{
    __shared__ float tile[64][kPackCols + 1];
    const int tile_id = blockIdx.x;
    const int c0 = blockIdx.y * kPackCols;
    const int nc = min(kPackCols, n_features - c0);
    const int r0 = tile_id * 64;
    for (int e = threadIdx.x; e < 64 * kPackCols; e += 256) {
        const int r = e / kPackCols, c = e % kPackCols;
        float v = 0.0f;
        if (c < nc && r0 + r < n_rows)
            v = in[(int64_t)(r0 + r) * n_features + c0 + c];
        tile[r][c] = v;
    }
    __syncthreads();
    float *o = out + (int64_t)tile_id * n_features * 64;
    for (int e = threadIdx.x; e < 64 * nc; e += 256) {
        const int c = e >> 6, r = e & 63;
        o[(int64_t)(c0 + c) * 64 + r] = tile[r][c];
    }
}

// The same re-tiling for every row-major family of a scoring call, one launch: block ->
// (family, tile, column block) through the families' block prefix.
__global__ void __launch_bounds__(256)
retile_kernel(const FamDesc *__restrict__ descs, int n_families)
{
    __shared__ float tile[64][kPackCols + 1];
    int lo = 0, hi = n_families - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (descs[mid].retile_block0 <= (int)blockIdx.x)
            lo = mid;
        else
            hi = mid - 1;
    }
    const FamDesc &d = descs[lo];
    const int local = blockIdx.x - d.retile_block0;
    const int tile_id = local / d.retile_colblocks;
    const int c0 = (local - tile_id * d.retile_colblocks) * kPackCols;
    const int n_features = d.n_features, n_rows = d.n_rows;
    const int nc = min(kPackCols, n_features - c0);
    const int r0 = tile_id * 64;
    const float *__restrict__ in = d.rowmajor_src;
    for (int e = threadIdx.x; e < 64 * kPackCols; e += 256) {
        const int r = e / kPackCols, c = e % kPackCols;
        float v = 0.0f;
        if (c < nc && r0 + r < n_rows)
            v = in[(int64_t)(r0 + r) * n_features + c0 + c];
        tile[r][c] = v;
    }
    __syncthreads();
    float *o = const_cast<float *>(d.features) + (int64_t)tile_id * n_features * 64;
    for (int e = threadIdx.x; e < 64 * nc; e += 256) {
        const int c = e >> 6, r = e & 63;
        o[(int64_t)(c0 + c) * 64 + r] = tile[r][c];
    }
}

int launch_retile(const FamDesc *d_desc, int n_families, int total_blocks, hipStream_t stream)
{
    hipLaunchKernelGGL(retile_kernel, dim3(total_blocks), dim3(256), 0, stream, d_desc, n_families);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "retile_kernel launch");
    return FS_OK;
}

int launch_pack_colblock64(const float *in, int64_t n_rows, int32_t n_features, float *out,
                           hipStream_t stream)
{
    const int tiles = (int)((n_rows + 63) / 64);
    const int col_blocks = (n_features + kPackCols - 1) / kPackCols;
    hipLaunchKernelGGL(pack_colblock64_kernel, dim3(tiles, col_blocks), dim3(256), 0, stream, in,
                       (int)n_rows, n_features, out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "pack_colblock64_kernel launch");
    return FS_OK;
}

}  // namespace fs
