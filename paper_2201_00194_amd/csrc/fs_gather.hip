// Population compaction: carry the selected programs of one or more families over into a new
// family (features re-tiled, CSR offsets rebuilt, scores copied), all on the device.
//
// The search that feeds the cost model is evolutionary (Section 2 of the paper: candidates are
// generated, the model estimates them, the best are kept); between generations the survivors
// of the cut keep their features and their scores, so only newly generated candidates need the
// traversal kernels.  Two kernels: offsets (lengths of the kept programs, block scan, scores),
// then rows (one workgroup per output tile copies 64 rows x all features; lane = output row, so
// writes are whole 256-byte columns and reads follow the source programs' contiguous rows).
#include "fs_internal.h"

namespace fs {

constexpr int kGatherMaxSources = 8;
constexpr int kGatherThreads = 1024;

struct GatherArgs {
    const float *features[kGatherMaxSources];
    const int32_t *prog_off[kGatherMaxSources];
    const float *score[kGatherMaxSources];
    int32_t first_prog[kGatherMaxSources + 1];   // programs of source s are first_prog[s]..first_prog[s+1]-1
    int32_t n_sources;
    int32_t n_features;
    const int32_t *keep;
    int32_t n_keep;
    float *out_features;
    int64_t out_row_capacity;
    int32_t *out_prog_off;
    float *out_score;
    int32_t *status;
};

__device__ __forceinline__ int source_of(const GatherArgs &a, int p)
{
    int s = 0;
    while (s + 1 < a.n_sources && p >= a.first_prog[s + 1])
        ++s;
    return s;
}

// out_prog_off = exclusive scan of the kept programs' lengths; scores copied.  One workgroup.
__global__ void __launch_bounds__(kGatherThreads)
gather_offsets_kernel(GatherArgs a)
{
    __shared__ long long s_sum[kGatherThreads];
    __shared__ int s_bad;
    const int tid = threadIdx.x;
    if (tid == 0)
        s_bad = 0;
    __syncthreads();
    const int per = (a.n_keep + kGatherThreads - 1) / kGatherThreads;
    const int i0 = min(tid * per, a.n_keep), i1 = min(i0 + per, a.n_keep);
    const int total_prog = a.first_prog[a.n_sources];
    long long mine = 0;
    for (int i = i0; i < i1; ++i) {
        const int p = a.keep[i];
        int len = 0;
        float sc = -__builtin_inff();
        if (p >= 0 && p < total_prog) {
            const int s = source_of(a, p), q = p - a.first_prog[s];
            len = a.prog_off[s][q + 1] - a.prog_off[s][q];
            if (a.score[s])
                sc = a.score[s][q];
        } else if (p != -1) {
            s_bad = 1;                               // -1 is the cut's padding: an empty program
        }
        if (a.out_score)
            a.out_score[i] = sc;
        mine += len;
    }
    s_sum[tid] = mine;
    __syncthreads();
    for (int off = 1; off < kGatherThreads; off <<= 1) {
        long long v = 0;
        if (tid >= off)
            v = s_sum[tid - off];
        __syncthreads();
        s_sum[tid] += v;
        __syncthreads();
    }
    long long at = s_sum[tid] - mine;
    const long long total = s_sum[kGatherThreads - 1];
    const bool fits = total <= a.out_row_capacity && total < ((long long)1 << 31);
    for (int i = i0; i < i1; ++i) {
        a.out_prog_off[i] = fits ? (int32_t)at : 0;
        const int p = a.keep[i];
        if (p >= 0 && p < total_prog) {
            const int s = source_of(a, p), q = p - a.first_prog[s];
            at += a.prog_off[s][q + 1] - a.prog_off[s][q];
        }
    }
    if (tid == 0) {
        a.out_prog_off[a.n_keep] = fits ? (int32_t)total : 0;
        *a.status = s_bad ? 2 : (fits ? 0 : 1);
    }
}

// One workgroup per output tile: 64 rows x all features.
__global__ void __launch_bounds__(256)
gather_rows_kernel(GatherArgs a)
{
    const int n_rows = a.out_prog_off[a.n_keep];
    const int r0 = blockIdx.x * 64;
    if (r0 >= n_rows)
        return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = r0 + lane;
    const int F = a.n_features;
    const float *src = nullptr;
    if (r < n_rows) {
        int lo = 0, hi = a.n_keep - 1;              // the kept program that owns output row r
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (a.out_prog_off[mid] <= r)
                lo = mid;
            else
                hi = mid - 1;
        }
        const int p = a.keep[lo];
        const int s = source_of(a, p), q = p - a.first_prog[s];
        const int64_t sr = (int64_t)a.prog_off[s][q] + (r - a.out_prog_off[lo]);
        src = a.features[s] + (sr >> 6) * F * 64 + (sr & 63);
    }
    float *dst = a.out_features + (int64_t)blockIdx.x * F * 64 + lane;
    for (int j = wave; j < F; j += 4)
        dst[(int64_t)j * 64] = src ? src[(int64_t)j * 64] : 0.0f;
}

}  // namespace fs

using namespace fs;

extern "C" int fs_gather_programs(int32_t n_features, int32_t n_sources, const fs_gather_src *src,
                                  const int32_t *keep, int32_t n_keep, float *out_features,
                                  int64_t out_row_capacity, int32_t *out_prog_off, float *out_score,
                                  int32_t *status, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (n_features < 1 || n_features > FS_MAX_FEATURES)
        return fail(FS_EINVAL, "fs_gather_programs: n_features %d outside [1, %d]", n_features, FS_MAX_FEATURES);
    if (n_sources < 1 || n_sources > kGatherMaxSources)
        return fail(n_sources < 1 ? FS_EINVAL : FS_EUNSUPPORTED,
                    "fs_gather_programs: n_sources %d outside [1, %d]", n_sources, kGatherMaxSources);
    if (!src)
        return fail(FS_EINVAL, "fs_gather_programs: src is NULL");
    if (n_keep < 0 || n_keep > FS_MAX_TOPK)
        return fail(n_keep < 0 ? FS_EINVAL : FS_EUNSUPPORTED,
                    "fs_gather_programs: n_keep %d outside [0, %d]", n_keep, FS_MAX_TOPK);
    if (out_row_capacity < 0 || out_row_capacity >= ((int64_t)1 << 31))
        return fail(FS_EINVAL, "fs_gather_programs: out_row_capacity %lld outside [0, 2^31)",
                    (long long)out_row_capacity);
    if (!out_prog_off || !status || (n_keep > 0 && !keep) || (out_row_capacity > 0 && !out_features))
        return fail(FS_EINVAL, "fs_gather_programs: NULL buffer");
    GatherArgs a;
    int64_t first = 0;
    for (int s = 0; s < kGatherMaxSources; ++s) {
        a.features[s] = nullptr;
        a.prog_off[s] = nullptr;
        a.score[s] = nullptr;
        a.first_prog[s] = (int32_t)first;
        if (s < n_sources) {
            if (src[s].n_programs < 0)
                return fail(FS_EINVAL, "fs_gather_programs: source %d: n_programs is negative", s);
            if (src[s].n_programs > 0 && (!src[s].features || !src[s].prog_off))
                return fail(FS_EINVAL, "fs_gather_programs: source %d: NULL buffer", s);
            a.features[s] = src[s].features;
            a.prog_off[s] = src[s].prog_off;
            a.score[s] = src[s].score;
            first += src[s].n_programs;
            if (first >= ((int64_t)1 << 31))
                return fail(FS_EINVAL, "fs_gather_programs: more than 2^31 programs");
        }
    }
    a.first_prog[kGatherMaxSources] = (int32_t)first;
    for (int s = n_sources; s < kGatherMaxSources; ++s)
        a.first_prog[s] = (int32_t)first;
    a.n_sources = n_sources;
    a.n_features = n_features;
    a.keep = keep;
    a.n_keep = n_keep;
    a.out_features = out_features;
    a.out_row_capacity = out_row_capacity;
    a.out_prog_off = out_prog_off;
    a.out_score = out_score;
    a.status = status;
    prof_start(kKernPack, stream);
    hipLaunchKernelGGL(gather_offsets_kernel, dim3(1), dim3(kGatherThreads), 0, stream, a);
    const int64_t tiles = (out_row_capacity + 63) / 64;
    if (tiles > 0 && n_keep > 0)
        hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)tiles), dim3(256), 0, stream, a);
    prof_stop(stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "gather kernels launch");
    return FS_OK;
}
