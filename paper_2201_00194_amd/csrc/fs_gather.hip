// Population compaction: carry the selected programs of one or more families over into a new
// family (features re-tiled, CSR offsets rebuilt, scores copied), all on the device.
//
// The search that feeds the cost model is evolutionary (Section 2 of the paper: candidates are
// generated, the model estimates them, the best are kept); between generations the survivors
// of the cut keep their features and their scores, so only newly generated candidates need the
// traversal kernels.  Three kernels: lengths of the kept programs and their scores, offsets
// (block scan of the lengths), then rows (one workgroup per output tile copies 64 rows x all
// features; lane = output row, so writes are whole 256-byte columns and reads follow the source
// programs' contiguous rows).
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

// Lengths of the kept programs into out_prog_off (-1 marks an index that is neither a program
// nor the cut's padding), scores copied.  The kept indices are in score order, i.e. scattered
// over the sources, so this part runs on many compute units.
__global__ void __launch_bounds__(256)
gather_lengths_kernel(GatherArgs a)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= a.n_keep)
        return;
    const int total_prog = a.first_prog[a.n_sources];
    const int p = a.keep[i];
    int len = 0;
    float sc = -__builtin_inff();
    if (p >= 0 && p < total_prog) {
        const int s = source_of(a, p), q = p - a.first_prog[s];
        len = a.prog_off[s][q + 1] - a.prog_off[s][q];
        if (a.score[s])
            sc = a.score[s][q];
    } else if (p != -1) {
        len = -1;                                    // -1 is the cut's padding: an empty program
    }
    a.out_prog_off[i] = len;
    if (a.out_score)
        a.out_score[i] = sc;
}

constexpr int kGatherPer = (FS_MAX_TOPK + kGatherThreads - 1) / kGatherThreads;   // kept programs per thread

// out_prog_off: lengths -> their exclusive scan.  One workgroup; thread t holds entries
// t, t + 1024, ... in registers (coalesced loads, all in flight at once).  Every run of 64
// entries is scanned inside its wavefront with shuffles, the 16 x 16 run totals are scanned by
// four wavefronts, and each entry's offset is its run's base plus its place in the run.
constexpr int kGatherWaves = kGatherThreads / 64;
constexpr int kGatherRuns = kGatherPer * kGatherWaves;       // 64-entry runs, in index order

__device__ __forceinline__ long long wave_inclusive_scan(long long v, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const long long t = __shfl_up(v, off);
        if (lane >= off)
            v += t;
    }
    return v;
}

__global__ void __launch_bounds__(kGatherThreads)
gather_offsets_kernel(GatherArgs a)
{
    static_assert(kGatherRuns == 256, "the run totals are scanned by four wavefronts");
    __shared__ long long s_run[kGatherRuns];         // totals of the runs, then their exclusive scan
    __shared__ long long s_quarter[4];
    __shared__ int s_bad;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0)
        s_bad = 0;
    __syncthreads();
    int len[kGatherPer];
#pragma unroll
    for (int u = 0; u < kGatherPer; ++u) {
        const int i = tid + u * kGatherThreads;
        len[u] = i < a.n_keep ? a.out_prog_off[i] : 0;
    }
    bool bad = false;
    long long incl[kGatherPer];
#pragma unroll
    for (int u = 0; u < kGatherPer; ++u) {
        bad |= len[u] < 0;
        len[u] = len[u] < 0 ? 0 : len[u];
        incl[u] = wave_inclusive_scan((long long)len[u], lane);
        if (lane == 63)
            s_run[u * kGatherWaves + wave] = incl[u];    // run (u, wave) covers entries u*1024 + wave*64 ...
    }
    if (bad)
        s_bad = 1;
    __syncthreads();
    long long run_incl = 0, run_total = 0;
    if (tid < kGatherRuns) {
        run_total = s_run[tid];
        run_incl = wave_inclusive_scan(run_total, lane);
        if (lane == 63)
            s_quarter[wave] = run_incl;
    }
    __syncthreads();
    if (tid < kGatherRuns) {
        long long before = 0;
        for (int w = 0; w < wave; ++w)
            before += s_quarter[w];
        s_run[tid] = before + run_incl - run_total;       // rows before this run
    }
    __syncthreads();
    const long long total = s_quarter[0] + s_quarter[1] + s_quarter[2] + s_quarter[3];
    const bool fits = total <= a.out_row_capacity && total < ((long long)1 << 31);
#pragma unroll
    for (int u = 0; u < kGatherPer; ++u) {
        const int i = tid + u * kGatherThreads;
        if (i < a.n_keep)
            a.out_prog_off[i] = fits ? (int32_t)(s_run[u * kGatherWaves + wave] + incl[u] - len[u]) : 0;
    }
    if (tid == 0) {
        a.out_prog_off[a.n_keep] = fits ? (int32_t)total : 0;
        *a.status = s_bad ? 2 : (fits ? 0 : 1);
    }
}

// One workgroup per output tile: 64 rows x all features.  A thread's loads are issued in
// batches before the stores that depend on them, so that the copy is not one round trip to
// memory per column.
constexpr int kGatherBatch = 8;

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
    const float *__restrict__ src = nullptr;
    if (r < n_rows) {
        // The kept program that owns output row r: the last index whose offset is <= r.  Rows
        // are spread about evenly over the programs, so the search starts from the proportional
        // guess and gallops away from it; equal-length programs need two probes.
        const int32_t *__restrict__ off = a.out_prog_off;
        int lo = 0, hi = a.n_keep - 1;
        const int g = min((int)(((int64_t)r * a.n_keep) / n_rows), hi);
        if (off[g] <= r) {
            lo = g;
            int step = 1;
            while (lo + step <= hi && off[lo + step] <= r) {
                lo += step;
                step <<= 1;
            }
            hi = min(hi, lo + step - 1);
        } else {                                    // g >= 1: off[0] = 0 <= r
            hi = g - 1;
            int c = hi, step = 1;
            while (c > 0 && off[c] > r) {
                hi = c - 1;
                c = max(c - step, 0);
                step <<= 1;
            }
            lo = c;
        }
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
    float *__restrict__ dst = a.out_features + (int64_t)blockIdx.x * F * 64 + lane;
    for (int j0 = wave; j0 < F; j0 += 4 * kGatherBatch) {
        float v[kGatherBatch];
#pragma unroll
        for (int u = 0; u < kGatherBatch; ++u) {
            const int j = j0 + 4 * u;
            v[u] = (src && j < F) ? src[(int64_t)j * 64] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < kGatherBatch; ++u) {
            const int j = j0 + 4 * u;
            if (j < F)
                dst[(int64_t)j * 64] = v[u];
        }
    }
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
    if (n_keep > 0)
        hipLaunchKernelGGL(gather_lengths_kernel, dim3((unsigned)((n_keep + 255) / 256)), dim3(256), 0, stream, a);
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
