// Per-family top-k: the k programs with the largest score, ordered by (score descending,
// index ascending) -- the cut that decides which candidates go on to measurement
// (Section 3.2 of the paper: sort by the estimate, keep the top k; Algorithm 1: k = g).
//
// Scores are mapped to unsigned keys whose integer order is the wanted order (-0 and +0
// share a key, NaN gets the lowest key).  One workgroup serves one request:
//   1. radix select (4 passes of 8 bits, histogram in LDS) finds the key of the k-th
//      best entry and how many entries that tie with it still fit;
//   2. an index-ordered sweep collects every entry above that key plus the lowest-index
//      ties, as 64-bit composites (key, ~index) in LDS;
//   3. a bitonic sort of the composites gives the final order; all composites differ, so
//      the result is unique.
#include "fs_internal.h"

namespace fs {

constexpr int kTopkThreads = 1024;

__device__ __forceinline__ uint32_t score_key(float s)
{
    if (s != s)
        return 0u;             // NaN: below every number
    s = s + 0.0f;              // -0 -> +0
    const uint32_t b = __float_as_uint(s);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Exclusive prefix count of `flag` over the block in thread order; `total` gets the sum.
// `wave_cnt` is LDS scratch of 16 ints.  Contains block barriers.
__device__ __forceinline__ int block_prefix_count(bool flag, int *wave_cnt, int &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long b = __ballot(flag);
    const int before = __popcll(b & ((1ull << lane) - 1ull));
    __syncthreads();
    if (lane == 0)
        wave_cnt[wave] = __popcll(b);
    __syncthreads();
    int base = 0, sum = 0;
    for (int w = 0; w < kTopkThreads / 64; ++w) {
        const int c = wave_cnt[w];
        if (w < wave)
            base += c;
        sum += c;
    }
    total = sum;
    return base + before;
}

__global__ void __launch_bounds__(kTopkThreads)
topk_kernel(const TopkDesc *__restrict__ descs)
{
    extern __shared__ unsigned long long cand[];   // [kpow2] then small scratch
    const TopkDesc d = descs[blockIdx.x];
    const int n = d.n, k = d.k;
    const int kk = min(n, k);
    const int tid = threadIdx.x;
    const float *__restrict__ score = d.score;

    for (int j = kk + tid; j < k; j += kTopkThreads) {
        d.out_idx[j] = -1;
        if (d.out_score)
            d.out_score[j] = -__builtin_inff();
    }
    if (kk == 0)
        return;
    int kpow2 = 1;
    while (kpow2 < kk)
        kpow2 <<= 1;
    int *hist = (int *)(cand + kpow2);    // 256 ints
    int *wave_cnt = hist + 256;           // 16 ints
    int *sel = wave_cnt + 16;             // [0] digit, [1] remaining need

    // ---- 1. key of the kk-th best entry ----
    uint32_t prefix = 0, mask = 0;
    int need = kk;
    if (kk < n) {
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256)
                hist[tid] = 0;
            __syncthreads();
            int run_digit = -1, run = 0;
            for (int i = tid; i < n; i += kTopkThreads) {
                const uint32_t key = score_key(score[i]);
                if ((key & mask) == prefix) {
                    const int dg = (key >> shift) & 255;
                    if (dg != run_digit) {
                        if (run)
                            atomicAdd(&hist[run_digit], run);
                        run_digit = dg;
                        run = 0;
                    }
                    ++run;
                }
            }
            if (run)
                atomicAdd(&hist[run_digit], run);
            __syncthreads();
            if (tid == 0) {
                int above = 0, dg = 255;
                for (; dg > 0; --dg) {
                    if (above + hist[dg] >= need)
                        break;
                    above += hist[dg];
                }
                sel[0] = dg;
                sel[1] = need - above;
            }
            __syncthreads();
            prefix |= (uint32_t)sel[0] << shift;
            mask |= 255u << shift;
            need = sel[1];
            __syncthreads();
        }
    } else {
        need = n;   // take everything; every key is >= 0
    }
    const uint32_t tau = prefix;
    const int need_eq = need;

    // ---- 2. collect, in index order ----
    int gt_done = 0, eq_done = 0;
    for (int base = 0; base < n; base += kTopkThreads) {
        const int i = base + tid;
        uint32_t key = 0;
        bool gt = false, eq = false;
        if (i < n) {
            key = score_key(score[i]);
            gt = key > tau;
            eq = key == tau;
        }
        int tot_gt, tot_eq;
        const int r_gt = block_prefix_count(gt, wave_cnt, tot_gt);
        const int r_eq = block_prefix_count(eq, wave_cnt, tot_eq);
        const unsigned long long comp =
            ((unsigned long long)key << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)i);
        if (gt)
            cand[gt_done + r_gt] = comp;                    // fewer than kk of these exist
        else if (eq && eq_done + r_eq < need_eq)
            cand[kk - 1 - (eq_done + r_eq)] = comp;
        gt_done += tot_gt;
        eq_done += tot_eq;
    }
    for (int j = kk + tid; j < kpow2; j += kTopkThreads)
        cand[j] = 0ull;                                     // below every real composite
    __syncthreads();

    // ---- 3. bitonic sort, descending ----
    for (int size = 2; size <= kpow2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = tid; t < (kpow2 >> 1); t += kTopkThreads) {
                const int lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                const int hi = lo | stride;
                const bool desc = (lo & size) == 0;
                const unsigned long long a = cand[lo], b = cand[hi];
                if ((a < b) == desc) {
                    cand[lo] = b;
                    cand[hi] = a;
                }
            }
            __syncthreads();
        }
    }
    for (int j = tid; j < kk; j += kTopkThreads) {
        const uint32_t idx = 0xFFFFFFFFu - (uint32_t)(cand[j] & 0xFFFFFFFFull);
        d.out_idx[j] = (int32_t)idx;
        if (d.out_score)
            d.out_score[j] = score[idx];
    }
}

int launch_topk(const TopkDesc *d_desc, int n_requests, int max_k, hipStream_t stream)
{
    int kpow2 = 1;
    while (kpow2 < max_k)
        kpow2 <<= 1;
    const size_t lds = (size_t)kpow2 * 8 + (256 + 16 + 2) * sizeof(int);
    static size_t configured[16] = {0};
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    if (lds > 65536 && (dev < 0 || dev >= 16 || configured[dev] < lds)) {
        FS_HIP(hipFuncSetAttribute((const void *)topk_kernel,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        if (dev >= 0 && dev < 16)
            configured[dev] = lds;
    }
    hipLaunchKernelGGL(topk_kernel, dim3(n_requests), dim3(kTopkThreads), lds, stream, d_desc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "topk_kernel launch");
    return FS_OK;
}

}  // namespace fs
