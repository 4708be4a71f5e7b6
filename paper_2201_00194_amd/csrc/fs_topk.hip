// Per-family top-k: the k programs with the largest score, ordered by (score descending,
// index ascending) -- the cut that decides which candidates go on to measurement
// (Section 3.2 of the paper: sort by the estimate, keep the top k; Algorithm 1: k = g).
//
// Scores are mapped to unsigned keys whose integer order is the wanted order (-0 and +0
// share a key, NaN gets the lowest key).  One workgroup serves one request:
//   1. radix select (4 passes of 8 bits, histogram in LDS) finds the key of the k-th
//      best entry and how many entries that tie with it still fit;
//   2. every wavefront owns a contiguous slice of the scores; it counts the entries above
//      that key and the ties in its slice, the counts are scanned, and a second sweep places
//      every entry above the key plus the lowest-index ties as 64-bit composites
//      (key, ~index) in LDS;
//   3. a bitonic sort of the composites gives the final order; all composites differ, so
//      the result is unique.
// A long request (>= 8192 entries) is cut into up to 16 slices, one workgroup each, which
// leave their best k composites in scratch, best first; a second kernel merges the slices'
// lists pairwise in LDS, keeping the best k of every pair, and writes the answer.  The union
// of the slices' best k holds the request's best k, and composites order the same way
// everywhere, so nothing changes in the result.  Cuts wider than 4096 do not fit that merge:
// they are cut into slices of about 2048 entries (up to 128) whose sorted lists are merged
// pairwise in global memory, level by level, each merge keeping the best k.
#include <cstring>
#include <mutex>

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

constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kTopkUnroll = 8;     // loads in flight per thread

// Keys of kTopkUnroll consecutive 64-element pieces starting at `base`, this lane's element of
// each; pieces past `end` read a clamped address and are flagged invalid by the caller.
__device__ __forceinline__ void load_keys(const float *__restrict__ score, int base, int end,
                                          int lane, uint32_t (&key)[kTopkUnroll])
{
    float v[kTopkUnroll];
#pragma unroll
    for (int u = 0; u < kTopkUnroll; ++u)
        v[u] = score[min(base + u * 64 + lane, end - 1)];
#pragma unroll
    for (int u = 0; u < kTopkUnroll; ++u)
        key[u] = score_key(v[u]);
}

__global__ void __launch_bounds__(kTopkThreads)
topk_kernel(const TopkDesc *__restrict__ descs)
{
    extern __shared__ unsigned long long cand[];   // [kpow2] then small scratch
    const TopkDesc d = descs[blockIdx.x];
    const int n = d.sub_end - d.sub_begin, k = d.k;   // this workgroup's entries
    const int kk = min(n, k);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *__restrict__ score = d.score + d.sub_begin;
    const uint32_t idx0 = (uint32_t)d.sub_begin;

    if (d.comp_out) {
        if (d.comp_pad)
            for (int j = kk + tid; j < k; j += kTopkThreads)
                d.comp_out[j] = 0ull;
    } else {
        for (int j = kk + tid; j < k; j += kTopkThreads) {
            d.out_idx[j] = -1;
            if (d.out_score)
                d.out_score[j] = -__builtin_inff();
        }
    }
    if (kk == 0)
        return;
    int kpow2 = 2;                        // at least 2: keeps the histogram 16-byte aligned
    while (kpow2 < kk)
        kpow2 <<= 1;
    int *hist = (int *)(cand + kpow2);    // 256 ints
    int *wave_cnt = hist + 256;           // 2 x 16 ints: per-wavefront counts (above, equal)
    int *sel = wave_cnt + 2 * kTopkWaves; // [0] digit, [1] remaining need

    // Every wavefront owns a contiguous, 64-aligned slice of the scores: slices in wavefront
    // order are the scores in index order.
    const int per_wave = (((n + kTopkWaves - 1) / kTopkWaves) + 63) & ~63;
    const int w_begin = min(wave * per_wave, n), w_end = min(w_begin + per_wave, n);

    // A wavefront whose slice is a single round of loads (requests of up to 8192 entries)
    // fetches its keys once and keeps them in registers for all six sweeps below.
    const bool cached = per_wave <= 64 * kTopkUnroll;
    uint32_t key[kTopkUnroll];
    if (cached && w_begin < w_end)
        load_keys(score, w_begin, w_end, lane, key);

    // ---- 1. key of the kk-th best entry ----
    uint32_t prefix = 0, mask = 0;
    int need = kk;
    if (kk < n) {
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256)
                hist[tid] = 0;
            __syncthreads();
            int run_digit = -1, run = 0;
            for (int base = w_begin; base < w_end; base += 64 * kTopkUnroll) {
                if (!cached)
                    load_keys(score, base, w_end, lane, key);
#pragma unroll
                for (int u = 0; u < kTopkUnroll; ++u) {
                    const bool valid = base + u * 64 + lane < w_end;
                    if (valid && (key[u] & mask) == prefix) {
                        const int dg = (key[u] >> shift) & 255;
                        if (dg != run_digit) {
                            if (run)
                                atomicAdd(&hist[run_digit], run);
                            run_digit = dg;
                            run = 0;
                        }
                        ++run;
                    }
                }
            }
            if (run)
                atomicAdd(&hist[run_digit], run);
            __syncthreads();
            if (wave == 0) {
                // The digit whose bin holds the need-th best entry: lane l owns bins 4l..4l+3,
                // a suffix sum over the lanes gives the entries in higher bins.
                const int4 c = *(const int4 *)&hist[4 * lane];
                const int total = c.x + c.y + c.z + c.w;
                int suffix = total;                       // inclusive: lanes >= this one
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const int v = __shfl_down(suffix, off);
                    if (lane + off < 64)
                        suffix += v;
                }
                int above = suffix - total;
                const int cnt[4] = {c.w, c.z, c.y, c.x};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (above < need && above + cnt[j] >= need) {
                        sel[0] = 4 * lane + 3 - j;
                        sel[1] = need - above;
                    }
                    above += cnt[j];
                }
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

    // ---- 2. collect, in index order: count per wavefront, scan, then place ----
    int my_gt = 0, my_eq = 0;
    for (int base = w_begin; base < w_end; base += 64 * kTopkUnroll) {
        if (!cached)
            load_keys(score, base, w_end, lane, key);
#pragma unroll
        for (int u = 0; u < kTopkUnroll; ++u) {
            const bool valid = base + u * 64 + lane < w_end;
            my_gt += __popcll(__ballot(valid && key[u] > tau));
            my_eq += __popcll(__ballot(valid && key[u] == tau));
        }
    }
    if (lane == 0) {
        wave_cnt[wave] = my_gt;
        wave_cnt[kTopkWaves + wave] = my_eq;
    }
    __syncthreads();
    int gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) {
        gt_before += wave_cnt[w];
        eq_before += wave_cnt[kTopkWaves + w];
    }
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int base = w_begin; base < w_end; base += 64 * kTopkUnroll) {
        if (!cached)
            load_keys(score, base, w_end, lane, key);
#pragma unroll
        for (int u = 0; u < kTopkUnroll; ++u) {
            const int i = base + u * 64 + lane;
            const bool valid = i < w_end;
            const bool gt = valid && key[u] > tau, eq = valid && key[u] == tau;
            const unsigned long long bg = __ballot(gt), be = __ballot(eq);
            const unsigned long long comp =
                ((unsigned long long)key[u] << 32) |
                (unsigned long long)(0xFFFFFFFFu - (idx0 + (uint32_t)i));
            if (gt) {
                cand[gt_before + __popcll(bg & below)] = comp;       // fewer than kk of these exist
            } else if (eq) {
                const int rank = eq_before + __popcll(be & below);   // index order among the ties
                if (rank < need_eq)
                    cand[kk - 1 - rank] = comp;
            }
            gt_before += __popcll(bg);
            eq_before += __popcll(be);
        }
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
    if (d.comp_out) {
        for (int j = tid; j < kk; j += kTopkThreads)
            d.comp_out[j] = cand[j];
        return;
    }
    for (int j = tid; j < kk; j += kTopkThreads) {
        const uint32_t idx = 0xFFFFFFFFu - (uint32_t)(cand[j] & 0xFFFFFFFFull);
        d.out_idx[j] = (int32_t)idx;
        if (d.out_score)
            d.out_score[j] = d.score[idx];
    }
}

// Second stage: the slices' sorted candidate lists into LDS (each padded to kp = 2^q >= k
// entries), then a tree of pairwise merges that each keep only the better kp entries:
// max(A[i], B[kp-1-i]) holds the best kp of two descending lists as a bitonic sequence, and
// q compare-exchange rounds sort it.  What is left in list 0 is the answer.
__global__ void __launch_bounds__(kTopkThreads)
topk_merge_kernel(const TopkMergeDesc *__restrict__ descs)
{
    extern __shared__ unsigned long long cand[];
    const TopkMergeDesc d = descs[blockIdx.x];
    const int tid = threadIdx.x;
    const int k = d.k, lists = d.n_comp / k;
    int q = 0;
    while ((1 << q) < k)
        ++q;
    const int kp = 1 << q;
    for (int j = tid; j < lists * kp; j += kTopkThreads) {
        const int l = j >> q, i = j & (kp - 1);
        cand[j] = i < k ? d.comp_in[l * k + i] : 0ull;
    }
    __syncthreads();
    for (int step = 1; step < lists; step <<= 1) {
        const int groups = (lists + 2 * step - 1) / (2 * step);
        for (int t = tid; t < groups * kp; t += kTopkThreads) {
            const int a = (t >> q) * 2 * step, i = t & (kp - 1);
            if (a + step < lists) {
                const unsigned long long x = cand[a * kp + i], y = cand[(a + step) * kp + kp - 1 - i];
                if (x < y)
                    cand[a * kp + i] = y;
            }
        }
        __syncthreads();
        for (int stride = kp >> 1; stride > 0; stride >>= 1) {
            for (int t = tid; t < groups * (kp >> 1); t += kTopkThreads) {
                const int a = (t >> (q - 1)) * 2 * step, u = t & ((kp >> 1) - 1);
                if (a + step < lists) {
                    const int lo = a * kp + (((u & ~(stride - 1)) << 1) | (u & (stride - 1)));
                    const int hi = lo + stride;
                    const unsigned long long x = cand[lo], y = cand[hi];
                    if (x < y) {
                        cand[lo] = y;
                        cand[hi] = x;
                    }
                }
            }
            __syncthreads();
        }
    }
    const int kk = min(d.n, k);
    for (int j = tid; j < k; j += kTopkThreads) {
        if (j < kk) {
            const uint32_t idx = 0xFFFFFFFFu - (uint32_t)(cand[j] & 0xFFFFFFFFull);
            d.out_idx[j] = (int32_t)idx;
            if (d.out_score)
                d.out_score[j] = d.score[idx];
        } else {
            d.out_idx[j] = -1;
            if (d.out_score)
                d.out_score[j] = -__builtin_inff();
        }
    }
}

// Merge of two descending lists of composites that live in global memory, for cuts too wide
// for the LDS merge.  All composites differ, so an entry's place in the merged list is its own
// position plus the number of entries of the other list that exceed it: one thread per entry
// finds that count by bisection and stores the entry if its place is among the best `lo`.
// blockIdx.y names the pair, blockIdx.x a run of kTopkThreads entries of (a then b).
__global__ void __launch_bounds__(kTopkThreads)
topk_pair_kernel(const TopkPairDesc *__restrict__ descs)
{
    const TopkPairDesc d = descs[blockIdx.y];
    const int e = blockIdx.x * kTopkThreads + threadIdx.x;
    if (e < d.la + d.lb) {
        const bool in_a = e < d.la;
        const unsigned long long *__restrict__ self = in_a ? d.a : d.b;
        const unsigned long long *__restrict__ other = in_a ? d.b : d.a;
        const int me = in_a ? e : e - d.la;
        if (me < d.lo) {
            const unsigned long long v = self[me];
            // entries of `other` above v, counted no further than would push v out of the cut
            int lo = 0, hi = min(in_a ? d.lb : d.la, d.lo - me);
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (other[mid] > v)
                    lo = mid + 1;
                else
                    hi = mid;
            }
            const int p = me + lo;
            if (p < d.lo) {
                if (d.out) {
                    d.out[p] = v;
                } else {
                    const uint32_t idx = 0xFFFFFFFFu - (uint32_t)(v & 0xFFFFFFFFull);
                    d.out_idx[p] = (int32_t)idx;
                    if (d.out_score)
                        d.out_score[p] = d.score[idx];
                }
            }
        }
    }
    if (!d.out && blockIdx.x == 0) {
        for (int p = d.lo + threadIdx.x; p < d.k; p += kTopkThreads) {
            d.out_idx[p] = -1;
            if (d.out_score)
                d.out_score[p] = -__builtin_inff();
        }
    }
}

int launch_topk_pairs(const TopkPairDesc *d_desc, int n_pairs, int max_entries, hipStream_t stream)
{
    const int runs = max_entries > 0 ? (max_entries + kTopkThreads - 1) / kTopkThreads : 1;
    constexpr int kMaxY = 32768;             // pairs per launch (grid.y)
    for (int at = 0; at < n_pairs; at += kMaxY) {
        const int cnt = n_pairs - at < kMaxY ? n_pairs - at : kMaxY;
        hipLaunchKernelGGL(topk_pair_kernel, dim3(runs, cnt), dim3(kTopkThreads), 0, stream, d_desc + at);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return fail_hip(e, "topk_pair_kernel launch");
    }
    return FS_OK;
}

int launch_topk_merge(const TopkMergeDesc *d_desc, int n_requests, int max_padded, hipStream_t stream)
{
    if (max_padded > kTopkMergeCap)
        return fail(FS_EUNSUPPORTED, "top-k merge of %d candidates exceeds %d", max_padded, kTopkMergeCap);
    const size_t lds = (size_t)max_padded * 8;
    static size_t configured[16] = {0};
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    if (lds > 65536 && (dev < 0 || dev >= 16 || configured[dev] < lds)) {
        FS_HIP(hipFuncSetAttribute((const void *)topk_merge_kernel,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        if (dev >= 0 && dev < 16)
            configured[dev] = lds;
    }
    hipLaunchKernelGGL(topk_merge_kernel, dim3(n_requests), dim3(kTopkThreads), lds, stream, d_desc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "topk_merge_kernel launch");
    return FS_OK;
}

int launch_topk(const TopkDesc *d_desc, int n_requests, int max_k, hipStream_t stream)
{
    int kpow2 = 2;
    while (kpow2 < max_k)
        kpow2 <<= 1;
    const size_t lds = (size_t)kpow2 * 8 + (256 + 2 * (kTopkThreads / 64) + 2) * sizeof(int);
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

// ---- fs_topk_noalloc: the same cut for callers that cannot allocate -----------------------------
// Descriptors and the slices' candidate lists live in a fixed device array instead of grown
// library scratch; the descriptors travel as a kernel argument (no staging buffer, no copy).
constexpr size_t kNoAllocBytes = 1u << 20;        // the whole array
constexpr size_t kNoAllocDescBytes = 3584;        // its head: descriptors (one kernel argument)
static __device__ __align__(256) unsigned char scratch[kNoAllocBytes];

struct DescBlob {
    uint32_t words[kNoAllocDescBytes / 4];
};

__global__ void __launch_bounds__(256)
topk_store_desc_kernel(DescBlob blob, uint32_t *dst, int n_words)
{
    for (int i = threadIdx.x; i < n_words; i += blockDim.x)
        dst[i] = blob.words[i];
}

static std::mutex g_noalloc_mu;
static unsigned char *g_noalloc_ptr[16] = {};     // device address of `scratch`, per device

}  // namespace fs

using namespace fs;

extern "C" int fs_topk_noalloc(int32_t n_requests, const fs_topk_req *reqs, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (n_requests < 0)
        return fail(FS_EINVAL, "fs_topk_noalloc: n_requests %d is negative", n_requests);
    if (n_requests == 0)
        return FS_OK;
    if (!reqs)
        return fail(FS_EINVAL, "fs_topk_noalloc: reqs is NULL");
    size_t n_blocks = 0, n_merge = 0, comp_total = 0;
    int max_k = 0, max_comp = 0;
    for (int i = 0; i < n_requests; ++i) {
        const fs_topk_req &r = reqs[i];
        if (r.n < 0 || r.k < 0)
            return fail(FS_EINVAL, "fs_topk_noalloc: request %d: n=%d k=%d must be non-negative", i, r.n, r.k);
        if (r.k > FS_MAX_TOPK)
            return fail(FS_EUNSUPPORTED, "fs_topk_noalloc: request %d: k=%d exceeds FS_MAX_TOPK=%d", i,
                        r.k, FS_MAX_TOPK);
        if (r.n > 0 && !r.score)
            return fail(FS_EINVAL, "fs_topk_noalloc: request %d: score is NULL", i);
        if (r.k > 0 && !r.out_idx)
            return fail(FS_EINVAL, "fs_topk_noalloc: request %d: out_idx is NULL", i);
        const TopkPlan p = topk_plan(r.n, r.k);
        if (p.mode == 2)
            return fail(FS_EUNSUPPORTED, "fs_topk_noalloc: request %d: cuts wider than 4096 of %d or "
                        "more entries are not served without allocation (use fs_topk)", i, kTopkSliceMin);
        n_blocks += (size_t)p.s;
        if (p.mode == 1) {
            ++n_merge;
            comp_total += (size_t)p.s * (size_t)r.k;
            int kp = 1;
            while (kp < r.k)
                kp <<= 1;
            if (p.s * kp > max_comp)
                max_comp = p.s * kp;
        }
        if (r.k > max_k)
            max_k = r.k;
    }
    if (max_k == 0)
        return FS_OK;
    const size_t merge_off = (sizeof(TopkDesc) * n_blocks + 15) & ~(size_t)15;
    const size_t desc_bytes = merge_off + sizeof(TopkMergeDesc) * n_merge;
    if (desc_bytes > kNoAllocDescBytes)
        return fail(FS_EUNSUPPORTED, "fs_topk_noalloc: %zu workgroups and %zu merges need %zu bytes of "
                    "descriptors, the limit is %zu (about 60 workgroups)", n_blocks, n_merge, desc_bytes,
                    kNoAllocDescBytes);
    if (comp_total * 8 > kNoAllocBytes - kNoAllocDescBytes)
        return fail(FS_EUNSUPPORTED, "fs_topk_noalloc: the sliced requests need %zu bytes of candidate "
                    "lists, the limit is %zu", comp_total * 8, kNoAllocBytes - kNoAllocDescBytes);

    std::lock_guard<std::mutex> lock(g_noalloc_mu);
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 16)
        return fail(FS_EUNSUPPORTED, "device ordinal %d not supported", dev);
    if (!g_noalloc_ptr[dev]) {
        // every device holds its own copy of the array, at its own address
        void *ptr = nullptr;
        FS_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr)
            return fail(FS_EDEVICE, "fs_topk_noalloc: no device address for the scratch array");
        g_noalloc_ptr[dev] = (unsigned char *)ptr;
    }
    unsigned char *base = g_noalloc_ptr[dev];

    DescBlob blob;
    memset(&blob, 0, sizeof(blob));
    TopkDesc *h = (TopkDesc *)blob.words;
    TopkMergeDesc *hm = (TopkMergeDesc *)((unsigned char *)blob.words + merge_off);
    unsigned long long *comp = (unsigned long long *)(base + kNoAllocDescBytes);
    size_t b = 0, m = 0;
    for (int i = 0; i < n_requests; ++i) {
        const fs_topk_req &r = reqs[i];
        const TopkPlan p = topk_plan(r.n, r.k);
        for (int j = 0; j < p.s; ++j, ++b) {
            h[b].score = r.score;
            h[b].out_idx = r.out_idx;
            h[b].out_score = r.out_score;
            h[b].n = r.n;
            h[b].k = r.k;
            const long long lo = (long long)j * p.per, hi = lo + p.per;
            h[b].sub_begin = (int32_t)(lo < r.n ? lo : r.n);
            h[b].sub_end = (int32_t)(hi < r.n ? hi : r.n);
            h[b].comp_pad = p.mode == 1 ? 1 : 0;
            h[b].pad = 0;
            h[b].comp_out = p.mode == 1 ? comp + (size_t)j * (size_t)r.k : nullptr;
        }
        if (p.mode == 1) {
            hm[m].comp_in = comp;
            hm[m].score = r.score;
            hm[m].out_idx = r.out_idx;
            hm[m].out_score = r.out_score;
            hm[m].n_comp = p.s * r.k;
            hm[m].n = r.n;
            hm[m].k = r.k;
            hm[m].pad = 0;
            comp += (size_t)p.s * (size_t)r.k;
            ++m;
        }
    }
    // Nothing in the array has to start at zero: every workgroup writes its whole list (padding
    // included) before the merge reads it, and the descriptors are rewritten by every call.
    hipLaunchKernelGGL(topk_store_desc_kernel, dim3(1), dim3(256), 0, stream, blob, (uint32_t *)base,
                       (int)((desc_bytes + 3) / 4));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "topk_store_desc_kernel launch");
    prof_start(kKernTopk, stream);
    int rc = launch_topk((const TopkDesc *)base, (int)n_blocks, max_k, stream);
    if (rc == FS_OK && n_merge)
        rc = launch_topk_merge((const TopkMergeDesc *)(base + merge_off), (int)n_merge, max_comp, stream);
    prof_stop(stream);
    return rc;
}
