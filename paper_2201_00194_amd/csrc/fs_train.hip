// Training of family cost models: histogram boosting rounds on the device.
//
// After every tuning step the tuner retrains the family's model on the measured candidates
// (Algorithm 1 of the paper, train_cost_model; Section 4.3 moves this to the GPU).  The
// arithmetic is stated in familyseer_train.h.  What makes it reproducible bit for bit is that
// every sum over rows is an integer sum (gradients in fixed point, curvature = rows of the
// program), so the atomics below may land in any order; gains and leaf values are evaluated
// in double from those integers in one fixed order of operations.
//
// Per round and family (all families of a batch share every launch; nothing returns to the
// host between rounds):
//   begin_tree   clear the heap of the tree to grow
//   grad         per program: s_p (row order), g_p, q_p; rows get (q_p, rows of p) and go
//                back to the root; the root's (G, H) are added up on the way
//   per level:   hist (LDS histograms per family, four features and up to 16 nodes; a
//                feature's most frequent bin is never counted, it is the node's total minus
//                the rest; with one slab of rows per family the same workgroup then finds the
//                best cut of each (node, feature), else the slabs add into a global buffer and
//                `split` searches there), pick (per node: best feature, split or leaf, child
//                ids in breadth-first order), part (rows of split nodes move to a child)
//   deep trees:  before level 5 the rows are regrouped once by their node (seg_*), so that
//                deeper histogram passes read only the segments of their nodes' ancestors
//   pick         once more at max_depth: what is left becomes leaves
//   update       row output += value of the row's leaf;  emit: heap -> flat model arrays
#include <math.h>
#include <stdlib.h>
#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "familyseer_train.h"
#include "fs_internal.h"
#include "fs_lds.h"

namespace fs {

constexpr int kHeapNodes = (1 << (FS_TRAIN_MAX_DEPTH + 1)) - 1;   // 2047
constexpr int kBins = FS_TRAIN_MAX_CUTS + 1;                      // 256
constexpr int kHistThreads = 1024;
constexpr int kHistRowsPerSlab = 65536;

// Deep trees: from this level on a histogram pass covers a small share of the nodes, and
// streaming all rows for every pass is what the time goes into.  Before that level's histograms
// the rows are regrouped once by their node of the level; the rows of a node's descendants stay
// inside its segment, so a pass over some nodes of a deeper level reads only the segments of
// their ancestors on this level.
constexpr int kSortLevel = 5;
constexpr int kSortSegs = 1 << kSortLevel;             // 32 nodes, heap indices 31..62
constexpr int kSortMinDepth = 7;                       // worth it when at least two levels use it

// heap node states
enum { kAbsent = 0, kOpen = 1, kInternal = 2, kLeaf = 3 };

struct TrainDesc {
    const uint8_t *bins;       // [feature / 4][r_pad][4]: the bins of four consecutive features
                               // of a row share one 32-bit word
    const int32_t *prog_off;
    const float *target;
    const int32_t *cut_off;    // device copies of the cut lists
    const float *cuts;
    const int32_t *hot_bin;    // per feature: its most frequent bin, which no histogram counts
                               // (it is the node's total minus the other bins)
    float *row_pred;
    float *prog_pred;
    int2 *qh;                  // per row: (gradient in fixed point, curvature)
    uint16_t *node_of_row;     // heap index of the node that holds the row
    unsigned long long *hist;  // [slot][feature][bin][2]: (G, H) of the level in work
    int32_t *h_state, *h_feat, *h_cut, *h_id;
    float *h_thr, *h_val;
    long long *h_G, *h_H;
    double *best_gain;         // [slot][feature]
    int32_t *best_cut;
    long long *best_GL, *best_HL;
    int32_t *counters;         // [0] next node id of the tree in work, [1] trees, [2] nodes
    unsigned long long *abs_q; // sum over the rows of |gradient| (fixed point) of the round in work
    int32_t *pk_feat, *pk_cut; // per node of a level: its best feature and cut (levels with many nodes)
    double *pk_gain;
    // Rows regrouped by their node of level kSortLevel (deep trees only, see train_seg_* below):
    uint8_t *s_bins;           // bins in that order, same layout as `bins`
    int2 *s_qh;
    int32_t *s_rowid;          // original row of a regrouped position
    uint16_t *s_node;          // node that holds it (kept up to date below kSortLevel)
    int32_t *s_dest;           // scratch: regrouped position of an original row, -1 if it stayed behind
    int32_t *seg_start;        // kSortSegs + 1: first position of every node of level kSortLevel
    int32_t *seg_cursor;       // kSortSegs: counts, then fill positions
    int32_t *m_tree_off, *m_feat, *m_left, *m_right;
    float *m_thr, *m_val;
    int64_t r_pad;
    int32_t n_features, n_rows, n_programs;
    float bias;
};

struct Params {
    double eta, lambda, min_gain, inv_scale;
    long long mcw;
    float grad_scale;
    int max_depth;
};

// ---- set-up kernels ----------------------------------------------------------------------

// bin = number of cuts <= x; NaN takes the last bin.  One block column per feature.
__global__ void __launch_bounds__(256)
train_bin_kernel(const float *__restrict__ x, int layout, int n_features, int n_rows,
                 int64_t r_pad, const int32_t *__restrict__ cut_off,
                 const float *__restrict__ cuts, uint8_t *__restrict__ bins)
{
    __shared__ float c[kBins];
    const int f = blockIdx.y;
    const int m = cut_off[f + 1] - cut_off[f];
    for (int i = threadIdx.x; i < m; i += blockDim.x)
        c[i] = cuts[cut_off[f] + i];
    __syncthreads();
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rows)
        return;
    const float v = layout == FS_COLBLOCK64
                        ? x[(int64_t)(r >> 6) * n_features * 64 + (int64_t)f * 64 + (r & 63)]
                        : x[(int64_t)r * n_features + f];
    int lo = 0, hi = m;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (c[mid] <= v)
            lo = mid + 1;
        else
            hi = mid;
    }
    if (v != v)
        lo = m;
    bins[((int64_t)(f >> 2) * r_pad + r) * 4 + (f & 3)] = (uint8_t)lo;
}

// The most frequent bin of every feature over the whole training set (lowest on ties).
__global__ void __launch_bounds__(256)
train_hot_bin_kernel(const uint8_t *__restrict__ bins, int n_rows, int64_t r_pad,
                     int32_t *__restrict__ hot_bin)
{
    __shared__ unsigned int cnt[kBins];
    __shared__ unsigned int s_best[kBins];
    __shared__ int s_arg[kBins];
    const int f = blockIdx.x, t = threadIdx.x;
    cnt[t] = 0u;
    __syncthreads();
    for (int r = t; r < n_rows; r += blockDim.x)
        atomicAdd(&cnt[bins[((int64_t)(f >> 2) * r_pad + r) * 4 + (f & 3)]], 1u);
    __syncthreads();
    s_best[t] = cnt[t];
    s_arg[t] = t;
    __syncthreads();
    for (int off = kBins / 2; off > 0; off >>= 1) {
        if (t < off) {
            const unsigned int a = s_best[t], b = s_best[t + off];
            if (b > a || (b == a && s_arg[t + off] < s_arg[t])) {
                s_best[t] = b;
                s_arg[t] = s_arg[t + off];
            }
        }
        __syncthreads();
    }
    if (t == 0)
        hot_bin[f] = s_arg[0];
}

// Rows of the longest program (sizes the curvature sums).
__global__ void __launch_bounds__(256)
train_max_len_kernel(const int32_t *__restrict__ prog_off, int n_programs, int32_t *__restrict__ out)
{
    int m = 0;
    for (int p = blockIdx.x * blockDim.x + threadIdx.x; p < n_programs; p += gridDim.x * blockDim.x)
        m = max(m, prog_off[p + 1] - prog_off[p]);
    for (int off = 32; off > 0; off >>= 1)
        m = max(m, __shfl_down(m, off));
    if ((threadIdx.x & 63) == 0)
        atomicMax(out, m);
}

__global__ void train_fill_kernel(float *p, int64_t n, float v)
{
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

// ---- per-round kernels -------------------------------------------------------------------

__global__ void __launch_bounds__(512)
train_begin_tree_kernel(const TrainDesc *__restrict__ descs)
{
    const TrainDesc &d = descs[blockIdx.x];
    for (int i = threadIdx.x; i < kHeapNodes; i += blockDim.x) {
        d.h_state[i] = i == 0 ? kOpen : kAbsent;
        d.h_G[i] = 0;
        d.h_H[i] = 0;
        d.h_id[i] = 0;
        d.h_val[i] = 0.0f;
    }
    if (threadIdx.x == 0) {
        d.counters[0] = 1;
        *d.abs_q = 0ull;
    }
    if (d.seg_cursor && threadIdx.x < kSortSegs)
        d.seg_cursor[threadIdx.x] = 0;
}

__device__ __forceinline__ int quantize(float g, float grad_scale)
{
    float t = g * grad_scale;
    t = fmaxf(t, -2147483520.0f);
    t = fminf(t, 2147483520.0f);
    return (int)rintf(t);
}

// One thread per program.  `with_grad` = false only refreshes prog_pred.
__global__ void __launch_bounds__(256)
train_grad_kernel(const TrainDesc *__restrict__ descs, float grad_scale, int with_grad)
{
    const TrainDesc &d = descs[blockIdx.y];
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    long long G = 0, H = 0;
    unsigned long long A = 0;                        // |gradient| x rows: bounds every histogram sum
    if (p < d.n_programs) {
        const int b = d.prog_off[p], e = d.prog_off[p + 1];
        float s = 0.0f;
        for (int r = b; r < e; ++r)
            s = s + d.row_pred[r];
        d.prog_pred[p] = s;
        if (with_grad) {
            const int q = quantize(s - d.target[p], grad_scale);
            const int len = e - b;
            for (int r = b; r < e; ++r) {
                d.qh[r] = make_int2(q, len);
                d.node_of_row[r] = 0;
            }
            G = (long long)q * len;
            H = (long long)len * len;
            A = (unsigned long long)(G < 0 ? -G : G);
        }
    }
    if (!with_grad)
        return;
    // root totals: wavefront sum, one atomic per wavefront
    for (int off = 32; off > 0; off >>= 1) {
        G += __shfl_down(G, off);
        H += __shfl_down(H, off);
        A += __shfl_down(A, off);
    }
    if ((threadIdx.x & 63) == 0 && H != 0) {
        atomicAdd((unsigned long long *)&d.h_G[0], (unsigned long long)G);
        atomicAdd((unsigned long long *)&d.h_H[0], (unsigned long long)H);
        atomicAdd(d.abs_q, A);
    }
}

// The node's own term of the gain, g*g/(H+lambda): the same for every cut of the node, so it is
// divided once per (node, feature) and not once per cut.
__device__ __forceinline__ double parent_term(long long G, long long H, double inv_scale, double lambda)
{
    const double g = (double)G * inv_scale;
    double t3 = g * g;
    t3 = t3 / ((double)H + lambda);
    return t3;
}

__device__ __forceinline__ double split_gain(long long GL, long long HL, long long G, long long H,
                                             double inv_scale, double lambda, double t3)
{
    const long long GR = G - GL, HR = H - HL;
    const double gl = (double)GL * inv_scale, gr = (double)GR * inv_scale;
    double t1 = gl * gl;
    t1 = t1 / ((double)HL + lambda);
    double t2 = gr * gr;
    t2 = t2 / ((double)HR + lambda);
    return (t1 + t2) - t3;
}

// Cross-lane steps of the cut search as DPP moves (register to register, no trip through the
// LDS crossbar as with __shfl): CTRL 0x110 + n = the lane n places down in its row of 16,
// 0x142 / 0x143 = last lane of the previous row / of the first two rows, for the rows named in
// ROW_MASK.  A lane without a source gets 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ long long dpp_ll(long long v)
{
    const int lo = dpp_i<CTRL, ROW_MASK>((int)v), hi = dpp_i<CTRL, ROW_MASK>((int)(v >> 32));
    return (long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned long long)(unsigned)lo);
}

// Inclusive prefix sum over the 64 lanes: four doubling steps inside the rows of 16, then the
// total of row 0 (2) goes to row 1 (3), then the total of the first 32 lanes to the last 32.
__device__ __forceinline__ long long wave_prefix_ll(long long v)
{
    v += dpp_ll<0x111, 0xf>(v);
    v += dpp_ll<0x112, 0xf>(v);
    v += dpp_ll<0x114, 0xf>(v);
    v += dpp_ll<0x118, 0xf>(v);
    v += dpp_ll<0x142, 0xa>(v);
    v += dpp_ll<0x143, 0xc>(v);
    return v;
}

__device__ __forceinline__ long long lane63_ll(long long v)
{
    const int lo = __builtin_amdgcn_readlane((int)v, 63), hi = __builtin_amdgcn_readlane((int)(v >> 32), 63);
    return (long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned long long)(unsigned)lo);
}

// One step of the arg-max over the lanes (largest gain, lowest cut on ties; cut 0 = nothing):
// the lane takes the other lane's pair if that is better.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void best_step(double &best, int &best_cut)
{
    const long long bits = __double_as_longlong(best);
    const double og = __longlong_as_double(dpp_ll<CTRL, ROW_MASK>(bits));
    const int oc = dpp_i<CTRL, ROW_MASK>(best_cut);
    if (oc != 0 && (best_cut == 0 || og > best || (og == best && oc < best_cut))) {
        best = og;
        best_cut = oc;
    }
}

// Best cut of feature f for the open node `node`, by one wavefront: lane l holds bins 4l..4l+3
// (g, h; the feature's most frequent bin holds 0 and is rebuilt here from the node's totals)
// and forms the left sums of the cuts 4l+1..4l+4.  Lane 0 writes the result for
// `pair` = slot * F + f.
//
// A cut behind an empty bin splits the node exactly as the cut before it does: same gain, and
// coming later it never wins.  (A row's curvature is at least 1, so a bin is empty exactly when
// its H is 0.)  Deep in a tree a node holds fewer rows than a feature has bins and most cuts
// drop out this way; when at most 64 are left they are handed out one per lane through
// `scratch` (kCutScratchBytes of LDS that only this wavefront touches), so that the wavefront pays for one
// round of double-precision divisions instead of four.  Measured: the cut search is two thirds
// of the histogram kernel's time at depth 10.
constexpr int kCutScratchBytes = 64 * (8 + 8 + 4);

__device__ __forceinline__ void wave_best_cut(const TrainDesc &d, const Params &prm, int node, int f,
                                              int pair, int lane, long long (&g)[4], long long (&h)[4],
                                              unsigned char *scratch)
{
    const long long G = d.h_G[node], H = d.h_H[node];
    const int hot = d.hot_bin[f];
    // inclusive prefix sums over the 256 bins, the hot bin still at 0
    const long long lane_g = g[0] + g[1] + g[2] + g[3], lane_h = h[0] + h[1] + h[2] + h[3];
    const long long pg = wave_prefix_ll(lane_g), ph = wave_prefix_ll(lane_h);
    // what the counted bins lack of the node's totals sits in the hot bin
    const long long hot_g = G - lane63_ll(pg), hot_h = H - lane63_ll(ph);
    long long before_g = pg - lane_g, before_h = ph - lane_h;
    if ((hot >> 2) < lane) {
        before_g += hot_g;
        before_h += hot_h;
    }
    if ((hot >> 2) == lane) {
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if ((hot & 3) == k) {
                g[k] = hot_g;
                h[k] = hot_h;
            }
    }
    bool filled[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        filled[k] = h[k] != 0;
#pragma unroll
    for (int k = 1; k < 4; ++k) {
        g[k] += g[k - 1];
        h[k] += h[k - 1];
    }
    const int m = d.cut_off[f + 1] - d.cut_off[f];
    const double t3 = parent_term(G, H, prm.inv_scale, prm.lambda);
    // cut 4l+k+1 (left = bins 0..4l+k) is worth evaluating if it is in range, follows a
    // non-empty bin and leaves enough curvature on both sides
    bool cand[4];
    unsigned long long vote[4];
    int n_cand = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const long long HL = before_h + h[k];
        cand[k] = 4 * lane + k + 1 <= m && filled[k] && HL >= prm.mcw && H - HL >= prm.mcw;
        vote[k] = __ballot(cand[k]);
        n_cand += __popcll(vote[k]);
    }
    int cut = 0;
    double gain = 0.0;
    long long bGL = 0, bHL = 0;
    if (n_cand <= 64) {
        // one candidate per lane (which lane takes which does not matter: ties are settled on
        // the cut number below)
        long long *s_GL = (long long *)scratch;
        long long *s_HL = s_GL + 64;
        int *s_cut = (int *)(s_HL + 64);
        const unsigned long long below = (1ull << lane) - 1ull;
        int first = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (cand[k]) {
                const int at = first + __popcll(vote[k] & below);
                s_GL[at] = before_g + g[k];
                s_HL[at] = before_h + h[k];
                s_cut[at] = 4 * lane + k + 1;
            }
            first += __popcll(vote[k]);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (lane < n_cand) {
            bGL = s_GL[lane];
            bHL = s_HL[lane];
            cut = s_cut[lane];
            gain = split_gain(bGL, bHL, G, H, prm.inv_scale, prm.lambda, t3);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();                         // the next search of this wavefront reuses the scratch
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (cand[k]) {
                const long long GL = before_g + g[k], HL = before_h + h[k];
                const double gn = split_gain(GL, HL, G, H, prm.inv_scale, prm.lambda, t3);
                if (cut == 0 || gn > gain) {                     // ascending cuts: first of equals stays
                    gain = gn;
                    cut = 4 * lane + k + 1;
                    bGL = GL;
                    bHL = HL;
                }
            }
        }
    }
    double best = gain;
    int best_cut = cut;
    // largest gain, lowest cut on ties: the same steps as the prefix sum leave the best of all
    // lanes in lane 63
    best_step<0x111, 0xf>(best, best_cut);
    best_step<0x112, 0xf>(best, best_cut);
    best_step<0x114, 0xf>(best, best_cut);
    best_step<0x118, 0xf>(best, best_cut);
    best_step<0x142, 0xa>(best, best_cut);
    best_step<0x143, 0xc>(best, best_cut);
    best_cut = __builtin_amdgcn_readlane(best_cut, 63);
    if (best_cut == 0) {
        if (lane == 0) {
            d.best_gain[pair] = 0.0;
            d.best_cut[pair] = 0;
            d.best_GL[pair] = 0;
            d.best_HL[pair] = 0;
        }
    } else if (cut == best_cut) {                                // exactly one lane holds the winner
        d.best_gain[pair] = gain;
        d.best_cut[pair] = cut;
        d.best_GL[pair] = bGL;
        d.best_HL[pair] = bHL;
    }
}

// Histograms of one level.  A workgroup takes a slab of rows, four consecutive features (one
// 32-bit word of bins per row) and a run of nodes of the level, and keeps their (G, H)
// histograms in LDS.  blockIdx = (slab, feature group, trainer * passes + pass); a pass covers
// consecutive nodes.  With one slab per family the workgroup holds the complete histograms and
// searches the cuts itself; with more slabs the partial histograms are added to the global
// buffer (which is all zero: the split kernel clears what it reads) and train_split_kernel
// does the search.
//
// Two forms of a bin in LDS.  Packed: one 64-bit word G * 2^hb + H, fed by one atomic per
// (row, feature); hb bits hold any curvature sum of the slab (the host knows rows x longest
// program) and the rest holds G as long as the sum of |gradient| over the trainer's rows,
// which train_grad_kernel leaves in abs_q, stays below 2^(63-hb).  Wide: G and H in 64 bits
// each, always safe; a workgroup launched for the packed form falls back to it, its nodes in
// two halves, when the gradients of its trainer are too large.  Both are exact integer sums.
constexpr int kHistFeats = 4;           // features per workgroup: one 32-bit word of bins per row
constexpr int kHistSlotsWide = 8;       // 8 nodes x 4 features x 256 bins x 16 B = 128 KB
constexpr int kHistSlotsPacked = 16;    // 16 nodes x 4 features x 256 bins x 8 B = 128 KB
// Behind the histograms: where the adds of rows that do not count land (rows past the end, of
// other nodes, or in the feature's most frequent bin), one word per lane and feature, so that
// the row loop has no branches.
constexpr int kHistTrashWords = (kHistFeats - 1) * kBins + 64;
static_assert(kBins * 8 >= kCutScratchBytes, "the cut search borrows its pair's own histogram");

// One run of `slots` nodes, the first being number `abs0` of its level (heap index node0).
template <bool PACKED>
__device__ __forceinline__ void hist_run(const TrainDesc &d, const Params &prm,
                                         unsigned long long *lds_hist, int node0, int abs0, int slots,
                                         int row0, int row1, int f0, int nf, const int (&hot)[kHistFeats],
                                         const uint32_t *__restrict__ words,
                                         const uint16_t *__restrict__ node_of,
                                         const int2 *__restrict__ qh_of, int n_slabs, int hb)
{
    const int pairs = slots * kHistFeats;
    unsigned long long *lds_h = lds_hist + pairs * kBins;       // wide form only
    for (int i = threadIdx.x; i < pairs * kBins * (PACKED ? 1 : 2); i += kHistThreads)
        lds_hist[i] = 0ull;
    __syncthreads();
    // Rows in batches of kUnroll per thread.  The loads of the next batch are issued before the
    // atomics of the current one, so that their latency passes while the LDS works.  (Indices
    // are clamped to the last row: a batch past the end loads that row again and counts nothing.)
    // The loop is bound by instruction issue, so it is kept free of branches: an add that does
    // not count goes to the lane's own trash word instead.
    constexpr int kUnroll = 4;
    const int trash = pairs * kBins * (PACKED ? 1 : 2) + (threadIdx.x & 63);
    int slot[kUnroll];
    uint32_t w[kUnroll];                                         // the row's bins of the four features
    int2 qh[kUnroll];
    // (global address space stated: plain pointers make flat loads, which also count as LDS
    // traffic and would make every wait for them a wait for the atomics too)
    auto g_node = FS_GLOBAL(const uint16_t, node_of);
    auto g_words = FS_GLOBAL(const uint32_t, words);
    auto g_qh = FS_GLOBAL(const int2, qh_of);
    auto fetch = [&](int base, int (&sl)[kUnroll], uint32_t (&ww)[kUnroll], int2 (&q)[kUnroll]) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t r = (uint32_t)min(base + u * kHistThreads, row1 - 1);   // 32-bit offsets from uniform bases
            sl[u] = (int)g_node[r] - node0;
            ww[u] = g_words[r];
            q[u] = g_qh[r];
        }
    };
    if (row0 < row1)
        fetch(row0 + threadIdx.x, slot, w, qh);
    for (int base = row0 + threadIdx.x; base < row1; base += kHistThreads * kUnroll) {
        int n_slot[kUnroll];
        uint32_t n_w[kUnroll];
        int2 n_qh[kUnroll];
        fetch(base + kHistThreads * kUnroll, n_slot, n_w, n_qh);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const bool counts = base + u * kHistThreads < row1 && (unsigned)slot[u] < (unsigned)slots;
            const unsigned long long both =
                (unsigned long long)((long long)qh[u].x * ((long long)1 << hb) + (long long)qh[u].y);
            const int row_at = slot[u] * (kHistFeats * kBins);
#pragma unroll
            for (int fi = 0; fi < kHistFeats; ++fi) {
                const int b = (w[u] >> (8 * fi)) & 255;
                // (a feature past the family's last has hot = 256 and its bins are 0: harmless)
                // (mask arithmetic, not a conditional: the compiler turns that into a branch)
                const int take = -(int)(counts & (b != hot[fi]));
                const int at = trash + ((row_at + b - trash) & take) + fi * kBins;
                if (PACKED) {
                    atomicAdd(&lds_hist[at], both);
                } else {
                    atomicAdd(&lds_hist[at], (unsigned long long)(long long)qh[u].x);
                    atomicAdd(&lds_hist[at + (at >= trash ? 0 : pairs * kBins)], (unsigned long long)qh[u].y);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            slot[u] = n_slot[u];
            w[u] = n_w[u];
            qh[u] = n_qh[u];
        }
    }
    __syncthreads();
    const long long h_mask = ((long long)1 << hb) - 1;
    auto bin_at = [&](int i, long long &g, long long &h) {
        if (PACKED) {
            const long long v = (long long)lds_hist[i];
            h = v & h_mask;
            g = (v - h) >> hb;                                   // v - h is a multiple of 2^hb
        } else {
            g = (long long)lds_hist[i];
            h = (long long)lds_h[i];
        }
    };
    if (n_slabs == 1) {
        // The whole histogram of these nodes and features is here: search the cuts right away
        // (one wavefront per (node, feature)); nothing goes through the global buffer.
        const int lane = threadIdx.x & 63;
        for (int pair = threadIdx.x >> 6; pair < pairs; pair += kHistThreads / 64) {
            const int slot = pair / kHistFeats, fi = pair % kHistFeats;
            const int node = node0 + slot;
            if (fi >= nf || d.h_state[node] != kOpen)
                continue;
            long long g[4], h[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                bin_at(pair * kBins + 4 * lane + k, g[k], h[k]);
            // The pair's bins are in registers now and no other wavefront reads them: their LDS
            // serves as the search's scratch (a wavefront's LDS accesses complete in order).
            wave_best_cut(d, prm, node, f0 + fi, (abs0 + slot) * d.n_features + f0 + fi, lane, g, h,
                          (unsigned char *)(lds_hist + pair * kBins));
        }
    } else {
        for (int i = threadIdx.x; i < pairs * kBins; i += kHistThreads) {
            const int pair = i / kBins, b = i - pair * kBins;
            const int slot = pair / kHistFeats, fi = pair % kHistFeats;
            long long g, h;
            bin_at(i, g, h);
            if (fi >= nf || h == 0)
                continue;
            const int64_t at = (((int64_t)(abs0 + slot) * d.n_features + (f0 + fi)) * kBins + b) * 2;
            atomicAdd(&d.hist[at], (unsigned long long)g);
            atomicAdd(&d.hist[at + 1], (unsigned long long)h);
        }
    }
    __syncthreads();                                             // LDS may be reused by the next run
}

template <bool PACKED>
__global__ void __launch_bounds__(kHistThreads)
train_hist_kernel(const TrainDesc *__restrict__ descs, int level, int passes, int rows_per_slab,
                  int n_slabs, int hb, int sorted, Params prm)
{
    extern __shared__ unsigned long long lds_hist[];
    const TrainDesc &d = descs[blockIdx.z / passes];
    const int pass = blockIdx.z % passes;
    int row0 = blockIdx.x * rows_per_slab;
    const int f0 = blockIdx.y * kHistFeats;
    if (row0 >= d.n_rows || f0 >= d.n_features)
        return;
    int row1 = min(row0 + rows_per_slab, d.n_rows);
    const int nf = min(kHistFeats, d.n_features - f0);
    const int n_slots = 1 << level;
    const int slots = min(PACKED ? kHistSlotsPacked : kHistSlotsWide, n_slots);
    const int abs0 = pass * slots;                               // first node of the pass, within the level
    const int node0 = n_slots - 1 + abs0;                        // its heap index
    if (sorted) {
        // regrouped rows (one slab): the segments of this pass's ancestors on level kSortLevel
        const int up = level - kSortLevel;
        row0 = d.seg_start[abs0 >> up];
        row1 = d.seg_start[((abs0 + slots - 1) >> up) + 1];
    }
    int hot[kHistFeats];
#pragma unroll
    for (int fi = 0; fi < kHistFeats; ++fi)
        hot[fi] = fi < nf ? d.hot_bin[f0 + fi] : 256;           // 256: no bin, nothing is skipped
    const uint32_t *__restrict__ words =
        (const uint32_t *)(sorted ? d.s_bins : d.bins) + (int64_t)blockIdx.y * d.r_pad;
    const uint16_t *__restrict__ node_of = sorted ? d.s_node : d.node_of_row;
    const int2 *__restrict__ qh_of = sorted ? d.s_qh : d.qh;
    if (PACKED) {
        if (*d.abs_q < (1ull << (63 - hb))) {
            hist_run<true>(d, prm, lds_hist, node0, abs0, slots, row0, row1, f0, nf, hot, words, node_of, qh_of,
                           n_slabs, hb);
        } else {
            const int half = slots > 1 ? slots / 2 : 1;          // the wide form takes twice the LDS per node
            for (int s = 0; s < slots; s += half)
                hist_run<false>(d, prm, lds_hist, node0 + s, abs0 + s, half, row0, row1, f0, nf, hot, words,
                                node_of, qh_of, n_slabs, 0);
        }
    } else {
        hist_run<false>(d, prm, lds_hist, node0, abs0, slots, row0, row1, f0, nf, hot, words, node_of, qh_of,
                        n_slabs, 0);
    }
}

// Best cut of one feature for one open node.  One wavefront per (node, feature); lane l owns
// bins 4l..4l+3 and the cuts 4l+1..4l+4.  The histogram entries are zeroed once read, so that
// the buffer is all zero again for the next level.  Only used when a family's rows span
// several slabs.
constexpr int kSplitWaves = 4;

__global__ void __launch_bounds__(64 * kSplitWaves)
train_split_kernel(const TrainDesc *__restrict__ descs, int level, Params prm)
{
    __shared__ __align__(8) unsigned char s_cut_scratch[kSplitWaves][kCutScratchBytes];
    const TrainDesc &d = descs[blockIdx.z];
    const int lane = threadIdx.x & 63;
    const int pair = blockIdx.x * kSplitWaves + (threadIdx.x >> 6);
    const int n_slots = 1 << level;
    if (pair >= n_slots * d.n_features)
        return;
    const int slot = pair / d.n_features, f = pair - slot * d.n_features;
    const int node = n_slots - 1 + slot;
    if (d.h_state[node] != kOpen)
        return;
    typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));
    u64x2 *hp = (u64x2 *)(d.hist + ((int64_t)pair * kBins + 4 * lane) * 2);
    long long g[4], h[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const u64x2 v = hp[k];
        g[k] = (long long)v.x;
        h[k] = (long long)v.y;
        hp[k] = (u64x2){0ull, 0ull};
    }
    wave_best_cut(d, prm, node, f, pair, lane, g, h, s_cut_scratch[threadIdx.x >> 6]);
}

// Per open node of the level: best feature, split or leaf; children get consecutive ids in
// slot order (breadth-first numbering).  One workgroup per trainer: first every wavefront
// finds the best feature of some of the nodes (lanes over features), then one thread per node
// decides.
constexpr int kPickThreads = 1024;
constexpr int kMaxSlots = 1 << FS_TRAIN_MAX_DEPTH;
static_assert(kMaxSlots <= kPickThreads, "one thread per node of the deepest level");
constexpr int kPickSpreadSlots = 64;     // levels with at least this many nodes reduce in a kernel of their own

// Best feature of node number `sl` of the level, by one wavefront (lanes over the features):
// largest gain, lowest feature on ties.  No candidate: feature -1.
__device__ __forceinline__ void wave_best_feature(const TrainDesc &d, int level, const Params &prm, int sl,
                                                  int lane, int &bf, int &bc, double &bg)
{
    const int n_slots = 1 << level;
    bf = -1;
    bc = 0;
    bg = 0.0;
    if (level < prm.max_depth && d.h_state[n_slots - 1 + sl] == kOpen) {
        for (int f = lane; f < d.n_features; f += 64) {          // ascending: first of equals stays
            const int64_t o = (int64_t)sl * d.n_features + f;
            const int c = d.best_cut[o];
            if (c == 0)
                continue;
            const double g = d.best_gain[o];
            if (bf < 0 || g > bg) {
                bg = g;
                bf = f;
                bc = c;
            }
        }
        for (int off = 32; off > 0; off >>= 1) {                 // largest gain, lowest feature on ties
            const double og = __shfl_xor(bg, off);
            const int of = __shfl_xor(bf, off), oc = __shfl_xor(bc, off);
            if (of >= 0 && (bf < 0 || og > bg || (og == bg && of < bf))) {
                bg = og;
                bf = of;
                bc = oc;
            }
        }
    }
}

// Levels with many nodes: the best feature of every node, one wavefront each, over the whole
// chip (train_pick_kernel, one workgroup per trainer, then only decides).
__global__ void __launch_bounds__(kPickThreads)
train_pick_reduce_kernel(const TrainDesc *__restrict__ descs, int level, Params prm)
{
    const TrainDesc &d = descs[blockIdx.y];
    const int lane = threadIdx.x & 63;
    const int sl = blockIdx.x * (kPickThreads / 64) + (threadIdx.x >> 6);
    if (sl >= (1 << level))
        return;
    int bf, bc;
    double bg;
    wave_best_feature(d, level, prm, sl, lane, bf, bc, bg);
    if (lane == 0) {
        d.pk_feat[sl] = bf;
        d.pk_cut[sl] = bc;
        d.pk_gain[sl] = bg;
    }
}

__global__ void __launch_bounds__(kPickThreads)
train_pick_kernel(const TrainDesc *__restrict__ descs, int level, int reduced, Params prm)
{
    __shared__ int s_scan[kMaxSlots];
    __shared__ int s_bf[kMaxSlots], s_bc[kMaxSlots];
    __shared__ double s_bg[kMaxSlots];
    const TrainDesc &d = descs[blockIdx.x];
    const int n_slots = 1 << level;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (reduced) {
        if ((int)threadIdx.x < n_slots) {
            s_bf[threadIdx.x] = d.pk_feat[threadIdx.x];
            s_bc[threadIdx.x] = d.pk_cut[threadIdx.x];
            s_bg[threadIdx.x] = d.pk_gain[threadIdx.x];
        }
    } else {
        for (int sl = wave; sl < n_slots; sl += kPickThreads / 64) {
            int bf, bc;
            double bg;
            wave_best_feature(d, level, prm, sl, lane, bf, bc, bg);
            if (lane == 0) {
                s_bf[sl] = bf;
                s_bc[sl] = bc;
                s_bg[sl] = bg;
            }
        }
    }
    __syncthreads();
    const int slot = threadIdx.x;
    const int node = n_slots - 1 + slot;
    const bool open = slot < n_slots && d.h_state[node] == kOpen;
    const int bf = open ? s_bf[slot] : -1, bc = open ? s_bc[slot] : 0;
    const double bg = open ? s_bg[slot] : 0.0;
    const bool split = open && bf >= 0 && bg > prm.min_gain;
    if (threadIdx.x < kMaxSlots)
        s_scan[threadIdx.x] = split ? 1 : 0;
    __syncthreads();
    for (int off = 1; off < kMaxSlots; off <<= 1) {
        int v = 0;
        if (threadIdx.x < kMaxSlots && (int)threadIdx.x >= off)
            v = s_scan[threadIdx.x - off];
        __syncthreads();
        if (threadIdx.x < kMaxSlots)
            s_scan[threadIdx.x] += v;
        __syncthreads();
    }
    const int before = threadIdx.x < kMaxSlots ? s_scan[threadIdx.x] - (split ? 1 : 0) : 0;
    const int total = s_scan[kMaxSlots - 1];
    const int next_id = d.counters[0];
    if (open) {
        const long long G = d.h_G[node], H = d.h_H[node];
        if (split) {
            const int64_t o = (int64_t)slot * d.n_features + bf;
            const long long GL = d.best_GL[o], HL = d.best_HL[o];
            const int lc = 2 * node + 1, rc = lc + 1;
            d.h_state[node] = kInternal;
            d.h_feat[node] = bf;
            d.h_cut[node] = bc;
            d.h_thr[node] = d.cuts[d.cut_off[bf] + bc - 1];
            d.h_state[lc] = kOpen;
            d.h_state[rc] = kOpen;
            d.h_G[lc] = GL;
            d.h_H[lc] = HL;
            d.h_G[rc] = G - GL;
            d.h_H[rc] = H - HL;
            d.h_id[lc] = next_id + 2 * before;
            d.h_id[rc] = next_id + 2 * before + 1;
        } else {
            const double g = (double)G * prm.inv_scale;
            d.h_state[node] = kLeaf;
            d.h_val[node] = (float)(-prm.eta * g / ((double)H + prm.lambda));
        }
    }
    __syncthreads();
    if (threadIdx.x == 0)
        d.counters[0] = next_id + 2 * total;
}

// Rows of the nodes that were split move to the left child if their bin is below the cut.
__global__ void __launch_bounds__(256)
train_part_kernel(const TrainDesc *__restrict__ descs, int level)
{
    const TrainDesc &d = descs[blockIdx.y];
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= d.n_rows)
        return;
    const int node = d.node_of_row[r];
    if (node < (1 << level) - 1 || d.h_state[node] != kInternal)
        return;
    const int f = d.h_feat[node];
    const int b = d.bins[((int64_t)(f >> 2) * d.r_pad + r) * 4 + (f & 3)];
    d.node_of_row[r] = (uint16_t)(2 * node + (b < d.h_cut[node] ? 1 : 2));
}

// The same for regrouped rows (levels from kSortLevel on): positions instead of rows.
__global__ void __launch_bounds__(256)
train_part_sorted_kernel(const TrainDesc *__restrict__ descs, int level)
{
    const TrainDesc &d = descs[blockIdx.y];
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= d.seg_start[kSortSegs])
        return;
    const int node = d.s_node[p];
    if (node < (1 << level) - 1 || d.h_state[node] != kInternal)
        return;
    const int f = d.h_feat[node];
    const int b = d.s_bins[((int64_t)(f >> 2) * d.r_pad + p) * 4 + (f & 3)];
    d.s_node[p] = (uint16_t)(2 * node + (b < d.h_cut[node] ? 1 : 2));
}

// Regrouping, step 1: rows per node of level kSortLevel (rows that stopped in a leaf above
// that level stay behind).  seg_cursor is zero when the tree begins.
__global__ void __launch_bounds__(256)
train_seg_count_kernel(const TrainDesc *__restrict__ descs)
{
    __shared__ int s_cnt[kSortSegs];
    const TrainDesc &d = descs[blockIdx.y];
    if (blockIdx.x * blockDim.x >= (unsigned)d.n_rows)
        return;
    if (threadIdx.x < kSortSegs)
        s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < d.n_rows) {
        const int seg = (int)d.node_of_row[r] - (kSortSegs - 1);
        if (seg >= 0 && seg < kSortSegs)
            atomicAdd(&s_cnt[seg], 1);
    }
    __syncthreads();
    if (threadIdx.x < kSortSegs && s_cnt[threadIdx.x] != 0)
        atomicAdd(&d.seg_cursor[threadIdx.x], s_cnt[threadIdx.x]);
}

// Step 2: seg_start = exclusive scan of the counts; seg_cursor = the same (fill positions).
__global__ void __launch_bounds__(64)
train_seg_scan_kernel(const TrainDesc *__restrict__ descs)
{
    static_assert(kSortSegs <= 64, "one wavefront scans the segments");
    const TrainDesc &d = descs[blockIdx.x];
    const int t = threadIdx.x;
    const int mine = t < kSortSegs ? d.seg_cursor[t] : 0;
    int incl = mine;
    for (int off = 1; off < 64; off <<= 1) {
        const int u = __shfl_up(incl, off);
        if (t >= off)
            incl += u;
    }
    if (t < kSortSegs) {
        d.seg_start[t] = incl - mine;
        d.seg_cursor[t] = incl - mine;
    }
    if (t == kSortSegs - 1)
        d.seg_start[kSortSegs] = incl;
}

// Step 3: a position for every row that goes on (order inside a segment is free: all sums over
// rows are integer sums); its node, gradient pair and row number move there.
__global__ void __launch_bounds__(256)
train_seg_place_kernel(const TrainDesc *__restrict__ descs)
{
    __shared__ int s_cnt[kSortSegs], s_base[kSortSegs];
    const TrainDesc &d = descs[blockIdx.y];
    if (blockIdx.x * blockDim.x >= (unsigned)d.n_rows)
        return;
    if (threadIdx.x < kSortSegs)
        s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    int seg = -1, rank = 0, node = 0;
    if (r < d.n_rows) {
        node = d.node_of_row[r];
        seg = node - (kSortSegs - 1);
        if (seg >= kSortSegs)
            seg = -1;                                            // cannot happen: no row is below this level yet
        if (seg >= 0)
            rank = atomicAdd(&s_cnt[seg], 1);
    }
    __syncthreads();
    if (threadIdx.x < kSortSegs && s_cnt[threadIdx.x] != 0)
        s_base[threadIdx.x] = atomicAdd(&d.seg_cursor[threadIdx.x], s_cnt[threadIdx.x]);
    __syncthreads();
    if (r < d.n_rows) {
        int p = -1;
        if (seg >= 0) {
            p = s_base[seg] + rank;
            d.s_rowid[p] = r;
            d.s_node[p] = (uint16_t)node;
            d.s_qh[p] = d.qh[r];
        }
        d.s_dest[r] = p;
    }
}

// Step 4: the bins follow, one 32-bit word (four features) per thread.
__global__ void __launch_bounds__(256)
train_seg_bins_kernel(const TrainDesc *__restrict__ descs)
{
    const TrainDesc &d = descs[blockIdx.z];
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= d.n_rows || (int)blockIdx.y * 4 >= d.n_features)
        return;
    const int p = d.s_dest[r];
    if (p < 0)
        return;
    const int64_t g = (int64_t)blockIdx.y * d.r_pad;
    ((uint32_t *)d.s_bins)[g + p] = ((const uint32_t *)d.bins)[g + r];
}

// Row outputs += value of the leaf that holds the row.  With regrouped rows (`sorted`), the
// rows that went on below kSortLevel are updated through their regrouped record, the others
// (in a leaf above that level) through node_of_row.
__global__ void __launch_bounds__(256)
train_update_kernel(const TrainDesc *__restrict__ descs, int sorted)
{
    const TrainDesc &d = descs[blockIdx.y];
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= d.n_rows)
        return;
    if (sorted) {
        if (r < d.seg_start[kSortSegs]) {
            const int row = d.s_rowid[r];
            d.row_pred[row] = d.row_pred[row] + d.h_val[d.s_node[r]];
        }
        const int node = d.node_of_row[r];
        if (node < kSortSegs - 1)
            d.row_pred[r] = d.row_pred[r] + d.h_val[node];
        return;
    }
    d.row_pred[r] = d.row_pred[r] + d.h_val[d.node_of_row[r]];
}

// Heap -> flat arrays, appended to the model.
__global__ void __launch_bounds__(512)
train_emit_kernel(const TrainDesc *__restrict__ descs)
{
    const TrainDesc &d = descs[blockIdx.x];
    const int n_trees = d.counters[1], base = d.counters[2], n_new = d.counters[0];
    for (int i = threadIdx.x; i < kHeapNodes; i += blockDim.x) {
        const int st = d.h_state[i];
        if (st != kInternal && st != kLeaf)
            continue;
        const int at = base + d.h_id[i];
        if (st == kInternal) {
            d.m_feat[at] = d.h_feat[i];
            d.m_thr[at] = d.h_thr[i];
            d.m_left[at] = d.h_id[2 * i + 1];
            d.m_right[at] = d.h_id[2 * i + 2];
            d.m_val[at] = 0.0f;
        } else {
            d.m_feat[at] = -1;
            d.m_thr[at] = 0.0f;
            d.m_left[at] = -1;
            d.m_right[at] = -1;
            d.m_val[at] = d.h_val[i];
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        d.counters[1] = n_trees + 1;
        d.counters[2] = base + n_new;
        d.m_tree_off[n_trees + 1] = base + n_new;
    }
}

}  // namespace fs

// ---- host side ----------------------------------------------------------------------------

struct fs_trainer {
    fs::TrainDesc h;          // host copy of the descriptor (device pointers inside)
    int device;
    int max_depth, max_trees;
    int trees_enqueued;
    int max_len;              // rows of the longest program
    std::vector<void *> allocs;
};

namespace fs {

static std::mutex g_train_mu;
struct BatchBuf {
    TrainDesc *d_desc = nullptr;
    TrainDesc *h_desc = nullptr;   // pinned
    int cap = 0;
    hipEvent_t copied = nullptr;
    bool pending = false;
};
static BatchBuf g_batch[16];

template <class T>
static int dev_alloc(fs_trainer *t, T **out, size_t count)
{
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, (count ? count : 1) * sizeof(T));
    if (e != hipSuccess)
        return e == hipErrorOutOfMemory ? fail(FS_ENOMEM, "hipMalloc of %zu bytes failed", count * sizeof(T))
                                        : fail_hip(e, "hipMalloc");
    if (t->allocs.size() == t->allocs.capacity()) {       // cannot happen with the reserve at creation
        (void)hipFree(p);
        return fail(FS_ENOMEM, "allocation table full");
    }
    t->allocs.push_back(p);
    *out = (T *)p;
    return FS_OK;
}

static int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, what);
    return FS_OK;
}

}  // namespace fs

using namespace fs;

extern "C" void fs_trainer_destroy(fs_trainer *t)
{
    if (!t)
        return;
    for (void *p : t->allocs)
        (void)hipFree(p);
    delete t;
}

extern "C" int fs_trainer_create(fs_trainer **out, int32_t n_features, const float *features,
                                 int32_t layout, int64_t n_rows, const int32_t *prog_off,
                                 int32_t n_programs, const float *target, const int32_t *cut_off,
                                 const float *cuts, float bias, int32_t max_depth, int32_t max_trees,
                                 void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (!out)
        return fail(FS_EINVAL, "fs_trainer_create: out is NULL");
    *out = nullptr;
    if (n_features < 1 || n_features > FS_MAX_FEATURES)
        return fail(FS_EINVAL, "fs_trainer_create: n_features=%d outside 1..%d", n_features, FS_MAX_FEATURES);
    if (n_rows < 1 || n_rows >= (int64_t)1 << 31 || n_programs < 1)
        return fail(FS_EINVAL, "fs_trainer_create: n_rows=%lld, n_programs=%d must be >= 1",
                    (long long)n_rows, n_programs);
    if (!features || !prog_off || !target || !cut_off || (!cuts && cut_off[n_features] > 0))
        return fail(FS_EINVAL, "fs_trainer_create: NULL argument");
    if (layout != FS_ROWMAJOR && layout != FS_COLBLOCK64)
        return fail(FS_EINVAL, "fs_trainer_create: unknown layout %d", layout);
    if (max_depth < 0 || max_depth > FS_TRAIN_MAX_DEPTH)
        return fail(FS_EUNSUPPORTED, "fs_trainer_create: max_depth=%d outside 0..%d", max_depth,
                    FS_TRAIN_MAX_DEPTH);
    if (max_trees < 1)
        return fail(FS_EINVAL, "fs_trainer_create: max_trees=%d must be >= 1", max_trees);
    if (cut_off[0] != 0)
        return fail(FS_EINVAL, "fs_trainer_create: cut_off[0] must be 0");
    for (int f = 0; f < n_features; ++f) {
        const int m = cut_off[f + 1] - cut_off[f];
        if (m < 0 || m > FS_TRAIN_MAX_CUTS)
            return fail(m < 0 ? FS_EINVAL : FS_EUNSUPPORTED,
                        "fs_trainer_create: feature %d has %d cuts (0..%d allowed)", f, m, FS_TRAIN_MAX_CUTS);
        for (int j = 0; j < m; ++j) {
            const float c = cuts[cut_off[f] + j];
            if (c != c || (j > 0 && !(cuts[cut_off[f] + j - 1] < c)))
                return fail(FS_EINVAL, "fs_trainer_create: cuts of feature %d are not ascending and distinct", f);
        }
    }
    fs_trainer *t = new (std::nothrow) fs_trainer();
    if (!t)
        return fail(FS_ENOMEM, "out of host memory");
    try {
        t->allocs.reserve(64);      // every later push_back stays within this (no throw past the C ABI)
    } catch (const std::bad_alloc &) {
        delete t;
        return fail(FS_ENOMEM, "out of host memory");
    }
    int rc = FS_OK;
    hipError_t e = hipGetDevice(&t->device);
    if (e != hipSuccess) {
        delete t;
        return fail_hip(e, "hipGetDevice");
    }
    t->max_depth = max_depth;
    t->max_trees = max_trees;
    t->trees_enqueued = 0;
    TrainDesc &h = t->h;
    h.n_features = n_features;
    h.n_rows = (int32_t)n_rows;
    h.n_programs = n_programs;
    h.bias = bias;
    h.r_pad = (n_rows + 255) & ~(int64_t)255;
    const int n_cuts = cut_off[n_features];
    const int hist_slots = max_depth > 0 ? 1 << (max_depth - 1) : 1;
    const int64_t node_cap = (int64_t)max_trees * ((1 << (max_depth + 1)) - 1);
    uint8_t *bins = nullptr;
    int32_t *d_prog_off = nullptr, *d_cut_off = nullptr;
    float *d_target = nullptr, *d_cuts = nullptr;
    int32_t *d_hot = nullptr;
#define TRY(x)            \
    if (rc == FS_OK)      \
    rc = (x)
    TRY(dev_alloc(t, &bins, (size_t)h.r_pad * 4 * (size_t)((n_features + 3) / 4)));
    TRY(dev_alloc(t, &d_prog_off, (size_t)n_programs + 1));
    TRY(dev_alloc(t, &d_target, (size_t)n_programs));
    TRY(dev_alloc(t, &d_cut_off, (size_t)n_features + 1));
    TRY(dev_alloc(t, &d_cuts, (size_t)n_cuts));
    TRY(dev_alloc(t, &d_hot, (size_t)n_features));
    TRY(dev_alloc(t, &h.row_pred, (size_t)n_rows));
    TRY(dev_alloc(t, &h.prog_pred, (size_t)n_programs));
    TRY(dev_alloc(t, &h.qh, (size_t)n_rows));
    TRY(dev_alloc(t, &h.node_of_row, (size_t)n_rows));
    h.hist = nullptr;       // only families that span several slabs need it: see ensure_hist
    TRY(dev_alloc(t, &h.h_state, (size_t)kHeapNodes));
    TRY(dev_alloc(t, &h.h_feat, (size_t)kHeapNodes));
    TRY(dev_alloc(t, &h.h_cut, (size_t)kHeapNodes));
    TRY(dev_alloc(t, &h.h_id, (size_t)kHeapNodes));
    TRY(dev_alloc(t, &h.h_thr, (size_t)kHeapNodes));
    TRY(dev_alloc(t, &h.h_val, (size_t)kHeapNodes));
    TRY(dev_alloc(t, &h.h_G, (size_t)kHeapNodes));
    TRY(dev_alloc(t, &h.h_H, (size_t)kHeapNodes));
    TRY(dev_alloc(t, &h.best_gain, (size_t)hist_slots * n_features));
    TRY(dev_alloc(t, &h.best_cut, (size_t)hist_slots * n_features));
    TRY(dev_alloc(t, &h.best_GL, (size_t)hist_slots * n_features));
    TRY(dev_alloc(t, &h.best_HL, (size_t)hist_slots * n_features));
    TRY(dev_alloc(t, &h.counters, (size_t)4));
    TRY(dev_alloc(t, &h.abs_q, (size_t)1));
    TRY(dev_alloc(t, &h.pk_feat, (size_t)kMaxSlots));
    TRY(dev_alloc(t, &h.pk_cut, (size_t)kMaxSlots));
    TRY(dev_alloc(t, &h.pk_gain, (size_t)kMaxSlots));
    TRY(dev_alloc(t, &h.m_tree_off, (size_t)max_trees + 1));
    TRY(dev_alloc(t, &h.m_feat, (size_t)node_cap));
    TRY(dev_alloc(t, &h.m_left, (size_t)node_cap));
    TRY(dev_alloc(t, &h.m_right, (size_t)node_cap));
    TRY(dev_alloc(t, &h.m_thr, (size_t)node_cap));
    TRY(dev_alloc(t, &h.m_val, (size_t)node_cap));
#undef TRY
    if (rc != FS_OK) {
        fs_trainer_destroy(t);
        return rc;
    }
    h.bins = bins;
    h.prog_off = d_prog_off;
    h.target = d_target;
    h.cut_off = d_cut_off;
    h.cuts = d_cuts;
    h.hot_bin = d_hot;
    const int32_t zeros[4] = {0, 0, 0, 0};
    e = hipMemcpyAsync(d_prog_off, prog_off, sizeof(int32_t) * ((size_t)n_programs + 1),
                       hipMemcpyDeviceToDevice, stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(d_target, target, sizeof(float) * (size_t)n_programs,
                           hipMemcpyDeviceToDevice, stream);
    // small host arrays: plain copies (these wait for the device)
    if (e == hipSuccess)
        e = hipMemcpy(d_cut_off, cut_off, sizeof(int32_t) * ((size_t)n_features + 1), hipMemcpyHostToDevice);
    if (e == hipSuccess && n_cuts > 0)
        e = hipMemcpy(d_cuts, cuts, sizeof(float) * (size_t)n_cuts, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(h.counters, zeros, sizeof(zeros), hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(h.m_tree_off, zeros, sizeof(int32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        fs_trainer_destroy(t);
        return fail_hip(e, "fs_trainer_create: copies");
    }
    hipLaunchKernelGGL(train_bin_kernel, dim3((unsigned)((n_rows + 255) / 256), (unsigned)n_features),
                       dim3(256), 0, stream, features, layout, n_features, (int)n_rows, h.r_pad,
                       (const int32_t *)d_cut_off, (const float *)d_cuts, bins);
    rc = check_launch("train_bin_kernel launch");
    if (rc == FS_OK) {
        hipLaunchKernelGGL(train_hot_bin_kernel, dim3((unsigned)n_features), dim3(256), 0, stream,
                           (const uint8_t *)bins, (int)n_rows, h.r_pad, d_hot);
        hipLaunchKernelGGL(train_fill_kernel, dim3(1024), dim3(256), 0, stream, h.row_pred,
                           (int64_t)n_rows, bias);
        rc = check_launch("trainer set-up kernels launch");
    }
    if (rc == FS_OK) {
        // counters[3] is free until training starts: longest program, read back here
        hipLaunchKernelGGL(train_max_len_kernel, dim3(256), dim3(256), 0, stream,
                           (const int32_t *)d_prog_off, n_programs, h.counters + 3);
        rc = check_launch("train_max_len_kernel launch");
        if (rc == FS_OK) {
            e = hipStreamSynchronize(stream);
            if (e == hipSuccess)
                e = hipMemcpy(&t->max_len, h.counters + 3, sizeof(int32_t), hipMemcpyDeviceToHost);
            if (e != hipSuccess)
                rc = fail_hip(e, "fs_trainer_create: reading the longest program");
        }
    }
    if (rc != FS_OK) {
        fs_trainer_destroy(t);
        return rc;
    }
    *out = t;
    return FS_OK;
}

// The global histogram buffer of a trainer whose rows span several slabs, all zero at first
// (the split kernel clears what it reads).
static int ensure_hist(fs_trainer *t, hipStream_t stream)
{
    if (t->h.hist)
        return FS_OK;
    const size_t slots = t->max_depth > 0 ? (size_t)1 << (t->max_depth - 1) : 1;
    const size_t words = slots * (size_t)t->h.n_features * kBins * 2;
    int rc = dev_alloc(t, &t->h.hist, words);
    if (rc != FS_OK)
        return rc;
    hipLaunchKernelGGL(train_fill_kernel, dim3(1024), dim3(256), 0, stream, (float *)t->h.hist,
                       (int64_t)words * 2, 0.0f);
    return check_launch("train_fill_kernel launch");
}

// Buffers for the rows regrouped by node (deep trees).
static int ensure_sort(fs_trainer *t)
{
    if (t->h.s_bins)
        return FS_OK;
    TrainDesc &h = t->h;
    const size_t groups = ((size_t)h.n_features + 3) / 4;
    int rc = dev_alloc(t, &h.s_qh, (size_t)h.n_rows);
    if (rc == FS_OK) rc = dev_alloc(t, &h.s_rowid, (size_t)h.n_rows);
    if (rc == FS_OK) rc = dev_alloc(t, &h.s_node, (size_t)h.n_rows);
    if (rc == FS_OK) rc = dev_alloc(t, &h.s_dest, (size_t)h.n_rows);
    if (rc == FS_OK) rc = dev_alloc(t, &h.seg_start, (size_t)kSortSegs + 1);
    if (rc == FS_OK) rc = dev_alloc(t, &h.seg_cursor, (size_t)kSortSegs);
    if (rc == FS_OK) rc = dev_alloc(t, &h.s_bins, groups * (size_t)h.r_pad * 4);   // last: marks the set complete
    return rc;
}

// Uploads the batch's descriptors; returns the device array.
static int upload_batch(int n, fs_trainer *const *trainers, hipStream_t stream, const TrainDesc **d_out)
{
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 16)
        return fail(FS_EUNSUPPORTED, "device ordinal %d not supported", dev);
    BatchBuf &b = g_batch[dev];
    if (!b.copied)
        FS_HIP(hipEventCreateWithFlags(&b.copied, hipEventDisableTiming));
    if (b.pending) {
        FS_HIP(hipEventSynchronize(b.copied));     // the previous upload has left the staging buffer
        b.pending = false;
    }
    if (b.cap < n) {
        // earlier batches may still be read by kernels in flight
        FS_HIP(hipDeviceSynchronize());
        if (b.d_desc)
            FS_HIP(hipFree(b.d_desc));
        if (b.h_desc)
            FS_HIP(hipHostFree(b.h_desc));
        b.d_desc = b.h_desc = nullptr;
        b.cap = 0;
        const int cap = n < 16 ? 16 : 2 * n;
        FS_HIP(hipMalloc((void **)&b.d_desc, sizeof(TrainDesc) * (size_t)cap));
        FS_HIP(hipHostMalloc((void **)&b.h_desc, sizeof(TrainDesc) * (size_t)cap, hipHostMallocDefault));
        b.cap = cap;
    }
    // Largest families first: the histogram launches have a workgroup per (family, four
    // features), a little more than one per compute unit, and those dispatched last should be
    // the short ones.  (The order of the descriptors is internal; kernels index by block.)
    std::vector<int> order;
    try {
        order.resize((size_t)n);
    } catch (...) {
        return fail(FS_ENOMEM, "out of host memory");
    }
    for (int i = 0; i < n; ++i)
        order[(size_t)i] = i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int c) { return trainers[a]->h.n_rows > trainers[c]->h.n_rows; });
    for (int i = 0; i < n; ++i)
        b.h_desc[i] = trainers[order[(size_t)i]]->h;
    FS_HIP(hipMemcpyAsync(b.d_desc, b.h_desc, sizeof(TrainDesc) * (size_t)n, hipMemcpyHostToDevice, stream));
    FS_HIP(hipEventRecord(b.copied, stream));
    b.pending = true;
    *d_out = b.d_desc;
    return FS_OK;
}

static int check_batch(const char *who, int n, fs_trainer *const *trainers)
{
    if (n < 0)
        return fail(FS_EINVAL, "%s: n_trainers %d is negative", who, n);
    if (n > 0 && !trainers)
        return fail(FS_EINVAL, "%s: trainers is NULL", who);
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    for (int i = 0; i < n; ++i) {
        if (!trainers[i])
            return fail(FS_EINVAL, "%s: trainer %d is NULL", who, i);
        if (trainers[i]->device != dev)
            return fail(FS_EINVAL, "%s: trainer %d lives on device %d, current is %d", who, i,
                        trainers[i]->device, dev);
        for (int j = 0; j < i; ++j)
            if (trainers[j] == trainers[i])
                return fail(FS_EINVAL, "%s: trainer %d appears twice in the batch", who, i);
    }
    return FS_OK;
}

extern "C" int fs_train_boost(int32_t n_trainers, fs_trainer *const *trainers, int32_t n_rounds,
                              const fs_train_params *p, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    int rc = check_batch("fs_train_boost", n_trainers, trainers);
    if (rc != FS_OK)
        return rc;
    if (!p)
        return fail(FS_EINVAL, "fs_train_boost: params is NULL");
    if (n_rounds < 0)
        return fail(FS_EINVAL, "fs_train_boost: n_rounds %d is negative", n_rounds);
    if (p->max_depth < 0 || p->max_depth > FS_TRAIN_MAX_DEPTH)
        return fail(FS_EUNSUPPORTED, "fs_train_boost: max_depth=%d outside 0..%d", p->max_depth,
                    FS_TRAIN_MAX_DEPTH);
    if (!(p->eta > 0.0f) || !(p->lambda >= 0.0f) || !(p->grad_scale > 0.0f) || isinf(p->grad_scale) ||
        isnan(p->min_gain) || isnan(p->min_child_weight))
        return fail(FS_EINVAL, "fs_train_boost: eta > 0, lambda >= 0, grad_scale > 0 required");
    int exp2 = 0;
    if (frexpf(p->grad_scale, &exp2) != 0.5f)
        return fail(FS_EINVAL, "fs_train_boost: grad_scale must be a power of two");
    if (n_trainers == 0 || n_rounds == 0)
        return FS_OK;
    int max_rows = 0, max_prog = 0, max_feat = 0, max_len = 0;
    for (int i = 0; i < n_trainers; ++i) {
        const fs_trainer *t = trainers[i];
        if (p->max_depth > t->max_depth)
            return fail(FS_EUNSUPPORTED, "fs_train_boost: trainer %d was created for max_depth %d", i, t->max_depth);
        if (t->trees_enqueued + n_rounds > t->max_trees)
            return fail(FS_EUNSUPPORTED, "fs_train_boost: trainer %d holds %d trees of at most %d", i,
                        t->trees_enqueued, t->max_trees);
        if (t->h.n_rows > max_rows) max_rows = t->h.n_rows;
        if (t->h.n_programs > max_prog) max_prog = t->h.n_programs;
        if (t->h.n_features > max_feat) max_feat = t->h.n_features;
        if (t->max_len > max_len) max_len = t->max_len;
    }
    std::lock_guard<std::mutex> lock(g_train_mu);
    int slab_rows = kHistRowsPerSlab;
    {
        const int v = tune(FS_TUNE_TRAIN_SLAB_ROWS);             // test / tuning override
        if (v >= 64 && v <= kHistRowsPerSlab)
            slab_rows = v;
    }
    // one slab per family up to slab_rows rows: the histogram workgroup then searches the cuts
    // itself and nothing is added up in global memory
    const int n_slabs = (max_rows + slab_rows - 1) / slab_rows;
    if (n_slabs > 1)
        for (int i = 0; i < n_trainers && rc == FS_OK; ++i)
            rc = ensure_hist(trainers[i], stream);
    // deep trees of one-slab families: rows regrouped by node before level kSortLevel
    bool use_sort = n_slabs == 1 && p->max_depth >= kSortMinDepth;
    if (tune(FS_TUNE_TRAIN_SORT) >= 0)                           // override: 0 never, 1 whenever possible
        use_sort = n_slabs == 1 && tune(FS_TUNE_TRAIN_SORT) != 0 && p->max_depth > kSortLevel;
    if (use_sort)
        for (int i = 0; i < n_trainers && rc == FS_OK; ++i)
            rc = ensure_sort(trainers[i]);
    if (rc != FS_OK)
        return rc;
    const TrainDesc *d = nullptr;
    rc = upload_batch(n_trainers, trainers, stream, &d);
    if (rc != FS_OK)
        return rc;
    Params prm;
    prm.eta = (double)p->eta;
    prm.lambda = (double)p->lambda;
    prm.min_gain = (double)p->min_gain;
    prm.inv_scale = 1.0 / (double)p->grad_scale;
    double mcw = ceil((double)p->min_child_weight);
    prm.mcw = mcw < 1.0 ? 1 : (mcw > 9e18 ? (long long)9e18 : (long long)mcw);
    prm.grad_scale = p->grad_scale;
    prm.max_depth = p->max_depth;

    static bool hist_configured[16] = {};
    {
        int dev = 0;
        FS_HIP(hipGetDevice(&dev));
        if (!hist_configured[dev]) {
            FS_HIP(hipFuncSetAttribute((const void *)train_hist_kernel<true>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kHistSlotsPacked * kHistFeats * kBins * 8 + kHistTrashWords * 8));
            FS_HIP(hipFuncSetAttribute((const void *)train_hist_kernel<false>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kHistSlotsWide * kHistFeats * kBins * 16 + kHistTrashWords * 8));
            hist_configured[dev] = true;
        }
    }
    const unsigned nt = (unsigned)n_trainers;
    const unsigned row_blocks = (unsigned)((max_rows + 255) / 256);
    const int rows_per_slab = (((max_rows + n_slabs - 1) / n_slabs) + 63) & ~63;
    // Bits that hold any curvature sum of a slab (rows x longest program bounds it).  The packed
    // form of the histograms needs room for the gradient sums beside them; beyond 31 bits the
    // wide form is launched right away.
    int hb = 1;
    {
        const long long bound = (long long)max_len * (long long)(rows_per_slab < max_rows ? rows_per_slab : max_rows);
        while (hb < 63 && ((long long)1 << hb) <= bound)
            ++hb;
    }
    bool packed = hb <= 31;
    if (tune(FS_TUNE_TRAIN_PACKED) == 0)                         // override: wide form only
        packed = false;
    for (int round = 0; round < n_rounds; ++round) {
        prof_start(kKernTrainOther, stream);
        hipLaunchKernelGGL(train_begin_tree_kernel, dim3(nt), dim3(512), 0, stream, d);
        hipLaunchKernelGGL(train_grad_kernel, dim3((unsigned)((max_prog + 255) / 256), nt), dim3(256), 0,
                           stream, d, prm.grad_scale, 1);
        prof_stop(stream);
        for (int level = 0; level < prm.max_depth; ++level) {
            const int n_slots = 1 << level;
            const int sorted = use_sort && level >= kSortLevel ? 1 : 0;
            const int per_pass = packed ? kHistSlotsPacked : kHistSlotsWide;
            const int slots = n_slots < per_pass ? n_slots : per_pass;
            const int passes = n_slots / slots;
            const dim3 hgrid((unsigned)n_slabs, (unsigned)((max_feat + kHistFeats - 1) / kHistFeats), nt * passes);
            prof_start(kKernTrainHist, stream);
            if (packed) {
                // a lone node still needs the 8 KB of its wide form for the fall-back
                size_t lds = (size_t)slots * kHistFeats * kBins * 8;
                if (lds < (size_t)kHistFeats * kBins * 16)
                    lds = (size_t)kHistFeats * kBins * 16;
                hipLaunchKernelGGL(train_hist_kernel<true>, hgrid, dim3(kHistThreads), lds + kHistTrashWords * 8,
                                   stream, d, level, passes, rows_per_slab, n_slabs, hb, sorted, prm);
            } else {
                hipLaunchKernelGGL(train_hist_kernel<false>, hgrid, dim3(kHistThreads),
                                   (size_t)slots * kHistFeats * kBins * 16 + kHistTrashWords * 8, stream, d, level, passes,
                                   rows_per_slab, n_slabs, 0, sorted, prm);
            }
            prof_stop(stream);
            prof_start(kKernTrainSplit, stream);
            if (n_slabs > 1)
                hipLaunchKernelGGL(train_split_kernel,
                                   dim3((unsigned)((n_slots * max_feat + kSplitWaves - 1) / kSplitWaves), 1u, nt),
                                   dim3(64 * kSplitWaves), 0, stream, d, level, prm);
            // from 64 nodes on the per-node reduction over the features gets the whole chip
            const int reduced = n_slots >= kPickSpreadSlots ? 1 : 0;
            if (reduced)
                hipLaunchKernelGGL(train_pick_reduce_kernel,
                                   dim3((unsigned)(n_slots / (kPickThreads / 64)), nt), dim3(kPickThreads), 0,
                                   stream, d, level, prm);
            hipLaunchKernelGGL(train_pick_kernel, dim3(nt), dim3(kPickThreads), 0, stream, d, level, reduced,
                               prm);
            prof_stop(stream);
            prof_start(kKernTrainOther, stream);
            if (sorted)
                hipLaunchKernelGGL(train_part_sorted_kernel, dim3(row_blocks, nt), dim3(256), 0, stream, d, level);
            else
                hipLaunchKernelGGL(train_part_kernel, dim3(row_blocks, nt), dim3(256), 0, stream, d, level);
            if (use_sort && level == kSortLevel - 1) {
                hipLaunchKernelGGL(train_seg_count_kernel, dim3(row_blocks, nt), dim3(256), 0, stream, d);
                hipLaunchKernelGGL(train_seg_scan_kernel, dim3(nt), dim3(64), 0, stream, d);
                hipLaunchKernelGGL(train_seg_place_kernel, dim3(row_blocks, nt), dim3(256), 0, stream, d);
                hipLaunchKernelGGL(train_seg_bins_kernel, dim3(row_blocks, (unsigned)((max_feat + 3) / 4), nt),
                                   dim3(256), 0, stream, d);
            }
            prof_stop(stream);
        }
        prof_start(kKernTrainOther, stream);
        hipLaunchKernelGGL(train_pick_kernel, dim3(nt), dim3(kPickThreads), 0, stream, d,
                           prm.max_depth, 0, prm);
        hipLaunchKernelGGL(train_update_kernel, dim3(row_blocks, nt), dim3(256), 0, stream, d,
                           use_sort ? 1 : 0);
        hipLaunchKernelGGL(train_emit_kernel, dim3(nt), dim3(512), 0, stream, d);
        prof_stop(stream);
        rc = check_launch("training kernels launch");
        if (rc != FS_OK)
            return rc;
    }
    for (int i = 0; i < n_trainers; ++i)
        trainers[i]->trees_enqueued += n_rounds;
    return FS_OK;
}

extern "C" int fs_trainer_size(const fs_trainer *t, int32_t *n_trees, int64_t *n_nodes, void *stream_)
{
    if (!t)
        return fail(FS_EINVAL, "fs_trainer_size: trainer is NULL");
    FS_HIP(hipStreamSynchronize((hipStream_t)stream_));
    int32_t c[4];
    FS_HIP(hipMemcpy(c, t->h.counters, sizeof(c), hipMemcpyDeviceToHost));
    if (n_trees)
        *n_trees = c[1];
    if (n_nodes)
        *n_nodes = c[2];
    return FS_OK;
}

extern "C" int fs_trainer_export(const fs_trainer *t, int32_t *tree_off, int32_t *split_feature,
                                 float *threshold, int32_t *left, int32_t *right, float *value,
                                 void *stream_)
{
    if (!t || !tree_off || !split_feature || !threshold || !left || !right || !value)
        return fail(FS_EINVAL, "fs_trainer_export: NULL argument");
    FS_HIP(hipStreamSynchronize((hipStream_t)stream_));
    int32_t c[4];
    FS_HIP(hipMemcpy(c, t->h.counters, sizeof(c), hipMemcpyDeviceToHost));
    const size_t n = (size_t)c[2];
    FS_HIP(hipMemcpy(tree_off, t->h.m_tree_off, sizeof(int32_t) * ((size_t)c[1] + 1), hipMemcpyDeviceToHost));
    if (n) {
        FS_HIP(hipMemcpy(split_feature, t->h.m_feat, sizeof(int32_t) * n, hipMemcpyDeviceToHost));
        FS_HIP(hipMemcpy(threshold, t->h.m_thr, sizeof(float) * n, hipMemcpyDeviceToHost));
        FS_HIP(hipMemcpy(left, t->h.m_left, sizeof(int32_t) * n, hipMemcpyDeviceToHost));
        FS_HIP(hipMemcpy(right, t->h.m_right, sizeof(int32_t) * n, hipMemcpyDeviceToHost));
        FS_HIP(hipMemcpy(value, t->h.m_val, sizeof(float) * n, hipMemcpyDeviceToHost));
    }
    return FS_OK;
}

extern "C" int fs_trainer_predictions(const fs_trainer *t, float *row_pred, float *prog_pred, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (!t)
        return fail(FS_EINVAL, "fs_trainer_predictions: trainer is NULL");
    fs_trainer *tt = const_cast<fs_trainer *>(t);
    int rc = check_batch("fs_trainer_predictions", 1, &tt);
    if (rc != FS_OK)
        return rc;
    std::lock_guard<std::mutex> lock(g_train_mu);
    if (prog_pred) {
        const TrainDesc *d = nullptr;
        rc = upload_batch(1, &tt, stream, &d);
        if (rc != FS_OK)
            return rc;
        hipLaunchKernelGGL(train_grad_kernel, dim3((unsigned)((t->h.n_programs + 255) / 256), 1u), dim3(256), 0,
                           stream, d, 1.0f, 0);
        rc = check_launch("train_grad_kernel launch");
        if (rc != FS_OK)
            return rc;
        FS_HIP(hipMemcpyAsync(prog_pred, t->h.prog_pred, sizeof(float) * (size_t)t->h.n_programs,
                              hipMemcpyDeviceToDevice, stream));
    }
    if (row_pred)
        FS_HIP(hipMemcpyAsync(row_pred, t->h.row_pred, sizeof(float) * (size_t)t->h.n_rows,
                              hipMemcpyDeviceToDevice, stream));
    return FS_OK;
}
