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
//   per level:   zero_hist, hist (LDS histograms per row slab and feature group, flushed
//                with 64-bit atomics), split (one workgroup per (node, feature): scan the
//                bins, best cut), pick (per node: best feature, split or leaf, child ids in
//                breadth-first order), part (rows of split nodes move to a child)
//   pick         once more at max_depth: what is left becomes leaves
//   update       row output += value of the row's leaf;  emit: heap -> flat model arrays
#include <math.h>
#include <mutex>
#include <new>
#include <vector>

#include "familyseer_train.h"
#include "fs_internal.h"

namespace fs {

constexpr int kHeapNodes = (1 << (FS_TRAIN_MAX_DEPTH + 1)) - 1;   // 511
constexpr int kBins = FS_TRAIN_MAX_CUTS + 1;                      // 256
constexpr int kHistThreads = 512;
constexpr int kHistRowsPerBlock = 4096;
constexpr int kHistPairs = 32;        // (node, feature) histograms a workgroup keeps in LDS

// heap node states
enum { kAbsent = 0, kOpen = 1, kInternal = 2, kLeaf = 3 };

struct TrainDesc {
    const uint8_t *bins;       // [feature][r_pad]
    const int32_t *prog_off;
    const float *target;
    const int32_t *cut_off;    // device copies of the cut lists
    const float *cuts;
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
    bins[(int64_t)f * r_pad + r] = (uint8_t)lo;
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
    if (threadIdx.x == 0)
        d.counters[0] = 1;
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
        }
    }
    if (!with_grad)
        return;
    // root totals: wavefront sum, one atomic per wavefront
    for (int off = 32; off > 0; off >>= 1) {
        G += __shfl_down(G, off);
        H += __shfl_down(H, off);
    }
    if ((threadIdx.x & 63) == 0 && H != 0) {
        atomicAdd((unsigned long long *)&d.h_G[0], (unsigned long long)G);
        atomicAdd((unsigned long long *)&d.h_H[0], (unsigned long long)H);
    }
}

__global__ void train_zero_hist_kernel(const TrainDesc *__restrict__ descs, int n_slots)
{
    const TrainDesc &d = descs[blockIdx.y];
    const int64_t n = (int64_t)n_slots * d.n_features * kBins * 2;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        d.hist[i] = 0ull;
}

// Histograms of one level.  A workgroup takes a slab of rows and `fg` consecutive features
// and keeps the (G, H) histograms of `slots` nodes x fg features in LDS (at most kHistPairs);
// blockIdx.z = trainer * passes + pass, a pass covering `slots` consecutive nodes.
__global__ void __launch_bounds__(kHistThreads)
train_hist_kernel(const TrainDesc *__restrict__ descs, int level, int fg, int slots, int passes)
{
    extern __shared__ unsigned long long lds_hist[];            // G: [pairs][256] u64
    unsigned int *lds_h = (unsigned int *)(lds_hist + kHistPairs * kBins);   // H: [pairs][256] u32
    const TrainDesc &d = descs[blockIdx.z / passes];
    const int pass = blockIdx.z % passes;
    const int row0 = blockIdx.x * kHistRowsPerBlock;
    if (row0 >= d.n_rows)
        return;
    const int row1 = min(row0 + kHistRowsPerBlock, d.n_rows);
    const int f0 = blockIdx.y * fg;
    const int nf = min(fg, d.n_features - f0);
    const int node0 = (1 << level) - 1 + pass * slots;          // heap index of slot 0
    const int pairs = slots * fg;
    for (int i = threadIdx.x; i < pairs * kBins; i += kHistThreads) {
        lds_hist[i] = 0ull;
        lds_h[i] = 0u;
    }
    __syncthreads();
    for (int r = row0 + threadIdx.x; r < row1; r += kHistThreads) {
        const int slot = (int)d.node_of_row[r] - node0;
        if ((unsigned)slot >= (unsigned)slots)
            continue;
        const int2 qh = d.qh[r];
        for (int fi = 0; fi < nf; ++fi) {
            const int b = d.bins[(int64_t)(f0 + fi) * d.r_pad + r];
            const int at = (slot * fg + fi) * kBins + b;
            atomicAdd(&lds_hist[at], (unsigned long long)(long long)qh.x);
            atomicAdd(&lds_h[at], (unsigned int)qh.y);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < pairs * kBins; i += kHistThreads) {
        const unsigned int h = lds_h[i];
        if (h == 0u)
            continue;
        const int pair = i / kBins, b = i - pair * kBins;
        const int slot = pair / fg, fi = pair - slot * fg;
        if (fi >= nf)
            continue;
        const int64_t at = (((int64_t)(pass * slots + slot) * d.n_features + (f0 + fi)) * kBins + b) * 2;
        atomicAdd(&d.hist[at], lds_hist[i]);
        atomicAdd(&d.hist[at + 1], (unsigned long long)h);
    }
}

__device__ __forceinline__ double split_gain(long long GL, long long HL, long long G, long long H,
                                             double inv_scale, double lambda)
{
    const long long GR = G - GL, HR = H - HL;
    const double gl = (double)GL * inv_scale, gr = (double)GR * inv_scale,
                 g = (double)G * inv_scale;
    double t1 = gl * gl;
    t1 = t1 / ((double)HL + lambda);
    double t2 = gr * gr;
    t2 = t2 / ((double)HR + lambda);
    double t3 = g * g;
    t3 = t3 / ((double)H + lambda);
    return (t1 + t2) - t3;
}

// Best cut of one feature for one open node: thread t owns bin t and cut t+1.
__global__ void __launch_bounds__(kBins)
train_split_kernel(const TrainDesc *__restrict__ descs, int level, Params prm)
{
    __shared__ long long sG[kBins], sH[kBins];
    __shared__ double s_gain[kBins];
    __shared__ int s_cut[kBins];
    const TrainDesc &d = descs[blockIdx.z];
    const int f = blockIdx.x, slot = blockIdx.y, t = threadIdx.x;
    if (f >= d.n_features)
        return;
    const int node = (1 << level) - 1 + slot;
    if (d.h_state[node] != kOpen)
        return;
    const int64_t at = (((int64_t)slot * d.n_features + f) * kBins + t) * 2;
    sG[t] = (long long)d.hist[at];
    sH[t] = (long long)d.hist[at + 1];
    __syncthreads();
    for (int off = 1; off < kBins; off <<= 1) {                  // inclusive scan over the bins
        long long g = 0, h = 0;
        if (t >= off) {
            g = sG[t - off];
            h = sH[t - off];
        }
        __syncthreads();
        sG[t] += g;
        sH[t] += h;
        __syncthreads();
    }
    const long long G = d.h_G[node], H = d.h_H[node];
    const int m = d.cut_off[f + 1] - d.cut_off[f];
    const long long GL = sG[t], HL = sH[t];                      // left side of cut t+1
    int cut = 0;
    double gain = 0.0;
    if (t + 1 <= m && HL >= prm.mcw && H - HL >= prm.mcw) {
        cut = t + 1;
        gain = split_gain(GL, HL, G, H, prm.inv_scale, prm.lambda);
    }
    s_gain[t] = gain;
    s_cut[t] = cut;
    __syncthreads();
    for (int off = kBins / 2; off > 0; off >>= 1) {              // largest gain, lowest cut on ties
        if (t < off) {
            const double ga = s_gain[t], gb = s_gain[t + off];
            const int ca = s_cut[t], cb = s_cut[t + off];
            if (cb != 0 && (ca == 0 || gb > ga || (gb == ga && cb < ca))) {
                s_gain[t] = gb;
                s_cut[t] = cb;
            }
        }
        __syncthreads();
    }
    const int best = s_cut[0];
    const int64_t o = (int64_t)slot * d.n_features + f;
    if (t == 0) {
        d.best_gain[o] = s_gain[0];
        d.best_cut[o] = best;
    }
    if (best != 0 && t == best - 1) {
        d.best_GL[o] = GL;
        d.best_HL[o] = HL;
    }
}

// Per open node of the level: best feature, split or leaf; children get consecutive ids in
// slot order (breadth-first numbering).  One workgroup per trainer, one thread per slot.
__global__ void __launch_bounds__(1 << FS_TRAIN_MAX_DEPTH)
train_pick_kernel(const TrainDesc *__restrict__ descs, int level, Params prm)
{
    __shared__ int s_scan[1 << FS_TRAIN_MAX_DEPTH];
    const TrainDesc &d = descs[blockIdx.x];
    const int slot = threadIdx.x, n_slots = 1 << level;
    const int node = n_slots - 1 + slot;
    const bool open = slot < n_slots && d.h_state[node] == kOpen;
    int bf = -1, bc = 0;
    double bg = 0.0;
    if (open && level < prm.max_depth) {
        for (int f = 0; f < d.n_features; ++f) {
            const int64_t o = (int64_t)slot * d.n_features + f;
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
    }
    const bool split = open && bf >= 0 && bg > prm.min_gain;
    s_scan[threadIdx.x] = split ? 1 : 0;
    __syncthreads();
    for (int off = 1; off < (int)blockDim.x; off <<= 1) {
        int v = 0;
        if ((int)threadIdx.x >= off)
            v = s_scan[threadIdx.x - off];
        __syncthreads();
        s_scan[threadIdx.x] += v;
        __syncthreads();
    }
    const int before = s_scan[threadIdx.x] - (split ? 1 : 0);
    const int total = s_scan[blockDim.x - 1];
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
    const int b = d.bins[(int64_t)d.h_feat[node] * d.r_pad + r];
    d.node_of_row[r] = (uint16_t)(2 * node + (b < d.h_cut[node] ? 1 : 2));
}

__global__ void __launch_bounds__(256)
train_update_kernel(const TrainDesc *__restrict__ descs)
{
    const TrainDesc &d = descs[blockIdx.y];
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= d.n_rows)
        return;
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
#define TRY(x)            \
    if (rc == FS_OK)      \
    rc = (x)
    TRY(dev_alloc(t, &bins, (size_t)h.r_pad * n_features));
    TRY(dev_alloc(t, &d_prog_off, (size_t)n_programs + 1));
    TRY(dev_alloc(t, &d_target, (size_t)n_programs));
    TRY(dev_alloc(t, &d_cut_off, (size_t)n_features + 1));
    TRY(dev_alloc(t, &d_cuts, (size_t)n_cuts));
    TRY(dev_alloc(t, &h.row_pred, (size_t)n_rows));
    TRY(dev_alloc(t, &h.prog_pred, (size_t)n_programs));
    TRY(dev_alloc(t, &h.qh, (size_t)n_rows));
    TRY(dev_alloc(t, &h.node_of_row, (size_t)n_rows));
    TRY(dev_alloc(t, &h.hist, (size_t)hist_slots * n_features * kBins * 2));
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
        hipLaunchKernelGGL(train_fill_kernel, dim3(1024), dim3(256), 0, stream, h.row_pred,
                           (int64_t)n_rows, bias);
        rc = check_launch("train_fill_kernel launch");
    }
    if (rc != FS_OK) {
        fs_trainer_destroy(t);
        return rc;
    }
    *out = t;
    return FS_OK;
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
    for (int i = 0; i < n; ++i)
        b.h_desc[i] = trainers[i]->h;
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
    int max_rows = 0, max_prog = 0, max_feat = 0;
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
    }
    std::lock_guard<std::mutex> lock(g_train_mu);
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
    const size_t hist_lds = (size_t)kHistPairs * kBins * 12;
    {
        int dev = 0;
        FS_HIP(hipGetDevice(&dev));
        if (!hist_configured[dev]) {
            FS_HIP(hipFuncSetAttribute((const void *)train_hist_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)hist_lds));
            hist_configured[dev] = true;
        }
    }
    const unsigned nt = (unsigned)n_trainers;
    const unsigned row_blocks = (unsigned)((max_rows + 255) / 256);
    const unsigned slabs = (unsigned)((max_rows + kHistRowsPerBlock - 1) / kHistRowsPerBlock);
    for (int round = 0; round < n_rounds; ++round) {
        hipLaunchKernelGGL(train_begin_tree_kernel, dim3(nt), dim3(512), 0, stream, d);
        hipLaunchKernelGGL(train_grad_kernel, dim3((unsigned)((max_prog + 255) / 256), nt), dim3(256), 0,
                           stream, d, prm.grad_scale, 1);
        for (int level = 0; level < prm.max_depth; ++level) {
            const int n_slots = 1 << level;
            const int fg = n_slots <= 8 ? 4 : (n_slots == 16 ? 2 : 1);
            const int slots = n_slots < kHistPairs ? n_slots : kHistPairs;
            const int passes = n_slots / slots;
            hipLaunchKernelGGL(train_zero_hist_kernel, dim3(256, nt), dim3(256), 0, stream, d, n_slots);
            hipLaunchKernelGGL(train_hist_kernel, dim3(slabs, (unsigned)((max_feat + fg - 1) / fg), nt * passes),
                               dim3(kHistThreads), hist_lds, stream, d, level, fg, slots, passes);
            hipLaunchKernelGGL(train_split_kernel, dim3((unsigned)max_feat, (unsigned)n_slots, nt), dim3(kBins),
                               0, stream, d, level, prm);
            hipLaunchKernelGGL(train_pick_kernel, dim3(nt), dim3(1 << FS_TRAIN_MAX_DEPTH), 0, stream, d, level, prm);
            hipLaunchKernelGGL(train_part_kernel, dim3(row_blocks, nt), dim3(256), 0, stream, d, level);
        }
        hipLaunchKernelGGL(train_pick_kernel, dim3(nt), dim3(1 << FS_TRAIN_MAX_DEPTH), 0, stream, d,
                           prm.max_depth, prm);
        hipLaunchKernelGGL(train_update_kernel, dim3(row_blocks, nt), dim3(256), 0, stream, d);
        hipLaunchKernelGGL(train_emit_kernel, dim3(nt), dim3(512), 0, stream, d);
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
