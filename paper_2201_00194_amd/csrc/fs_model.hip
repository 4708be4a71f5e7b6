// fs_model_create / fs_model_destroy: validation of the caller's ensemble and packing into
// the two device formats (flat global-memory nodes; LDS-staged chunk images).
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "fs_internal.h"

using namespace fs;

namespace {

struct PackedTree {
    std::vector<uint32_t> words;     // tree image; child offsets relative to the tree start
    std::vector<uint16_t> slot_ids;  // caller's local id per 4-byte slot
    std::vector<uint32_t> fix;       // word indices whose low 16 bits need + tree base
    int depth = 0;
};

// Breadth-first relabelling that puts the two children of a node next to each other.
// Returns false if the node graph is not a tree (a shared child), or if compact is asked for
// and the tree is not perfect of `depth`.
bool pack_tree(const int32_t *sf, const float *thr, const int32_t *left, const int32_t *right,
               const float *val, int32_t sz, int n_features, bool compact, int depth,
               PackedTree *out)
{
    std::vector<int32_t> order;
    std::vector<int32_t> level;
    order.push_back(0);
    level.push_back(0);
    int max_level = 0;
    for (size_t i = 0; i < order.size(); ++i) {
        const int32_t n = order[i];
        if (sf[n] >= 0) {
            order.push_back(left[n]);
            level.push_back(level[i] + 1);
            order.push_back(right[n]);
            level.push_back(level[i] + 1);
            if (level[i] + 1 > max_level)
                max_level = level[i] + 1;
            if (order.size() > (size_t)sz)
                return false;   // some node has two parents: not a tree, would unfold without bound
        }
    }
    out->depth = max_level;
    const size_t n = order.size();
    // position of the first child of order[i] in `order`: children are appended in visit order
    std::vector<uint32_t> first_child(n, 0);
    {
        uint32_t next = 1;
        for (size_t i = 0; i < n; ++i)
            if (sf[order[i]] >= 0) {
                first_child[i] = next;
                next += 2;
            }
    }
    const uint32_t nan_col = (uint32_t)n_features * 256u;
    if (!compact) {
        out->words.assign(2 * n, 0);
        out->slot_ids.assign(2 * n, 0);
        for (size_t i = 0; i < n; ++i) {
            const int32_t o = order[i];
            uint32_t w0, w1;
            if (sf[o] >= 0) {
                memcpy(&w0, &thr[o], 4);
                w1 = (((uint32_t)sf[o] * 256u) << 16) | (8u * first_child[i]);
            } else {
                memcpy(&w0, &val[o], 4);
                // own offset - 8; the tree base is at least 8, so this never underflows
                w1 = (nan_col << 16) | ((8u * (uint32_t)i - 8u) & 0xFFFFu);
            }
            out->words[2 * i] = w0;
            out->words[2 * i + 1] = w1;
            out->fix.push_back((uint32_t)(2 * i + 1));
            out->slot_ids[2 * i] = (uint16_t)o;
            out->slot_ids[2 * i + 1] = (uint16_t)o;
        }
        return true;
    }
    // compact: internal nodes first (8 bytes), then leaves (4 bytes), both in visit order
    const size_t n_int = ((size_t)1 << depth) - 1, n_leaf = (size_t)1 << depth;
    if (n != n_int + n_leaf)
        return false;
    for (size_t i = 0; i < n; ++i)
        if ((sf[order[i]] >= 0) != (i < n_int) || level[i] != (i < n_int ? level[i] : depth))
            return false;
    out->words.assign(2 * n_int + n_leaf, 0);
    out->slot_ids.assign(2 * n_int + n_leaf, 0);
    for (size_t i = 0; i < n_int; ++i) {
        const int32_t o = order[i];
        uint32_t w0;
        memcpy(&w0, &thr[o], 4);
        const uint32_t c = first_child[i];
        const uint32_t child_off = (c < n_int) ? 8u * c : (uint32_t)(8u * n_int + 4u * (c - n_int));
        out->words[2 * i] = w0;
        out->words[2 * i + 1] = (((uint32_t)sf[o] * 256u) << 16) | child_off;
        out->fix.push_back((uint32_t)(2 * i + 1));
        out->slot_ids[2 * i] = out->slot_ids[2 * i + 1] = (uint16_t)o;
    }
    for (size_t j = 0; j < n_leaf; ++j) {
        const int32_t o = order[n_int + j];
        memcpy(&out->words[2 * n_int + j], &val[o], 4);
        out->slot_ids[2 * n_int + j] = (uint16_t)o;
    }
    return true;
}

// Depth of every leaf equal to `*depth` (set from the first leaf) and the tree perfect?
bool tree_is_perfect(const int32_t *sf, const int32_t *left, const int32_t *right, int32_t sz,
                     int *depth)
{
    std::vector<int32_t> lev((size_t)sz, -1);
    lev[0] = 0;
    int64_t reach = 0;
    int d = -1;
    for (int32_t n = 0; n < sz; ++n) {       // children have larger ids: one forward pass
        if (lev[n] < 0)
            continue;
        ++reach;
        if (sf[n] >= 0) {
            if (lev[left[n]] >= 0 || lev[right[n]] >= 0 || left[n] == right[n])
                return false;                // shared child: not a tree
            lev[left[n]] = lev[right[n]] = lev[n] + 1;
        } else {
            if (d < 0)
                d = lev[n];
            else if (d != lev[n])
                return false;
        }
    }
    if (d < 1 || d > 14 || reach != ((int64_t)2 << d) - 1)
        return false;
    if (*depth < 0)
        *depth = d;
    return *depth == d;
}

// Largest chunk image: node offsets are 16 bits, and the kernel stages the next chunk in
// kPrefetchRegs 16-byte registers per thread.
// How many trees a chunk should get.  The wavefronts that share a tile (`share` of them) split a
// chunk's trees into runs of at most 8 and walk a run's trees side by side, so a chunk costs a
// fixed part (copy, barriers, ordered sum), a part per run of its busiest wavefront (the
// dependent LDS reads of one walk) and a part per tree of that wavefront.  Weights fitted to
// measurements, in units of one chunk with one run of few trees: 0.73 fixed, 0.27 per run,
// 0.175 per tree -- e.g. 25 trees over 3 wavefronts are two runs each where 24 are one.  Two
// plans are priced: equal chunks, and chunks that are a multiple of `share` x 8 or of `share`
// with the remainder in a last short chunk; the second is taken if it is clearly cheaper.
// Returns the trees per chunk (`fit` = how many fit in LDS).
static int chunk_tree_target(int n_trees, int fit, int share)
{
    auto cost = [share](int n) {
        const int groups = share * ((n + 8 * share - 1) / (8 * share));
        const int runs = groups / share, per = (n + groups - 1) / groups;
        return 0.73 + runs * (0.27 + 0.175 * per);
    };
    if (fit < 1) fit = 1;
    const int even_chunks = (n_trees + fit - 1) / fit;
    const int even = (n_trees + even_chunks - 1) / even_chunks;
    double best_cost = even_chunks * cost(even);
    int best = even;
    const int step = fit >= 8 * share ? 8 * share : share;
    const int whole = fit / step * step;
    if (whole >= step) {
        const int full = n_trees / whole, rest = n_trees - full * whole;
        const double c = full * cost(whole) + (rest ? cost(rest) : 0.0);
        if (c < 0.95 * best_cost) {
            best_cost = c;
            best = whole;
        }
    }
    return best;
}

// ---- chunk plan of the LDS-staged format --------------------------------------------------------
// The wavefronts that share a tile (`share` of them) split a chunk's trees; every wavefront
// walks its trees in runs of at most 8, side by side, a run to the depth of its deepest tree.
// Trees are therefore sorted by depth and cut into runs of similar depth (the cheapest cut of
// the sorted list into runs no longer than an even split would make them), and the runs are
// dealt out most expensive first, each to the wavefront with the least work so far.  Cost in the
// planner's units (weights fitted to measurements on depth-8 trees: one chunk with one run of few
// trees = 1): a chunk costs 0.73 (copy, barriers, ordered sum) + the work of its busiest
// wavefront, a run (0.034 + 0.022 x trees of the run) x (levels of the run + 1).
struct RunPlan {
    int first, count, depth;         // walk-order entries [first, first + count)
};
struct SlotPlan {
    std::vector<int> order;          // trees of the chunk (indices relative to it) in walk order
    std::vector<RunPlan> runs;       // in walk order: the runs of slot 0, then of slot 1, ...
    int slot_start[17];              // slot s walks runs [slot_start[s], slot_start[s + 1])
    double cost;
};

static double run_cost(int trees, int levels) { return (0.034 + 0.022 * trees) * (levels + 1); }

// `by_depth`: the chunk's trees (relative indices) sorted by depth, deepest first.
static void deal_trees(const std::vector<int> &by_depth, const int *depth, int share, SlotPlan *out)
{
    const int n = (int)by_depth.size();
    const int rounds = (n + 8 * share - 1) / (8 * share);
    int cap = (n + share * rounds - 1) / (share * rounds);
    if (cap > 8) cap = 8;
    if (cap < 1) cap = 1;
    struct Piece { int first, count; double cost; };
    std::vector<Piece> pieces;
    std::vector<int> list;           // the trees in the order the pieces index
    // Plain plan: the trees in their own order, share x rounds runs whose sizes differ by at most
    // one, every run to the depth of its deepest tree.
    long plain_levels = 0;
    {
        const int n_runs = share * rounds, base = n / n_runs, rem = n - base * n_runs;
        for (int j = 0, at = 0; j < n_runs; ++j) {
            const int cnt = base + (j < rem ? 1 : 0);
            int d = 0;
            for (int k = 0; k < cnt; ++k)
                d = std::max(d, depth[at + k]);
            plain_levels += (long)cnt * d;
            at += cnt;
        }
    }
    // Sorted plan: cheapest cut of the depth-sorted list into runs of at most `cap`
    std::vector<double> best((size_t)n + 1, 1e300);
    std::vector<int> from((size_t)n + 1, 0);
    best[0] = 0.0;
    for (int i = 0; i < n; ++i)
        for (int c = 1; c <= cap && i + c <= n; ++c) {
            const double v = best[(size_t)i] + run_cost(c, depth[by_depth[(size_t)i]]);
            if (v < best[(size_t)(i + c)] - 1e-12) {
                best[(size_t)(i + c)] = v;
                from[(size_t)(i + c)] = i;
            }
        }
    long sorted_levels = 0;
    for (int j = n; j > 0; j = from[(size_t)j]) {
        pieces.push_back({from[(size_t)j], j - from[(size_t)j],
                          run_cost(j - from[(size_t)j], depth[by_depth[(size_t)from[(size_t)j]]])});
        sorted_levels += (long)(j - from[(size_t)j]) * depth[by_depth[(size_t)from[(size_t)j]]];
    }
    // Sorting pays when it takes a tenth of the walked levels away (measured: with fewer shallow
    // trees the uneven wavefronts it leaves cost what the skipped levels save).
    const bool sorted = 10 * sorted_levels <= 9 * plain_levels;
    if (sorted) {
        list = by_depth;
        std::reverse(pieces.begin(), pieces.end());  // deepest (most expensive per tree) first
        std::stable_sort(pieces.begin(), pieces.end(), [](const Piece &x, const Piece &y) { return x.cost > y.cost; });
    } else {
        pieces.clear();
        list.resize((size_t)n);
        for (int j = 0; j < n; ++j)
            list[(size_t)j] = j;
        const int n_runs = share * rounds, base = n / n_runs, rem = n - base * n_runs;
        for (int j = 0, at = 0; j < n_runs; ++j) {
            const int cnt = base + (j < rem ? 1 : 0);
            if (cnt == 0)
                continue;
            // the kernel walks a run to the depth of its FIRST tree: put the deepest first
            int deepest = at;
            for (int k = 1; k < cnt; ++k)
                if (depth[at + k] > depth[deepest])
                    deepest = at + k;
            std::swap(list[(size_t)at], list[(size_t)deepest]);
            pieces.push_back({at, cnt, run_cost(cnt, depth[list[(size_t)at]])});
            at += cnt;
        }
    }
    std::vector<std::vector<Piece>> bins((size_t)share);
    std::vector<double> load((size_t)share, 0.0);
    if (sorted) {
        for (const Piece &pc : pieces) {
            int to = 0;
            for (int b = 1; b < share; ++b)
                if (load[(size_t)b] < load[(size_t)to] - 1e-12)
                    to = b;
            bins[(size_t)to].push_back(pc);
            load[(size_t)to] += pc.cost;
        }
    } else {
        for (size_t j = 0; j < pieces.size(); ++j) {      // run j to slot j mod share
            bins[j % (size_t)share].push_back(pieces[j]);
            load[j % (size_t)share] += pieces[j].cost;
        }
    }
    out->order.clear();
    out->runs.clear();
    out->cost = 0.0;
    for (int b = 0; b < share; ++b) {
        out->slot_start[b] = (int)out->runs.size();
        for (const Piece &pc : bins[(size_t)b]) {
            out->runs.push_back({(int)out->order.size(), pc.count, depth[list[(size_t)pc.first]]});
            for (int j = 0; j < pc.count; ++j)
                out->order.push_back(list[(size_t)(pc.first + j)]);
        }
        if (load[(size_t)b] > out->cost)
            out->cost = load[(size_t)b];
    }
    for (int b = share; b <= 16; ++b)
        out->slot_start[b] = (int)out->runs.size();
    out->cost += 0.73;
}

size_t chunk_image_limit(int mode)
{
    const size_t by_regs = (size_t)kLdsModeWaves[mode] * 64 * kPrefetchRegs * 16;
    return by_regs < (size_t)kMaxChunkBytes ? by_regs : (size_t)kMaxChunkBytes;
}

// Rank-coded image of a model of perfect trees of one depth (see fs_rank.hip): per feature the
// sorted distinct thresholds; per tree 2^(depth+1) words, word i = heap node i (1-based),
// splits as rank << 16 | offset of the feature in a rank tile, leaves as value bits; plus the caller's node id per word.
void build_rank_format(fs_model *m, int n_features, int n_trees, int depth, const int32_t *tree_off,
                       const int32_t *sf, const float *thr, const int32_t *left,
                       const int32_t *right, const float *val, std::vector<uint32_t> *nodes,
                       std::vector<uint16_t> *ids, std::vector<float> *cuts)
{
    // thresholds per feature: -0 joins +0, NaN thresholds never send anything left (rank 0)
    std::vector<std::vector<float>> per((size_t)n_features);
    const int64_t n_nodes = tree_off[n_trees];
    for (int64_t g = 0; g < n_nodes; ++g)
        if (sf[g] >= 0 && thr[g] == thr[g])
            per[(size_t)sf[g]].push_back(thr[g] + 0.0f);
    size_t max_cuts = 0;
    for (int f = 0; f < n_features; ++f) {
        std::vector<float> &v = per[(size_t)f];
        std::sort(v.begin(), v.end());
        v.erase(std::unique(v.begin(), v.end()), v.end());
        if (v.size() > max_cuts) max_cuts = v.size();
    }
    int bits = 2;                                         // stride of 2^bits entries per feature
    while ((((size_t)1 << bits) - 1) < max_cuts)
        ++bits;
    const size_t len = (size_t)1 << bits;
    if (bits > 15 || len * 4 > (size_t)kBinTableBytes)
        return;                                           // ranks must fit 16 bits and LDS
    // per feature: the sorted keys, padded with NaN to 2^bits - 1, as an implicit search tree in
    // breadth-first order: node 2^l + k (k-th of level l) holds sorted key (2k+1)*2^(bits-l-1) - 1
    cuts->assign(len * (size_t)n_features, __builtin_nanf(""));
    for (int f = 0; f < n_features; ++f) {
        const std::vector<float> &v = per[(size_t)f];
        float *tab = cuts->data() + (size_t)f * len;
        for (int l = 0; l < bits; ++l)
            for (size_t k = 0; k < ((size_t)1 << l); ++k) {
                const size_t sorted_idx = (2 * k + 1) * ((size_t)1 << (bits - l - 1)) - 1;
                if (sorted_idx < v.size())
                    tab[((size_t)1 << l) + k] = v[sorted_idx];
            }
    }

    const size_t words = (size_t)2 << depth;              // per tree, word 0 unused
    nodes->assign(words * (size_t)n_trees, 0u);
    ids->assign(words * (size_t)n_trees, 0);
    std::vector<int32_t> at(words);                       // caller's node at heap position i
    for (int t = 0; t < n_trees; ++t) {
        const int32_t o = tree_off[t];
        at[1] = 0;
        for (size_t i = 1; i < words; ++i) {
            const int32_t n = at[i];
            uint32_t w;
            if (sf[o + n] >= 0) {
                at[2 * i] = left[o + n];
                at[2 * i + 1] = right[o + n];
                const float th = thr[o + n];
                uint32_t rank = 0;
                if (th == th) {
                    const std::vector<float> &v = per[(size_t)sf[o + n]];
                    rank = 1u + (uint32_t)(std::lower_bound(v.begin(), v.end(), th + 0.0f) - v.begin());
                }
                w = (rank << 16) | rank_feature_offset(sf[o + n]);
            } else {
                memcpy(&w, &val[o + n], 4);
            }
            (*nodes)[(size_t)t * words + i] = w;
            (*ids)[(size_t)t * words + i] = (uint16_t)n;
        }
    }

    // tiles per workgroup (must divide the wavefront count): most (tiles x trees per chunk)
    const size_t tree_bytes = words * 4, tile_bytes = (size_t)rank_tile_cols(n_features) * 128;
    const size_t reg_limit = (size_t)kRankPrefetchRegs * 64 * kRankWaves * 16;
    int best_t = 0, best_per = 0, best_score = -1;
    const int forced = tune(FS_TUNE_RANK_TILES);
    const int choices[] = {6, 4, 3, 2, 1};
    for (int nt : choices) {
        if (forced > 0 && nt != forced)
            continue;
        const long avail = (long)kRankLdsBytes - (long)nt * (long)tile_bytes - 64;
        if (avail < (long)(tree_bytes + (size_t)nt * 256))
            continue;
        size_t per_c = (size_t)avail / (tree_bytes + (size_t)nt * 256);
        if (per_c > reg_limit / tree_bytes) per_c = reg_limit / tree_bytes;
        if (per_c > (size_t)kMaxChunkTrees) per_c = kMaxChunkTrees;
        if (per_c < 1)
            continue;
        int score = nt * (int)per_c;
        if (score > 64) score = 64;
        if (score > best_score) {
            best_score = score;
            best_t = nt;
            best_per = (int)per_c;
        }
    }
    if (best_t == 0)
        return;
    m->rank_ok = true;
    m->rk_depth = depth;
    m->rk_tiles = best_t;
    m->rk_trees_per_chunk = chunk_tree_target(n_trees, best_per, kRankWaves / best_t);
    m->rk_tree_bytes = (int32_t)tree_bytes;
    m->rk_tile0 = kRankLdsBytes - best_t * (int32_t)tile_bytes;
    m->cut_bits = bits;
    if (tune(FS_TUNE_VERBOSE) > 0)
        fprintf(stderr, "fs_model_create: rank-coded depth=%d tiles=%d trees/chunk=%d max_cuts=%zu\n",
                depth, best_t, best_per, max_cuts);
}

void free_device(fs_model *m)
{
    if (m->d_nodes) (void)hipFree(m->d_nodes);
    if (m->d_tree_off) (void)hipFree(m->d_tree_off);
    if (m->d_image) (void)hipFree(m->d_image);
    if (m->d_chunks) (void)hipFree(m->d_chunks);
    if (m->d_slot_ids) (void)hipFree(m->d_slot_ids);
    if (m->d_rk_nodes) (void)hipFree(m->d_rk_nodes);
    if (m->d_rk_ids) (void)hipFree(m->d_rk_ids);
    if (m->d_cuts) (void)hipFree(m->d_cuts);
}

template <typename T>
hipError_t upload(T **dst, const std::vector<T> &src)
{
    *dst = nullptr;
    if (src.empty())
        return hipSuccess;
    hipError_t e = hipMalloc((void **)dst, src.size() * sizeof(T));
    if (e != hipSuccess)
        return e;
    return hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice);
}

}  // namespace

extern "C" int fs_model_create(fs_model **out, int32_t n_features, int32_t n_trees,
                               const int32_t *tree_off, const int32_t *split_feature,
                               const float *threshold, const int32_t *left,
                               const int32_t *right, const float *value, float bias)
{
    if (!out)
        return fail(FS_EINVAL, "fs_model_create: out is NULL");
    *out = nullptr;
    if (n_features < 1 || n_features > FS_MAX_FEATURES)
        return fail(FS_EINVAL, "fs_model_create: n_features %d outside [1, %d]", n_features,
                    FS_MAX_FEATURES);
    if (n_trees < 0)
        return fail(FS_EINVAL, "fs_model_create: n_trees %d is negative", n_trees);
    if (!tree_off)
        return fail(FS_EINVAL, "fs_model_create: tree_off is NULL");
    if (tree_off[0] != 0)
        return fail(FS_EINVAL, "fs_model_create: tree_off[0] must be 0");
    for (int t = 0; t < n_trees; ++t) {
        int64_t sz = (int64_t)tree_off[t + 1] - tree_off[t];
        if (sz < 1 || sz > FS_MAX_TREE_NODES)
            return fail(FS_EINVAL, "fs_model_create: tree %d has %lld nodes (allowed 1..%d)", t,
                        (long long)sz, FS_MAX_TREE_NODES);
    }
    const int64_t n_nodes = tree_off[n_trees];
    if (n_nodes > 0 && (!split_feature || !threshold || !left || !right || !value))
        return fail(FS_EINVAL, "fs_model_create: a node array is NULL");

    try {
        // ---- validation + flat format ----
        std::vector<GNode> nodes((size_t)n_nodes);
        std::vector<int32_t> depth((size_t)n_nodes, 0);
        int32_t max_depth = 0;
        for (int t = 0; t < n_trees; ++t) {
            const int32_t o = tree_off[t];
            const int32_t sz = tree_off[t + 1] - o;
            for (int32_t n = 0; n < sz; ++n) {
                const int32_t g = o + n;
                GNode nd;
                if (split_feature[g] < 0) {
                    memcpy(&nd.x, &value[g], 4);
                    nd.y = -1;
                    nd.z = nd.w = g;
                } else {
                    if (split_feature[g] >= n_features)
                        return fail(FS_EINVAL, "fs_model_create: tree %d node %d splits on feature "
                                    "%d but the model has %d", t, n, split_feature[g], n_features);
                    if (left[g] <= n || left[g] >= sz || right[g] <= n || right[g] >= sz)
                        return fail(FS_EINVAL, "fs_model_create: tree %d node %d has child ids "
                                    "(%d, %d); they must lie in (%d, %d)", t, n, left[g], right[g],
                                    n, sz);
                    memcpy(&nd.x, &threshold[g], 4);
                    nd.y = split_feature[g];
                    nd.z = o + left[g];
                    nd.w = o + right[g];
                    const int32_t dl = depth[g] + 1;   // parents come before their children
                    if (depth[o + left[g]] < dl) depth[o + left[g]] = dl;
                    if (depth[o + right[g]] < dl) depth[o + right[g]] = dl;
                }
                if (depth[g] > max_depth)
                    max_depth = depth[g];
                nodes[(size_t)g] = nd;
            }
        }

        fs_model *m = new (std::nothrow) fs_model();
        if (!m)
            return fail(FS_ENOMEM, "fs_model_create: host allocation failed");
        memset(m, 0, sizeof(*m));
        m->n_features = n_features;
        m->n_trees = n_trees;
        m->max_depth = max_depth;
        m->n_nodes = n_nodes;
        m->bias = bias;

        // ---- LDS-staged format ----
        std::vector<uint8_t> image;
        std::vector<ChunkHdr> chunks;
        std::vector<uint16_t> slot_ids;
        const int tile_bytes = (n_features + 1) * 256;
        if (n_trees > 0 && n_features <= 255) {
            int common_depth = -1;
            bool compact = true;
            for (int t = 0; t < n_trees && compact; ++t) {
                const int32_t o = tree_off[t];
                compact = tree_is_perfect(split_feature + o, left + o, right + o,
                                          tree_off[t + 1] - o, &common_depth);
            }
            std::vector<PackedTree> trees((size_t)n_trees);
            size_t max_tree = 0, sum_tree = 0;
            bool all_trees = true;
            for (int t = 0; t < n_trees && all_trees; ++t) {
                const int32_t o = tree_off[t];
                all_trees = pack_tree(split_feature + o, threshold + o, left + o, right + o,
                                      value + o, tree_off[t + 1] - o, n_features, compact,
                                      common_depth, &trees[(size_t)t]);
                const size_t b = trees[(size_t)t].words.size() * 4;
                max_tree = b > max_tree ? b : max_tree;
                sum_tree += b;
            }
            const size_t avg_tree = sum_tree / (size_t)n_trees;
            // Pick the workgroup shape and the number of row tiles per workgroup.  More tiles
            // mean fewer passes of the model through LDS, but less room for trees; what hides
            // LDS latency is the number of independent walks in flight (tiles x trees
            // resident), so that comes first.  The small shape is taken when it still gets 8
            // or more trees into a chunk.
            int best_t = 0, best_score = -1, best_mode = 0;
            size_t best_avail = 0;
            const int forced_tiles = tune(FS_TUNE_LDS_TILES), forced_mode = tune(FS_TUNE_LDS_MODE);
            for (int mode = kLdsModes - 1; mode >= 0 && all_trees && best_t == 0; --mode) {
                // The half-LDS shape (two workgroups per compute unit) measured no faster on
                // any workload and doubles the model traffic from L2: tuning aid only.
                if (mode == 0 && forced_mode != 1)
                    continue;
                if (forced_mode >= 1 && forced_mode <= kLdsModes && mode != forced_mode - 1)
                    continue;
                const int max_tiles = mode == 0 ? 1 : kLdsMaxTiles;
                for (int nt = max_tiles; nt >= 1; --nt) {
                    if (mode == 1 && forced_tiles >= 1 && forced_tiles <= kLdsMaxTiles &&
                        nt != forced_tiles)
                        continue;
                    const long avail = (long)kLdsModeBytes[mode] - (long)nt * tile_bytes - 64;
                    const size_t per_tree_val = (size_t)nt * 256;
                    const size_t per_tree_tab = 4;   // a tree word of a run record
                    const size_t head = (size_t)(kLdsMaxWaves + 12) * kRunBytes + 16;   // records + padding
                    if (avail < (long)(max_tree + head + per_tree_val))
                        continue;
                    const size_t max_img = chunk_image_limit(mode);
                    if (max_img < max_tree + head)
                        continue;
                    size_t by_chunk = (max_img - head) / (avg_tree + per_tree_tab);
                    size_t by_avail = ((size_t)avail - head) / (avg_tree + per_tree_tab + per_tree_val);
                    size_t per = by_chunk < by_avail ? by_chunk : by_avail;
                    if (per < 1) per = 1;
                    if (per > (size_t)kMaxChunkTrees) per = kMaxChunkTrees;
                    if (mode == 0 && per < 8 && forced_mode != 1)
                        continue;
                    int score = nt * (int)per;
                    if (score > 64) score = 64;   // measured: beyond ~5 trees per wavefront more
                                                  // tiles win, below it more trees per chunk do
                    if (score > best_score) {
                        best_score = score;
                        best_t = nt;
                        best_mode = mode;
                        best_avail = (size_t)avail;
                    }
                }
            }
            if (best_t > 0 && tune(FS_TUNE_VERBOSE) > 0)
                fprintf(stderr, "fs_model_create: mode=%d tiles=%d avail=%zu avg_tree=%zu "
                        "max_tree=%zu compact=%d\n", best_mode, best_t, best_avail, avg_tree,
                        max_tree, (int)compact);
            if (best_t > 0) {
                const size_t per_tree_val = (size_t)best_t * 256;
                m->lds_ok = true;
                m->compact = compact;
                m->lds_tiles = best_t;
                m->lds_mode = best_mode;
                // Trees per chunk: estimated from the average tree, then balanced over the
                // wavefronts that share a tile (chunk_tree_target); a chunk ends early if its
                // trees are larger than average and the next one does not fit.
                const int share = kLdsModeWaves[best_mode] / best_t;
                const size_t img_limit = chunk_image_limit(best_mode);
                std::vector<int> tdepth((size_t)n_trees);
                for (int t = 0; t < n_trees; ++t)
                    tdepth[(size_t)t] = trees[(size_t)t].depth;
                // (every tree may need a run record of its own on top of the slots' first records)
                const size_t head0 = (size_t)kLdsMaxWaves * kRunBytes + 16;
                size_t est_per = (best_avail - head0) / (avg_tree + kRunBytes + per_tree_val);
                const size_t est_img = (img_limit - head0) / (avg_tree + kRunBytes);
                if (est_per > est_img) est_per = est_img;
                if (est_per > (size_t)kMaxChunkTrees) est_per = kMaxChunkTrees;
                if (est_per < 1) est_per = 1;
                const int even_cap = chunk_tree_target(n_trees, (int)est_per, share);
                std::vector<int> bounds(1, 0);
                for (int t = 0; t < n_trees;) {
                    int cnt = 0;
                    size_t body = 0;
                    while (t + cnt < n_trees && cnt < kMaxChunkTrees && cnt < even_cap) {
                        const size_t bt = trees[(size_t)(t + cnt)].words.size() * 4;
                        // run records in front of the nodes: at most one per slot and one per tree
                        const size_t img = ((size_t)(kLdsMaxWaves + cnt + 1) * kRunBytes + body + bt + 15) & ~(size_t)15;
                        if (img > img_limit || img + (size_t)(cnt + 1) * per_tree_val > best_avail)
                            break;
                        body += bt;
                        ++cnt;
                    }
                    t += cnt;                                 // cnt >= 1 by the choice of best_t
                    bounds.push_back(t);
                }
                for (size_t ci = 0; ci + 1 < bounds.size(); ++ci) {
                    const int t = bounds[ci], cnt = bounds[ci + 1] - bounds[ci];
                    size_t body = 0;
                    for (int j = 0; j < cnt; ++j)
                        body += trees[(size_t)(t + j)].words.size() * 4;
                    std::vector<int> by_depth((size_t)cnt);
                    for (int j = 0; j < cnt; ++j)
                        by_depth[(size_t)j] = j;
                    std::stable_sort(by_depth.begin(), by_depth.end(), [&](int x, int y) {
                        return tdepth[(size_t)(t + x)] > tdepth[(size_t)(t + y)];
                    });
                    SlotPlan sp;
                    deal_trees(by_depth, tdepth.data() + t, share, &sp);
                    // (the plan's cost is in units of about 1.5 us: configs[3] 12.1 for 18 us a group)
                    m->lds_group_us += 1.5f * (float)sp.cost;
                    // records: one per slot first (its first run, or an empty one), then the rest
                    std::vector<int> rec_of(sp.runs.size(), -1);     // record index of every run
                    int n_rec = kLdsMaxWaves;
                    for (int b = 0; b < share; ++b)
                        for (int r = sp.slot_start[b]; r < sp.slot_start[b + 1]; ++r)
                            rec_of[(size_t)r] = r == sp.slot_start[b] ? b : n_rec++;
                    const size_t table = ((size_t)n_rec * kRunBytes + 7) & ~(size_t)7;
                    const size_t bytes = (table + body + 15) & ~(size_t)15;
                    ChunkHdr h;
                    memset(&h, 0, sizeof(h));
                    h.byte_off = (uint32_t)image.size();
                    h.bytes = (uint32_t)bytes;
                    h.n_trees = (uint32_t)cnt;
                    h.first_tree = (uint32_t)t;
                    h.slot_off = (uint32_t)slot_ids.size();
                    image.resize(image.size() + bytes, 0);
                    slot_ids.resize(slot_ids.size() + bytes / 4, 0);
                    uint8_t *img = image.data() + h.byte_off;
                    uint16_t *ids = slot_ids.data() + h.slot_off;
                    size_t pos = table;
                    uint32_t dmax = 0;
                    std::vector<uint32_t> root_at((size_t)cnt);
                    for (int j = 0; j < cnt; ++j) {
                        PackedTree &pt = trees[(size_t)(t + j)];
                        const uint32_t base = (uint32_t)pos;
                        root_at[(size_t)j] = base;
                        for (uint32_t wi : pt.fix) {
                            const uint32_t w = pt.words[wi];
                            pt.words[wi] = (w & 0xFFFF0000u) | (((w & 0xFFFFu) + base) & 0xFFFFu);
                        }
                        memcpy(img + pos, pt.words.data(), pt.words.size() * 4);
                        memcpy(ids + pos / 4, pt.slot_ids.data(), pt.slot_ids.size() * 2);
                        pos += pt.words.size() * 4;
                        if ((uint32_t)pt.depth > dmax) dmax = (uint32_t)pt.depth;
                    }
                    h.depth = dmax;
                    for (int b = 0; b < share; ++b)
                        for (int r = sp.slot_start[b]; r < sp.slot_start[b + 1]; ++r) {
                            const RunPlan &rp = sp.runs[(size_t)r];
                            const int next = r + 1 < sp.slot_start[b + 1] ? rec_of[(size_t)(r + 1)] + 1 : 0;
                            uint32_t rec[kRunWords];
                            rec[0] = (uint32_t)rp.count | ((uint32_t)next << 4) | ((uint32_t)rp.depth << 16);
                            for (int k = 0; k < 8; ++k) {
                                const int j = sp.order[(size_t)(rp.first + (k < rp.count ? k : 0))];
                                rec[1 + k] = root_at[(size_t)j] | ((uint32_t)j << 16);
                            }
                            memcpy(img + (size_t)rec_of[(size_t)r] * kRunBytes, rec, sizeof(rec));
                        }
                    chunks.push_back(h);
                }
                if (tune(FS_TUNE_VERBOSE) > 0) {
                    fprintf(stderr, "fs_model_create: %zu chunks, trees per chunk:", chunks.size());
                    for (const ChunkHdr &c : chunks)
                        fprintf(stderr, " %u", c.n_trees);
                    fprintf(stderr, "\n");
                }
                m->n_chunks = (int32_t)chunks.size();
                m->image_bytes = image.size();
                m->lds_tile0 = kLdsModeBytes[best_mode] - best_t * tile_bytes;
            }
        }

        // ---- rank-coded format: deep perfect trees ----
        std::vector<uint32_t> rk_nodes;
        std::vector<uint16_t> rk_ids;
        std::vector<float> cuts;
        {
            const int want = tune(FS_TUNE_RANK);   // -1 automatic, 0 never, 1 whenever possible
            int depth = -1;
            bool perfect = n_trees > 0 && n_features <= 511 && want != 0;
            for (int t = 0; t < n_trees && perfect; ++t) {
                const int32_t o = tree_off[t];
                perfect = tree_is_perfect(split_feature + o, left + o, right + o, tree_off[t + 1] - o,
                                          &depth);
            }
            // measured: pays from depth 8 on (3 KB per tree in the 8-byte-node format)
            if (perfect && (want == 1 || depth >= 8) && depth <= 12)
                build_rank_format(m, n_features, n_trees, depth, tree_off, split_feature, threshold,
                                  left, right, value, &rk_nodes, &rk_ids, &cuts);
        }

        hipError_t e = hipGetDevice(&m->device);
        if (e == hipSuccess) {
            std::vector<int32_t> toff(tree_off, tree_off + n_trees + 1);
            e = upload(&m->d_tree_off, toff);
        }
        if (e == hipSuccess) e = upload(&m->d_nodes, nodes);
        if (e == hipSuccess) e = upload(&m->d_image, image);
        if (e == hipSuccess) e = upload(&m->d_chunks, chunks);
        if (e == hipSuccess) e = upload(&m->d_slot_ids, slot_ids);
        if (e == hipSuccess && m->rank_ok) {
            e = upload(&m->d_rk_nodes, rk_nodes);
            if (e == hipSuccess) e = upload(&m->d_rk_ids, rk_ids);
            if (e == hipSuccess) e = upload(&m->d_cuts, cuts);
        }
        if (e != hipSuccess) {
            free_device(m);
            delete m;
            return fail_hip(e, "fs_model_create: device upload");
        }
        *out = m;
        return FS_OK;
    } catch (const std::bad_alloc &) {
        return fail(FS_ENOMEM, "fs_model_create: host allocation failed");
    }
}

extern "C" void fs_model_destroy(fs_model *m)
{
    if (!m)
        return;
    free_device(m);
    delete m;
}
