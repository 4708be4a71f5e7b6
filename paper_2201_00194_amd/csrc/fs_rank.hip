// Rank-coded scoring for models of deep perfect trees.
//
// A split "x[f] < thr" only asks how x[f] orders against the thresholds the model itself
// uses on feature f.  Let cuts_f be those thresholds, sorted and distinct, and
//     rank(x) = number of cuts_f that are <= x            (NaN: 65535)
//     rank(thr) = 1 + position of thr in cuts_f           (NaN threshold: 0)
// then  x < thr  <=>  rank(x) < rank(thr), exactly: the walk over 16-bit ranks reaches the
// same leaves as the walk over the fp32 values (Section 4.2 of the paper: the family's model
// estimates each candidate; nothing in the estimate changes).  What it buys: a feature tile
// takes 2 bytes per value instead of 4 and a split node 4 bytes instead of 8, so a compute
// unit's LDS holds twice the rows and twice the trees -- deep trees otherwise leave room for
// only a handful of trees per chunk and the model has to stream through LDS once per 128 rows.
//
// Two kernels:
//   rank_code_kernel     fp32 feature tiles -> u16 rank tiles (binary search in LDS-resident
//                        threshold tables, one feature group per workgroup)
//   traverse_rank_kernel the LDS-staged walk over rank tiles; trees in heap order without
//                        child pointers (node i has children 2i, 2i+1, 1-based), leaves are the
//                        last level; tile-sharing wavefronts, parked leaf values and the
//                        ordered per-row sum as in the fp32 kernel
#include "fs_internal.h"
#include "fs_lds.h"

namespace fs {

// ------------------------------------------------------------------------------------------------
// rank coding
// ------------------------------------------------------------------------------------------------
constexpr int kBinThreads = 1024;

// Every feature's thresholds are padded with NaN to 2^q - 1 keys (q the same for all features
// of a model) and stored as an implicit search tree in breadth-first order (word 0 unused,
// node i has children 2i and 2i+1).  The count of keys <= x is then a branch-free descent
// with q fixed steps,   i = 2i + (key[i] <= x),   rank = i - 2^q   (NaN padding never compares
// <=).  Breadth-first order matters on this memory: the nodes of one level are neighbours, so
// the lanes' reads spread over the LDS banks, whereas the probes of a bisection of the sorted
// array are a power-of-two stride apart and all fall into the same bank.  Four searches run
// interleaved per wavefront.
constexpr int kBinChains = 4;

__global__ void __launch_bounds__(kBinThreads, 8)     // two workgroups per compute unit
rank_code_kernel(const FamDesc *__restrict__ descs, int n_families)
{
    int lo = 0, hi = n_families - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (descs[mid].bin_block0 <= (int)blockIdx.x)
            lo = mid;
        else
            hi = mid - 1;
    }
    const FamDesc &d = descs[lo];
    const int local = blockIdx.x - d.bin_block0;
    const int group = local % d.bin_groups, tile_block = local / d.bin_groups;
    const int F = d.n_features;
    const int f0 = group * d.bin_feats_per_group;
    const int gf = min(d.bin_feats_per_group, F - f0);
    const int n_tiles = (d.n_rows + 63) >> 6;
    const int tpb = d.bin_tiles_per_block;
    const int t0 = tile_block * tpb;
    const int nt = min(tpb, n_tiles - t0);
    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const int q = d.cut_bits;                       // table stride 2^q entries
    const int len = 1 << q;

    // this group's padded threshold tables: one contiguous, 16-byte aligned run, straight from
    // memory to LDS (what is left below 64 pieces goes through a register)
    {
        auto cuts = FS_GLOBAL(const u32x4, d.cuts + (int64_t)f0 * len);
        const int n16 = gf * len / 4;
        const int rest = lds_fill_direct(cuts, 0u, n16, wave, kBinThreads / 64, lane) + tid;
        if (rest < n16)
            lds_store_u4(16u * (uint32_t)rest, cuts[rest]);
        lds_direct_wait();
    }
    __syncthreads();

    auto X = FS_GLOBAL(const float, d.features);
    auto R = FS_GLOBAL(uint16_t, d.ranks);
    // A wavefront takes tiles wave, wave+16, ... of the block and, per tile, the group's
    // features four at a time (one search chain each).  The next round's values are fetched
    // while the current round is searched.
    const int n_waves = kBinThreads / 64;
    const int rounds_per_tile = (gf + kBinChains - 1) / kBinChains;
    // Element (tile, feature f0 + j, lane) of the input: column-blocked tiles, or row-major rows
    // (the row index is clamped: the last tile of a row-major matrix has no padding rows).
    const bool rowmajor = d.layout == FS_ROWMAJOR;
    auto x_at = [&](int tile, int j) -> int64_t {
        if (rowmajor)
            return (int64_t)min(tile * 64 + lane, d.n_rows - 1) * F + f0 + j;
        return ((int64_t)tile * F + f0 + j) * 64 + lane;
    };
    int t = wave, jg = 0;                            // current round: tile t, features 4*jg..
    float xn[kBinChains];
    if (t < nt) {
#pragma unroll
        for (int k = 0; k < kBinChains; ++k)
            xn[k] = X[x_at(t0 + t, min(k, gf - 1))];
    }
    while (t < nt) {
        const int j0 = jg * kBinChains;
        const int64_t base = (int64_t)(t0 + t) * rank_tile_cols(F) * 64 + 2 * lane;   // u16 units
        float x[kBinChains];
        uint32_t pos[kBinChains], tab[kBinChains];
#pragma unroll
        for (int k = 0; k < kBinChains; ++k) {
            x[k] = xn[k];
            tab[k] = 4u * (uint32_t)(min(j0 + k, gf - 1) * len);
            pos[k] = 1u;                             // node of the implicit search tree
        }
        // next round
        int tn = t, jn = jg + 1;
        if (jn == rounds_per_tile) {
            jn = 0;
            tn = t + n_waves;
        }
        if (tn < nt) {
#pragma unroll
            for (int k = 0; k < kBinChains; ++k)
                xn[k] = X[x_at(t0 + tn, min(jn * kBinChains + k, gf - 1))];
        }
        for (int s = 0; s < q; ++s) {
            float c[kBinChains];
#pragma unroll
            for (int k = 0; k < kBinChains; ++k)
                c[k] = lds_f(tab[k] + 4u * pos[k]);
#pragma unroll
            for (int k = 0; k < kBinChains; ++k)
                pos[k] = 2u * pos[k] + ((c[k] <= x[k]) ? 1u : 0u);
        }
        uint32_t r[kBinChains];
#pragma unroll
        for (int k = 0; k < kBinChains; ++k)
            r[k] = (x[k] != x[k]) ? 65535u : (pos[k] - (uint32_t)len);
        if ((f0 & 1) == 0) {
            // chains 2i and 2i+1 hold the two features of one word of the tile
            auto R2 = FS_GLOBAL(uint32_t, d.ranks);
#pragma unroll
            for (int k = 0; k < kBinChains; k += 2) {
                const int64_t at = base + (rank_feature_offset(f0 + j0 + k) >> 1);   // even
                if (j0 + k + 1 < gf)
                    R2[at >> 1] = r[k] | (r[k + 1] << 16);
                else if (j0 + k < gf)
                    R[at] = (uint16_t)r[k];
            }
        } else {
#pragma unroll
            for (int k = 0; k < kBinChains; ++k)
                if (j0 + k < gf)
                    R[base + (rank_feature_offset(f0 + j0 + k) >> 1)] = (uint16_t)r[k];
        }
        t = tn;
        jg = jn;
    }
}

int launch_rank_code(const FamDesc *d_desc, int n_families, int total_blocks, hipStream_t stream)
{
    static bool configured[16] = {};
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 16 || !configured[dev]) {
        hipFuncAttributes attr;
        FS_HIP(hipFuncGetAttributes(&attr, (const void *)rank_code_kernel));
        if (attr.sharedSizeBytes != 0)
            return fail(FS_EDEVICE, "rank_code_kernel was built with %zu bytes of static LDS",
                        (size_t)attr.sharedSizeBytes);
        FS_HIP(hipFuncSetAttribute((const void *)rank_code_kernel,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kBinTableBytes));
        if (dev >= 0 && dev < 16)
            configured[dev] = true;
    }
    hipLaunchKernelGGL(rank_code_kernel, dim3(total_blocks), dim3(kBinThreads), kBinTableBytes,
                       stream, d_desc, n_families);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "rank_code_kernel launch");
    return FS_OK;
}

// ------------------------------------------------------------------------------------------------
// traversal over rank tiles
// ------------------------------------------------------------------------------------------------
// LDS map:  [0, trees*tree_bytes)               current chunk: trees back to back, each
//                                               2^(depth+1) words: [unused][splits in heap
//                                               order, 1-based][leaf values]
//           [tile0 - trees*T*256, tile0)        leaf values parked per [tree][tile][lane]
//           [tile0 + t*Fc*128, ...)             tile t: features 2i, 2i+1 of row l in the word at
//                                               i*256 + 4*l (Fc = F rounded up to even)
// A split word is rank(thr) << 16 | offset of the feature in a tile (i*256 + 2*(f & 1)).

// K trees at once for this lane's row.  base[k] = LDS address of tree k; the 1-based heap
// index i lives at A = base + 4*i, and the step i' = 2i + c is taken on the address itself:
// A' = 2A + (4c - base)   (one select between two per-tree constants and one shift-add).
template <int K>
__device__ __forceinline__ void rank_walk(const uint32_t (&base)[K], int depth, uint32_t lane_base,
                                          uint32_t (&idx)[K], float (&v)[K])
{
    uint32_t A[K], left[K], right[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        A[k] = base[k] + 4u;
        left[k] = 0u - base[k];
        right[k] = 4u - base[k];
        // keep the two constants as they are: the compiler would otherwise fold the select
        // into select(0,4) - base and spend two more instructions per visit
        asm volatile("" : "+v"(left[k]), "+v"(right[k]));
    }
    for (int l = 0; l < depth; ++l) {
        uint32_t nd[K], x[K];
#pragma unroll
        for (int k = 0; k < K; ++k)
            nd[k] = lds_u(A[k]);
#pragma unroll
        for (int k = 0; k < K; ++k)
            x[k] = lds_u16((nd[k] & 0xFFFFu) + lane_base);
#pragma unroll
        for (int k = 0; k < K; ++k)
            A[k] = (A[k] << 1) + ((x[k] < (nd[k] >> 16)) ? left[k] : right[k]);
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        v[k] = lds_f(A[k]);
        idx[k] = (A[k] - base[k]) >> 2;
    }
}

template <int K, bool DUMP>
__device__ __forceinline__ void rank_walk_k(int g, int depth, uint32_t tree_bytes,
                                            uint32_t lane_base, uint32_t val_addr,
                                            uint32_t val_stride, const uint16_t *ids_,
                                            uint16_t *leaf_out_)
{
    uint32_t base[K], idx[K];
    float v[K];
#pragma unroll
    for (int k = 0; k < K; ++k)
        base[k] = (uint32_t)(g + k) * tree_bytes;
    rank_walk<K>(base, depth, lane_base, idx, v);
#pragma unroll
    for (int k = 0; k < K; ++k)
        lds_store_f(val_addr + (uint32_t)(g + k) * val_stride, v[k]);
    if (DUMP) {
        if (leaf_out_) {
            auto ids = FS_GLOBAL(const uint16_t, ids_);
            auto leaf_out = FS_GLOBAL(uint16_t, leaf_out_);
            const uint32_t per_tree = tree_bytes >> 2;
#pragma unroll
            for (int k = 0; k < K; ++k)
                leaf_out[g + k] = ids[(uint32_t)(g + k) * per_tree + idx[k]];
        }
    }
}

template <bool DUMP>
__device__ __forceinline__ void rank_walk_n(int count, int g, int depth, uint32_t tree_bytes,
                                            uint32_t lane_base, uint32_t val_addr,
                                            uint32_t val_stride, const uint16_t *ids,
                                            uint16_t *leaf_out)
{
    switch (count) {
    case 8: rank_walk_k<8, DUMP>(g, depth, tree_bytes, lane_base, val_addr, val_stride, ids, leaf_out); break;
    case 7: rank_walk_k<7, DUMP>(g, depth, tree_bytes, lane_base, val_addr, val_stride, ids, leaf_out); break;
    case 6: rank_walk_k<6, DUMP>(g, depth, tree_bytes, lane_base, val_addr, val_stride, ids, leaf_out); break;
    case 5: rank_walk_k<5, DUMP>(g, depth, tree_bytes, lane_base, val_addr, val_stride, ids, leaf_out); break;
    case 4: rank_walk_k<4, DUMP>(g, depth, tree_bytes, lane_base, val_addr, val_stride, ids, leaf_out); break;
    case 3: rank_walk_k<3, DUMP>(g, depth, tree_bytes, lane_base, val_addr, val_stride, ids, leaf_out); break;
    case 2: rank_walk_k<2, DUMP>(g, depth, tree_bytes, lane_base, val_addr, val_stride, ids, leaf_out); break;
    case 1: rank_walk_k<1, DUMP>(g, depth, tree_bytes, lane_base, val_addr, val_stride, ids, leaf_out); break;
    default: break;
    }
}

constexpr int kRankThreads = 64 * kRankWaves;
constexpr int kRankTileBatch = 11;   // 16-byte loads in flight per thread while tiles are fetched
                                     // (six 164-feature rank tiles are 10.25 pieces per thread)

template <bool DUMP>
__global__ void __launch_bounds__(kRankThreads)
traverse_rank_kernel(const FamDesc *__restrict__ descs, int n_families)
{
    int lo = 0, hi = n_families - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (descs[mid].rk_block0 <= (int)blockIdx.x)
            lo = mid;
        else
            hi = mid - 1;
    }
    const FamDesc &d = descs[lo];
    const int tid = threadIdx.x;
    const int wave = uniform(tid >> 6), lane = tid & 63;
    const int T = d.rk_tiles;                   // tiles per workgroup (divides 12)
    const int S = kRankWaves / T;               // wavefronts sharing a tile
    const int my_tile = wave % T, my_slot = wave / T;
    const int n_tiles = (d.n_rows + 63) >> 6;
    const int tile_first = (blockIdx.x - d.rk_block0) * T;
    const int tiles_here = min(T, n_tiles - tile_first);
    const bool active = my_tile < tiles_here;
    const int F = d.n_features;
    const int Fc = rank_tile_cols(F);
    const uint32_t tile_bytes = (uint32_t)Fc * 128u;
    const uint32_t tile0 = (uint32_t)d.rk_tile0;
    const uint32_t lane_base = tile0 + (uint32_t)my_tile * tile_bytes + 4u * (uint32_t)lane;
    const uint32_t tree_bytes = (uint32_t)d.rk_tree_bytes;
    const int per_chunk = d.rk_trees_per_chunk;
    const int n_trees = d.n_trees;
    const int depth = d.rk_depth;
    const int n_chunks = (n_trees + per_chunk - 1) / per_chunk;
    // tree_bytes = 2^(depth+3) is a multiple of 16, so every chunk starts 16-byte aligned

    // ---- first chunk: global -> registers ----
    u32x4 pf[kRankPrefetchRegs];
    auto image = FS_GLOBAL(const u32x4, d.rk_nodes);
    const int tree16 = (int)(tree_bytes >> 4);
    // The first chunk and the tiles go straight from memory to LDS, 1 KB per wavefront-wide
    // load; what is left of each (fewer than 64 pieces) goes through registers.
    const int first16 = min(per_chunk, n_trees) * tree16;
    const int first_rest = lds_fill_direct(image, 0u, first16, wave, kRankWaves, lane) + tid;
    if (first_rest < first16)
        pf[0] = image[first_rest];
    // ---- rank tiles: consecutive tiles are one contiguous run ----
    {
        auto src = FS_GLOBAL(const u32x4, d.ranks + (int64_t)tile_first * Fc * 64);
        const int per_tile = Fc * 8;                       // 16-byte pieces per tile
        const int n16 = tiles_here * per_tile;
        const int done = lds_fill_direct(src, tile0, n16, wave, kRankWaves, lane);
        for (int base = done + tid; base < n16; base += kRankTileBatch * kRankThreads) {
            u32x4 t4[kRankTileBatch];
#pragma unroll
            for (int q = 0; q < kRankTileBatch; ++q)
                t4[q] = src[min(base + q * kRankThreads, n16 - 1)];
#pragma unroll
            for (int q = 0; q < kRankTileBatch; ++q) {
                const int i = base + q * kRankThreads;
                if (i < n16)
                    lds_store_u4(tile0 + 16u * (uint32_t)i, t4[q]);   // tiles are contiguous in LDS too
            }
        }
    }
    if (first_rest < first16)
        lds_store_u4(16u * (uint32_t)first_rest, pf[0]);
    lds_direct_wait();
    __syncthreads();

    const int r = (tile_first + my_tile) * 64 + lane;
    float acc = d.bias;
    uint16_t *leaf_row = nullptr;
    if (DUMP) {
        if (active && d.leaf_idx && r < d.n_rows)
            leaf_row = d.leaf_idx + (int64_t)r * n_trees;
    }
    const uint32_t val_stride = (uint32_t)T * 256u;

    // Wavefronts 0..T-1 do the ordered sums.  When the others can carry a whole chunk in their
    // prefetch registers they copy it alone, so a sum and the copy run side by side.
    const int n_copiers = kRankThreads - 64 * T;
    for (int c = 0; c < n_chunks; ++c) {
        const int first = c * per_chunk;
        const int n = uniform(min(per_chunk, n_trees - first));
        int n_next = 0, cp_id = tid, cp_n = kRankThreads;
        if (c + 1 < n_chunks) {                            // next chunk: global -> registers
            n_next = min(per_chunk, n_trees - first - per_chunk);
            const int n16 = n_next * tree16;
            auto src = image + (int64_t)(first + per_chunk) * tree16;
            if (n16 <= kRankPrefetchRegs * n_copiers) {
                cp_n = n_copiers;
                cp_id = tid - 64 * T;                      // negative in the summing wavefronts
            }
            if (cp_id >= 0) {
#pragma unroll
                for (int j = 0; j < kRankPrefetchRegs; ++j)
                    pf[j] = src[min(cp_id + j * cp_n, n16 - 1)];
            }
        }
        const uint32_t val0 = tile0 - (uint32_t)per_chunk * val_stride;   // fixed: above any image
        if (active) {
            const uint32_t val_addr = val0 + (uint32_t)my_tile * 256u + 4u * (uint32_t)lane;
            const uint16_t *ids = d.rk_ids + (int64_t)first * (tree_bytes >> 2);
            uint16_t *leaf_out = leaf_row ? leaf_row + first : nullptr;
            const int n_groups = S * ((n + 8 * S - 1) / (8 * S));
            const int base = n / n_groups, rem = n - base * n_groups;
            for (int j = my_slot; j < n_groups; j += S) {
                const int g = j * base + min(j, rem);
                const int count = base + (j < rem ? 1 : 0);
                rank_walk_n<DUMP>(count, g, depth, tree_bytes, lane_base, val_addr, val_stride, ids,
                                  leaf_out);
            }
        }
        __syncthreads();       // every walk of this chunk is done and its values are parked
        if (active && my_slot == 0) {
            const uint32_t va = val0 + (uint32_t)my_tile * 256u + 4u * (uint32_t)lane;
            ordered_add_n(acc, va, val_stride, n);
        }
        if (c + 1 < n_chunks) {
            const int n16 = n_next * tree16;
            if (cp_id >= 0) {
#pragma unroll
                for (int j = 0; j < kRankPrefetchRegs; ++j) {
                    const int i = cp_id + j * cp_n;
                    if (i < n16)
                        lds_store_u4(16u * (uint32_t)i, pf[j]);
                }
            }
            __syncthreads();
        }
    }
    if (active && my_slot == 0 && r < d.n_rows)
        FS_GLOBAL(float, d.row_score)[r] = acc;
}

int launch_traverse_rank(const FamDesc *d_desc, int n_families, int total_blocks, bool dump,
                         hipStream_t stream)
{
    static bool configured[16][2] = {};
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    const void *fn = dump ? (const void *)traverse_rank_kernel<true>
                          : (const void *)traverse_rank_kernel<false>;
    if (dev < 0 || dev >= 16 || !configured[dev][dump ? 1 : 0]) {
        hipFuncAttributes attr;
        FS_HIP(hipFuncGetAttributes(&attr, fn));
        if (attr.sharedSizeBytes != 0)
            return fail(FS_EDEVICE, "traverse_rank_kernel was built with %zu bytes of static LDS",
                        (size_t)attr.sharedSizeBytes);
        FS_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kRankLdsBytes));
        if (dev >= 0 && dev < 16)
            configured[dev][dump ? 1 : 0] = true;
    }
    if (dump)
        hipLaunchKernelGGL(traverse_rank_kernel<true>, dim3(total_blocks), dim3(kRankThreads),
                           kRankLdsBytes, stream, d_desc, n_families);
    else
        hipLaunchKernelGGL(traverse_rank_kernel<false>, dim3(total_blocks), dim3(kRankThreads),
                           kRankLdsBytes, stream, d_desc, n_families);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "traverse_rank_kernel launch");
    return FS_OK;
}

}  // namespace fs
