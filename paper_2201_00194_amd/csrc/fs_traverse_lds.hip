// LDS-staged traversal: the hot kernel of fs_score_families.
//
// The family's model estimates every candidate (Section 4.2 of the paper); here that is,
// per statement row, a walk through every tree and a sum of the reached leaves in tree
// order.
//
// A workgroup (6 wavefronts and one tile on half a compute unit's LDS, or 12 wavefronts and
// up to three tiles on all of it) holds its 64-row feature tiles in LDS in the
// column-blocked layout they have in HBM: row l of a tile is lane l, and column j sits at
// j*256 + l*4, so a gather of 64 different features by 64 lanes touches 64 different
// words in 64 different banks (no conflict whatever the features are).  The model streams
// through LDS in chunks.  The wavefronts that share a tile split the chunk's trees among
// themselves and every lane walks several trees at once; that keeps 24 or more independent
// walks in flight per compute unit, which is what hides the LDS latency.  Each walk ends
// by parking its leaf value in LDS; one wavefront per tile then adds the chunk's values to
// the row's running sum in tree order, so the row score has the bits of a plain
// sequential fp32 sum.  The next chunk is fetched into registers while the current one is
// being walked.  A chunk's trees are cut into runs of similar depth that are dealt to the
// wavefronts (run records at the head of the chunk image).
//
// In a long launch a workgroup takes several consecutive groups of tiles (MULTI): only the
// first group's tiles are fetched with nothing else to do; the next group's tiles, and the
// model's first chunk again, are fetched into registers while the last chunk of the current
// group is being walked, and stored to LDS once those walks are done.
//
// LDS map:  [0, chunk bytes)                    current model chunk (node offsets are
//                                               absolute LDS addresses)
//           [tile0 - trees*tiles*256, tile0)    leaf values [tree][tile][lane]
//           [tile0 + t*tile, ... + tile)        tile t, tile = (F+1)*256 B; column F is all
//                                               NaN: a leaf "splits" on it, fails '<' and
//                                               stays where it is
#include "fs_internal.h"
#include "fs_lds.h"

namespace fs {

constexpr int kTileBatch = 8;    // 16-byte loads in flight per thread while tiles are fetched

// One run: K trees of the current chunk, walked side by side for this lane's row to `depth`
// split levels (the depth of the run's deepest tree; a walk that reaches its leaf earlier stays
// there).  `tab` holds the tree words of the run record (root offset | place in the chunk).
// Every walk parks its leaf value in the value row of its tree; DUMP also reports the leaf ids.
// COMPACT: perfect trees with 4-byte leaves, so the last split level steps by 4.
template <int K, bool COMPACT, bool DUMP>
__device__ __forceinline__ void walk_k(const uint32_t (&tab)[8], int depth, uint32_t lane_base,
                                       uint32_t val_addr, uint32_t val_stride,
                                       const uint16_t *slot_ids_, uint16_t *leaf_out_)
{
    auto slot_ids = FS_GLOBAL(const uint16_t, slot_ids_);
    auto leaf_out = FS_GLOBAL(uint16_t, leaf_out_);
    uint32_t a[K];
    float v[K];
#pragma unroll
    for (int k = 0; k < K; ++k)
        a[k] = tab[k] & 0xFFFFu;
    const int full_levels = COMPACT ? depth - 1 : depth;
    for (int l = 0; l < full_levels; ++l) {
        u32x2 nd[K];
        float x[K];
#pragma unroll
        for (int k = 0; k < K; ++k)
            nd[k] = lds_u2(a[k]);
#pragma unroll
        for (int k = 0; k < K; ++k)
            x[k] = lds_f((nd[k].y >> 16) + lane_base);
#pragma unroll
        for (int k = 0; k < K; ++k)
            a[k] = (nd[k].y & 0xFFFFu) + ((x[k] < __uint_as_float(nd[k].x)) ? 0u : 8u);
    }
    if (COMPACT) {
        u32x2 nd[K];
        float x[K];
#pragma unroll
        for (int k = 0; k < K; ++k)
            nd[k] = lds_u2(a[k]);
#pragma unroll
        for (int k = 0; k < K; ++k)
            x[k] = lds_f((nd[k].y >> 16) + lane_base);
#pragma unroll
        for (int k = 0; k < K; ++k)
            a[k] = (nd[k].y & 0xFFFFu) + ((x[k] < __uint_as_float(nd[k].x)) ? 0u : 4u);
    }
#pragma unroll
    for (int k = 0; k < K; ++k)
        v[k] = lds_f(a[k]);
#pragma unroll
    for (int k = 0; k < K; ++k)
        lds_store_f(val_addr + (tab[k] >> 16) * val_stride, v[k]);
    if (DUMP) {
        if (leaf_out_) {
#pragma unroll
            for (int k = 0; k < K; ++k)
                leaf_out[tab[k] >> 16] = slot_ids[a[k] >> 2];
        }
    }
}

template <bool COMPACT, bool DUMP>
__device__ __forceinline__ void walk_n(int count, const uint32_t (&tab)[8], int depth, uint32_t lane_base,
                                       uint32_t val_addr, uint32_t val_stride,
                                       const uint16_t *slot_ids, uint16_t *leaf_out)
{
    switch (count) {
    case 8: walk_k<8, COMPACT, DUMP>(tab, depth, lane_base, val_addr, val_stride, slot_ids, leaf_out); break;
    case 7: walk_k<7, COMPACT, DUMP>(tab, depth, lane_base, val_addr, val_stride, slot_ids, leaf_out); break;
    case 6: walk_k<6, COMPACT, DUMP>(tab, depth, lane_base, val_addr, val_stride, slot_ids, leaf_out); break;
    case 5: walk_k<5, COMPACT, DUMP>(tab, depth, lane_base, val_addr, val_stride, slot_ids, leaf_out); break;
    case 4: walk_k<4, COMPACT, DUMP>(tab, depth, lane_base, val_addr, val_stride, slot_ids, leaf_out); break;
    case 3: walk_k<3, COMPACT, DUMP>(tab, depth, lane_base, val_addr, val_stride, slot_ids, leaf_out); break;
    case 2: walk_k<2, COMPACT, DUMP>(tab, depth, lane_base, val_addr, val_stride, slot_ids, leaf_out); break;
    case 1: walk_k<1, COMPACT, DUMP>(tab, depth, lane_base, val_addr, val_stride, slot_ids, leaf_out); break;
    default: break;
    }
}

// The fields of a chunk header the kernel keeps in (scalar) registers.
struct ChunkView {
    uint32_t byte_off, bytes, n_trees, first_tree, slot_off;
};

__device__ __forceinline__ ChunkView load_chunk(const ChunkHdr *hdr_)
{
    auto hdr = FS_CONST(ChunkHdr, hdr_);
    ChunkView v;
    v.byte_off = hdr->byte_off;
    v.bytes = hdr->bytes;
    v.n_trees = hdr->n_trees;
    v.first_tree = hdr->first_tree;
    v.slot_off = hdr->slot_off;
    return v;
}

template <bool DUMP, bool MULTI>
__global__ void __launch_bounds__(64 * kLdsMaxWaves)
traverse_lds_kernel(const FamDesc *__restrict__ descs, int n_families, int mode, int groups_per_wg)
{
    const int kLdsThreads = blockDim.x;
    const int kLdsWaves = kLdsThreads >> 6;
    int lo = 0, hi = n_families - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (descs[mid].lds_block0[mode] <= (int)blockIdx.x)
            lo = mid;
        else
            hi = mid - 1;
    }
    const FamDesc &d = descs[lo];
    const int tid = threadIdx.x;
    const int wave = uniform(tid >> 6), lane = tid & 63;
    const int T = d.lds_tiles;                  // tiles per workgroup
    const int my_tile = wave % T, my_slot = wave / T;
    const int n_tiles = (d.n_rows + 63) >> 6;
    const int F = d.n_features;
    // A workgroup takes several consecutive tile groups when the next group's tiles can wait in
    // registers (column-blocked input whose tiles fit kLdsTileRegs pieces per thread): they are
    // fetched while the last chunk of the current group is walked.
    const int n_groups = (n_tiles + T - 1) / T;
    const int G = MULTI ? lds_groups_per_wg(d.layout, F, T, kLdsThreads, groups_per_wg) : 1;
    const int g_first = (blockIdx.x - d.lds_block0[mode]) * G;
    const int g_end = min(g_first + G, n_groups);
    const uint32_t tile_bytes = (uint32_t)(F + 1) * 256u;
    const uint32_t tile0 = (uint32_t)d.lds_tile0;
    const uint32_t lane_base = tile0 + (uint32_t)my_tile * tile_bytes + 4u * (uint32_t)lane;
    const int per_tile = F * 16;                           // 16-byte pieces per tile
    u32x4 pf[kPrefetchRegs];
    ChunkView h = load_chunk(d.chunks);
    {
        // the workgroup's first group: chunk and tiles straight from memory
        const int tile_first = g_first * T;
        const int tiles_here = min(T, n_tiles - tile_first);

        // ---- first chunk: global -> registers (lands while the tiles are being fetched) ----
        // Loads are unconditional with clamped indices (no branches between them, so they all go
        // out back to back); only the LDS writes are predicated.
        // (Row-major input stages its rows at LDS offset 0 first, so there the chunk waits in
        // registers; column-blocked input lets chunk and tiles go straight from memory to LDS.)
        const bool direct = d.layout != FS_ROWMAJOR;
        {
            auto src = FS_GLOBAL(const u32x4, d.image + h.byte_off);
            const int n16 = (int)(h.bytes >> 4);
            if (direct) {
                const int done = lds_fill_direct(src, 0u, n16, wave, kLdsWaves, lane);
                if (done + tid < n16)
                    pf[0] = src[done + tid];                   // fewer than 64 pieces are left
            } else {
#pragma unroll
                for (int j = 0; j < kPrefetchRegs; ++j)
                    pf[j] = src[min(tid + j * kLdsThreads, n16 - 1)];
            }
        }
        // ---- feature tiles ----
        if (d.layout == FS_ROWMAJOR) {
            // Row-major input (the host side only sends it here when F % 4 == 0 and at least 8
            // padded rows fit below tile0): a tile is 64 consecutive rows = one contiguous run.  It
            // is fetched with 16-byte loads into a staging area at LDS offset 0 (the chunk region,
            // not yet in use) with a row stride of F + 1 words, as many rows at a time as fit, then
            // copied across with lane = row: the odd stride makes the column reads conflict-free,
            // the writes are whole columns.
            const uint32_t Fp = (uint32_t)F + 1u;
            const int stage_rows = min(64, (int)(tile0 / (4u * Fp)));   // rows the staging area takes
            for (int t = 0; t < tiles_here; ++t) {
                const int r0 = (tile_first + t) * 64;
                const int rows_here = min(64, d.n_rows - r0);
                for (int s0 = 0; s0 < 64; s0 += stage_rows) {            // uniform trip count
                    const int s1 = min(s0 + stage_rows, rows_here);      // rows [s0, s1) of the tile
                    if (s0 < s1) {
                        auto src = FS_GLOBAL(const u32x4, d.features + (int64_t)(r0 + s0) * F);
                        const int n16 = (s1 - s0) * (F >> 2);
                        for (int base = tid; base < n16; base += kTileBatch * kLdsThreads) {
                            u32x4 t4[kTileBatch];
#pragma unroll
                            for (int q = 0; q < kTileBatch; ++q)
                                t4[q] = src[min(base + q * kLdsThreads, n16 - 1)];
#pragma unroll
                            for (int q = 0; q < kTileBatch; ++q) {
                                const int i = base + q * kLdsThreads;
                                if (i < n16) {
                                    const int e = 4 * i, row = e / F, col = e - row * F;
                                    const uint32_t at = 4u * ((uint32_t)row * Fp + (uint32_t)col);
                                    lds_store_f(at, __uint_as_float(t4[q].x));
                                    lds_store_f(at + 4u, __uint_as_float(t4[q].y));
                                    lds_store_f(at + 8u, __uint_as_float(t4[q].z));
                                    lds_store_f(at + 12u, __uint_as_float(t4[q].w));
                                }
                            }
                        }
                    }
                    __syncthreads();
                    if (lane >= s0 && lane < s0 + stage_rows) {
                        for (int j = wave; j < F; j += kLdsWaves) {
                            const uint32_t from = 4u * ((uint32_t)(lane - s0) * Fp + (uint32_t)j);
                            const uint32_t to =
                                tile0 + (uint32_t)t * tile_bytes + (uint32_t)j * 256u + 4u * (uint32_t)lane;
                            lds_store_f(to, lane < s1 ? lds_f(from) : 0.0f);
                        }
                    }
                    __syncthreads();   // the staging area is free again (next rows, then the chunk)
                }
            }
            if (tid < 64 * tiles_here)
                lds_store_f(tile0 + (uint32_t)(tid >> 6) * tile_bytes + (uint32_t)F * 256u +
                                4u * (uint32_t)(tid & 63), __builtin_nanf(""));
        } else {
            // consecutive tiles are one contiguous run in HBM
            auto src = FS_GLOBAL(const u32x4, d.features + (int64_t)tile_first * F * 64);
            const int n16 = tiles_here * per_tile;
            if ((per_tile & 63) == 0) {
                // F % 4 == 0: every group of 64 pieces lies inside one tile
                const int n_groups = n16 >> 6;
                for (int g = wave; g < n_groups; g += kLdsWaves) {
                    const int i0 = g << 6;
                    const int t = i0 / per_tile, j0 = i0 - t * per_tile;
                    lds_fill_direct(src + i0, tile0 + (uint32_t)t * tile_bytes + 16u * (uint32_t)j0, 64, 0, 1,
                                    lane);
                }
            } else
            // two tiles are 7 pieces per thread: one batch, one exposure of the HBM latency
            for (int base = tid; base < n16; base += kTileBatch * kLdsThreads) {
                u32x4 t4[kTileBatch];
#pragma unroll
                for (int q = 0; q < kTileBatch; ++q)
                    t4[q] = src[min(base + q * kLdsThreads, n16 - 1)];
#pragma unroll
                for (int q = 0; q < kTileBatch; ++q) {
                    const int i = base + q * kLdsThreads;
                    if (i < n16) {
                        const int t = i / per_tile, j = i - t * per_tile;
                        lds_store_u4(tile0 + (uint32_t)t * tile_bytes + 16u * (uint32_t)j, t4[q]);
                    }
                }
            }
            if (tid < 64 * tiles_here)
                lds_store_f(tile0 + (uint32_t)(tid >> 6) * tile_bytes + (uint32_t)F * 256u +
                                4u * (uint32_t)(tid & 63), __builtin_nanf(""));
        }
        {
            const int n16 = (int)(h.bytes >> 4);
            if (direct) {
                const int i = (n16 & ~63) + tid;
                if (i < n16)
                    lds_store_u4(16u * (uint32_t)i, pf[0]);
                lds_direct_wait();
            } else {
#pragma unroll
                for (int j = 0; j < kPrefetchRegs; ++j) {
                    const int i = tid + j * kLdsThreads;
                    if (i < n16)
                        lds_store_u4(16u * (uint32_t)i, pf[j]);
                }
            }
        }
        __syncthreads();
    }

  // Later groups of the workgroup arrive through registers (tp and pf below).
    for (int grp = g_first; grp < g_end; ++grp) {
        const int tile_first = grp * T;
        const int tiles_here = min(T, n_tiles - tile_first);
        const bool active = my_tile < tiles_here;
        const int r = (tile_first + my_tile) * 64 + lane;
        float acc = d.bias;
        uint16_t *leaf_row = nullptr;
        if (DUMP) {
            if (active && d.leaf_idx && r < d.n_rows)
                leaf_row = d.leaf_idx + (int64_t)r * d.n_trees;
        }
        const bool compact = d.compact != 0;
        const int n_chunks = d.n_chunks;
        const uint32_t val_stride = (uint32_t)T * 256u;        // bytes between trees' value rows

        // Wavefronts 0..T-1 do the ordered sums.  When the others can carry a whole chunk in their
        // prefetch registers they copy it alone, so a sum and the copy run side by side.
        const int n_copiers = kLdsThreads - 64 * T;
        for (int c = 0; c < n_chunks; ++c) {
            // After the last chunk of a group that is not the workgroup's last, the next group's
            // tiles travel the same way as the next chunk (and the first chunk comes back when the
            // model has more than one).
            const bool last = c + 1 == n_chunks;
            const bool wrap = MULTI && last && grp + 1 < g_end;
            const bool fetch = !last || (wrap && n_chunks > 1);
            ChunkView hn = h;
            int n16_next = 0, cp_id = tid, cp_n = kLdsThreads;
            u32x4 tp[kLdsTileRegs];
            if (fetch) {                                       // next chunk: global -> registers
                hn = load_chunk(d.chunks + (last ? 0 : c + 1));
                auto src = FS_GLOBAL(const u32x4, d.image + hn.byte_off);
                n16_next = (int)(hn.bytes >> 4);
                if (n16_next <= kPrefetchRegs * n_copiers) {
                    cp_n = n_copiers;
                    cp_id = tid - 64 * T;                      // negative in the summing wavefronts
                }
                if (cp_id >= 0) {
#pragma unroll
                    for (int j = 0; j < kPrefetchRegs; ++j)
                        pf[j] = src[min(cp_id + j * cp_n, n16_next - 1)];
                }
            }
            if (wrap) {
                const int next_first = (grp + 1) * T;
                const int n16t = min(T, n_tiles - next_first) * per_tile;
                auto src = FS_GLOBAL(const u32x4, d.features + (int64_t)next_first * F * 64);
#pragma unroll
                for (int q = 0; q < kLdsTileRegs; ++q)
                    tp[q] = src[min(tid + q * kLdsThreads, n16t - 1)];
            }
            const int n = uniform((int)h.n_trees);
            const uint32_t val0 = tile0 - (uint32_t)n * val_stride;   // packing keeps it above the image
            if (active) {
                const uint32_t val_addr = val0 + (uint32_t)my_tile * 256u + 4u * (uint32_t)lane;
                const uint16_t *ids = d.slot_ids + h.slot_off;
                uint16_t *leaf_out = leaf_row ? leaf_row + h.first_tree : nullptr;
                // this wavefront's runs of the chunk: record my_slot, then the records chained to it
                uint32_t rec = (uint32_t)(kRunBytes * my_slot);
                for (;;) {
                    uint32_t tab[8];
                    const uint32_t head = lds_u(rec);            // same address in every lane: broadcast
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        tab[k] = lds_u(rec + 4u + 4u * (uint32_t)k);
                    const uint32_t run = (uint32_t)uniform((int)head);
                    const int count = (int)(run & 0xFu), depth = (int)(run >> 16);
                    if (count == 0)
                        break;                                   // idle slot
                    if (compact)
                        walk_n<true, DUMP>(count, tab, depth, lane_base, val_addr, val_stride, ids, leaf_out);
                    else
                        walk_n<false, DUMP>(count, tab, depth, lane_base, val_addr, val_stride, ids, leaf_out);
                    const uint32_t next = (run >> 4) & 0xFFFu;
                    if (next == 0)
                        break;
                    rec = (uint32_t)kRunBytes * (next - 1u);
                }
            }
            __syncthreads();       // every walk of this chunk is done and its values are parked
            if (active && my_slot == 0) {
                const uint32_t va = val0 + (uint32_t)my_tile * 256u + 4u * (uint32_t)lane;
                ordered_add_n(acc, va, val_stride, n);
            }
            if (fetch || wrap) {
                // The next image may be long enough to reach into the value rows that are being
                // summed right now (only when chunk sizes differ a lot): then wait for the readers.
                if (fetch && 16u * (uint32_t)n16_next > val0)
                    __syncthreads();
                if (fetch && cp_id >= 0) {
#pragma unroll
                    for (int j = 0; j < kPrefetchRegs; ++j) {
                        const int i = cp_id + j * cp_n;
                        if (i < n16_next)
                            lds_store_u4(16u * (uint32_t)i, pf[j]);
                    }
                }
                if (wrap) {                                    // every walk of this group is done
                    const int n16t = min(T, n_tiles - (grp + 1) * T) * per_tile;
#pragma unroll
                    for (int q = 0; q < kLdsTileRegs; ++q) {
                        const int i = tid + q * kLdsThreads;
                        if (i < n16t) {
                            // piece i of tile t sits 16 * i + 256 * t above tile0 (the NaN column of
                            // every tile before it); at most kLdsMaxTiles = 3 tiles, so no division
                            const int t = (i >= per_tile ? 1 : 0) + (i >= 2 * per_tile ? 1 : 0);
                            lds_store_u4(tile0 + 16u * (uint32_t)i + 256u * (uint32_t)t, tp[q]);
                        }
                    }
                }
                __syncthreads();
            }
            h = hn;
        }
        if (active && my_slot == 0 && r < d.n_rows)
            FS_GLOBAL(float, d.row_score)[r] = acc;
    }   // tile groups of this workgroup
}

int launch_traverse_lds(const FamDesc *d_desc, int n_families, int mode, int total_blocks,
                        int groups_per_wg, bool dump, hipStream_t stream)
{
    const int kLdsBytes = kLdsModeBytes[mode];
    const int kLdsThreads = 64 * kLdsModeWaves[mode];
    static bool configured[16][4] = {};
    int dev = 0;
    FS_HIP(hipGetDevice(&dev));
    const bool multi = groups_per_wg > 1;
    auto kernel = dump ? (multi ? traverse_lds_kernel<true, true> : traverse_lds_kernel<true, false>)
                       : (multi ? traverse_lds_kernel<false, true> : traverse_lds_kernel<false, false>);
    const int form = (dump ? 2 : 0) + (multi ? 1 : 0);
    if (dev < 0 || dev >= 16 || !configured[dev][form]) {
        // The kernel addresses LDS absolutely from 0, so it must own all of it: no static LDS
        // (nothing the compiler may have moved there either).
        hipFuncAttributes attr;
        FS_HIP(hipFuncGetAttributes(&attr, (const void *)kernel));
        if (attr.sharedSizeBytes != 0)
            return fail(FS_EDEVICE, "traverse_lds_kernel was built with %zu bytes of static LDS",
                        (size_t)attr.sharedSizeBytes);
        FS_HIP(hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kLdsModeBytes[kLdsModes - 1]));
        if (dev >= 0 && dev < 16)
            configured[dev][form] = true;
    }
    hipLaunchKernelGGL(kernel, dim3(total_blocks), dim3(kLdsThreads), kLdsBytes, stream, d_desc,
                       n_families, mode, groups_per_wg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "traverse_lds_kernel launch");
    return FS_OK;
}

}  // namespace fs
