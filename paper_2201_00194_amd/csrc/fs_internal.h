// Internal declarations shared by the library's translation units (not installed).
#ifndef FS_INTERNAL_H
#define FS_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "familyseer.h"

namespace fs {

// ---- error reporting ---------------------------------------------------------------------
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
int fail_hip(hipError_t e, const char *what);

#define FS_HIP(call)                                   \
    do {                                               \
        hipError_t fs_e_ = (call);                     \
        if (fs_e_ != hipSuccess)                       \
            return ::fs::fail_hip(fs_e_, #call);       \
    } while (0)

// ---- test and tuning overrides (fs_tune_set); -1 = automatic ---------------------------------
int tune(int option);

// ---- device-side model formats -------------------------------------------------------------

// Node of the reference device layout (global memory).  One entry per node, trees
// concatenated in the caller's numbering, child ids already offset to global node indices.
//   x: bits of threshold (internal) or of the leaf value (leaf)
//   y: split feature, or -1 at a leaf
//   z: global index of the left child    w: of the right child
typedef int4 GNode;

// ---- LDS-staged model format -------------------------------------------------------------------
// The ensemble is cut into chunks of consecutive trees.  A chunk is a byte image that is copied
// verbatim to LDS offset 0:
//     [run records of the wavefront slots] [further run records] [nodes ...]   (multiple of 16)
// A node is 8 bytes {w0, w1}:
//     internal: w0 = threshold bits, w1 = (feature * 256) << 16 | byte offset of the LEFT child;
//               the right child sits right after the left one
//     leaf:     w0 = value bits,     w1 = (n_features * 256) << 16 | (own offset - 8):
//               it reads the all-NaN column, fails '<' and so steps back onto itself
// In "compact" chunks (every tree of the model perfect and of one depth >= 1) leaves are 4-byte
// values only, laid out after the tree's internal nodes; the last split level then steps by 4.
//
// Walk order.  The wavefronts that share a tile ("slots") split the chunk's trees.  Trees are
// sorted by depth and cut into runs of at most 8 trees of similar depth; a run is walked side by
// side, to the depth of its first (deepest) tree, and the runs are dealt to the slots so that the
// slots have about the same work.  A run record is kRunWords uint32: word 0 = number of trees
// (bits 0-3) | index of the slot's next run record + 1, or 0 (bits 4-15) | depth (bits 16-31);
// words 1..8 = the run's trees: LDS offset of the root (bits 0-15) | index of the tree in its
// chunk, i.e. the place the ordered sum gives it (bits 16-23); unused tree words repeat the first.
// Record s (s < kLdsMaxWaves) is the first run of slot s (no trees: the slot is idle).
constexpr int kRunWords = 9;
constexpr int kRunBytes = 4 * kRunWords;

struct ChunkHdr {
    uint32_t byte_off;    // into the packed image
    uint32_t bytes;       // multiple of 16
    uint32_t n_trees;
    uint32_t depth;       // split levels of the deepest tree of the chunk
    uint32_t first_tree;  // model-wide index of the chunk's first tree
    uint32_t slot_off;    // into the id map: entry [slot_off + (lds byte offset >> 2)]
    uint32_t pad0;
    uint32_t pad1;
};

// LDS map of the traversal kernel (bytes):
//   [0, chunk bytes)                       model chunk (run records, nodes)
//   [tile0 - n_trees*tiles*256, tile0)     leaf values [tree in chunk][tile][lane] (fp32)
//   [tile0, 160 KB)                        `tiles` feature tiles of (n_features+1)*256 bytes,
//                                          tile0 = 160 KB - tiles * tile bytes
// Two workgroup shapes.  "small": half a compute unit's LDS, 6 wavefronts, one tile -- two
// such workgroups share a compute unit, so one walks while the other is busy with barriers,
// the ordered sum or the next chunk.  "big": the whole LDS, 12 wavefronts, 1-3 tiles -- for
// models whose trees are too large to give a small workgroup enough trees per chunk.
constexpr int kLdsModes = 2;
constexpr int kLdsModeBytes[kLdsModes] = {80 * 1024, 160 * 1024};
constexpr int kLdsModeWaves[kLdsModes] = {6, 12};
constexpr int kLdsMaxWaves = 12;
constexpr int kLdsMaxTiles = 3;         // 64-row tiles per workgroup (1, 2 or 3)
constexpr int kMaxChunkBytes = 65536 - 16;
constexpr int kMaxChunkTrees = 96;
constexpr int kPrefetchRegs = 6;        // 16-byte registers per thread for the next chunk

}  // namespace fs

// The opaque model: host copy of what validation needs plus device arrays.
struct fs_model {
    int32_t n_features;
    int32_t n_trees;
    int32_t max_depth;     // longest root-to-leaf path (in splits) over all trees
    int64_t n_nodes;
    float bias;
    int device;
    fs::GNode *d_nodes;    // [n_nodes]
    int32_t *d_tree_off;   // [n_trees + 1]
    // LDS-staged format (absent if the model does not fit it)
    bool lds_ok;
    bool compact;          // perfect trees of one depth, 4-byte leaves
    int32_t lds_mode;      // workgroup shape chosen for this model (index into kLdsMode*)
    int32_t lds_tiles;     // 64-row tiles per workgroup chosen for this model
    int32_t lds_tile0;     // LDS byte offset of the first feature tile
    float lds_group_us;    // the planner's estimate of one tile group's time in the LDS kernel
    int32_t n_chunks;
    uint8_t *d_image;      // all chunk images back to back
    fs::ChunkHdr *d_chunks;
    uint16_t *d_slot_ids;  // caller's local node id per 4-byte slot (leaves only meaningful)
    size_t image_bytes;
    // Rank-coded format (deep perfect trees): features become 16-bit ranks among the model's
    // own thresholds of that feature, nodes shrink to 4 bytes (see fs_traverse_rank.hip)
    bool rank_ok;
    int32_t rk_depth;          // common depth of the trees
    int32_t rk_tiles;          // 64-row tiles per workgroup
    int32_t rk_trees_per_chunk;
    int32_t rk_tree_bytes;     // 4 * 2^(depth+1): heap words 1 .. 2^(depth+1)-1, word 0 unused
    int32_t rk_tile0;          // LDS byte offset of the first (u16) feature tile
    uint32_t *d_rk_nodes;      // [n_trees][2^(depth+1)] 1-based heap order: splits then leaf values
    uint16_t *d_rk_ids;        // same shape: caller's local node id
    float *d_cuts;             // [n_features][2^cut_bits]: the feature's sorted distinct
                               // thresholds, NaN-padded, as a breadth-first search tree
    int32_t cut_bits;
};

namespace fs {

// ---- per-family descriptor as the kernels see it --------------------------------------------
struct FamDesc {
    const GNode *nodes;
    const int32_t *tree_off;
    const float *features;
    const int32_t *prog_off;
    float *prog_score;
    float *row_score;      // never NULL on the device: caller's buffer or library scratch
    uint16_t *leaf_idx;    // may be NULL
    int32_t n_trees;
    int32_t n_features;
    int32_t layout;
    int32_t n_rows;
    int32_t n_programs;
    float bias;
    int32_t trav_block0;   // first block of the global-memory traversal grid of this family
    int32_t seg_block0;    // first block of the segmented-sum grid
    // LDS-staged traversal
    const uint8_t *image;
    const ChunkHdr *chunks;
    const uint16_t *slot_ids;
    int32_t n_chunks;
    int32_t lds_tile0;
    int32_t lds_tiles;
    int32_t compact;
    int32_t lds_block0[kLdsModes];   // first block of this family in each LDS launch
    // rank-coded traversal
    const uint32_t *rk_nodes;
    const uint16_t *rk_ids;
    const float *cuts;
    uint16_t *ranks;                 // scratch: rank-coded feature tiles [tile][feature][64]
    int32_t rk_depth, rk_tiles, rk_trees_per_chunk, rk_tree_bytes, rk_tile0;
    int32_t rk_block0;               // first block of the rank traversal grid
    int32_t bin_block0;              // first block of the rank-coding grid
    int32_t bin_groups;              // feature groups of this family in the rank-coding grid
    int32_t bin_feats_per_group;
    int32_t bin_tiles_per_block;
    // row-major input: re-tiled into scratch before the LDS kernels (features then points there)
    const float *rowmajor_src;
    int32_t retile_block0;           // first block of the re-tiling grid
    int32_t retile_colblocks;        // column blocks per tile (0: family not re-tiled)
    int32_t cut_bits;                // threshold tables are padded to 2^cut_bits entries
    int32_t pad;
};

// One workgroup of the first top-k stage: the whole request, or one slice of a large one.
struct TopkDesc {
    const float *score;
    int32_t *out_idx;
    float *out_score;      // may be NULL
    int32_t n;             // entries of the request
    int32_t k;
    int32_t sub_begin, sub_end;      // the slice [sub_begin, sub_end) this workgroup ranks
    unsigned long long *comp_out;    // NULL: final answer to out_idx/out_score; else the slice's
                                     // best min(k, slice length) (key, ~index) composites, best first
    int32_t comp_pad;                // 1: pad comp_out with 0 up to k entries
    int32_t pad;
};

// Second stage of a large request: merge the slices' candidates.
struct TopkMergeDesc {
    const unsigned long long *comp_in;   // n_comp composites (0 = padding)
    const float *score;
    int32_t *out_idx;
    float *out_score;      // may be NULL
    int32_t n_comp;
    int32_t n;             // entries of the request
    int32_t k;
    int32_t pad;
};


// One merge of two lists of composites (each best first) in global memory: the best `lo` of
// their union go to `out` (composites), or, at the last level of a request, to its
// out_idx / out_score (then `lo` = min(n, k) and entries up to k are padded with -1 / -inf).
struct TopkPairDesc {
    const unsigned long long *a, *b;
    unsigned long long *out;       // NULL at the last level
    const float *score;
    int32_t *out_idx;
    float *out_score;              // may be NULL
    int32_t la, lb, lo, k;
};

// u16 rank tiles keep the features of a row in pairs: features 2i and 2i+1 of row l share the
// 32-bit word at i*256 + 4*l of the tile, so that lane l always reads from LDS bank l whichever
// feature it asks for (with one u16 column after the other, two lanes would meet in every bank).
// A tile therefore has an even number of columns.
__host__ __device__ inline int rank_tile_cols(int n_features) { return (n_features + 1) & ~1; }
__host__ __device__ inline uint32_t rank_feature_offset(int f) { return (uint32_t)(f >> 1) * 256u + (uint32_t)(f & 1) * 2u; }

// ---- launchers (each returns FS_OK or records an error) ---------------------------------------
int launch_traverse_global(const FamDesc *d_desc, int n_families, int total_blocks,
                           hipStream_t stream);
int launch_traverse_lds(const FamDesc *d_desc, int n_families, int mode, int total_blocks,
                        int groups_per_wg, bool dump, hipStream_t stream);
// Tile groups one workgroup of the LDS traversal takes in a row; host (workgroup counts) and
// kernel agree on it through this function.  From its second group on a workgroup receives the
// tiles through registers, kLdsTileRegs 16-byte pieces per thread, so `want` only holds for
// column-blocked input whose `tiles` tiles fit there; other families get one group per workgroup.
constexpr int kLdsTileRegs = 7;
__host__ __device__ inline int lds_groups_per_wg(int layout, int n_features, int tiles, int threads,
                                                 int want)
{
    if (layout != FS_COLBLOCK64 || tiles * n_features * 16 > kLdsTileRegs * threads)
        return 1;
    return want < 1 ? 1 : want;
}
int launch_rank_code(const FamDesc *d_desc, int n_families, int total_blocks, hipStream_t stream);
int launch_traverse_rank(const FamDesc *d_desc, int n_families, int total_blocks, bool dump,
                         hipStream_t stream);
int launch_segsum(const FamDesc *d_desc, int n_families, int total_blocks, hipStream_t stream);
int launch_topk(const TopkDesc *d_desc, int n_blocks, int max_k, hipStream_t stream);
// max_padded: largest (slices * k rounded up to a power of two) over the requests
int launch_topk_merge(const TopkMergeDesc *d_desc, int n_requests, int max_padded, hipStream_t stream);
constexpr int kTopkSliceMin = 8192;      // requests at least this long are split into slices
constexpr int kTopkSliceEntries = 2048;  // of at least this many entries
constexpr int kTopkMaxSlices = 16;
constexpr int kTopkMergeCap = 16384;     // composites (lists padded to a power of two) the merge holds in LDS
constexpr int kTopkWideSlice = 2048;     // slice length of cuts too wide for the LDS merge (k > 4096)
constexpr int kTopkWideMaxSlices = 128;
// How a top-k request of n entries and cut k is served:
//   mode 0  one workgroup, finished by the first kernel;
//   mode 1  long request, k <= 4096: `s` slices of `per` entries (one workgroup each) leave their
//           best k in scratch and one workgroup merges them in LDS;
//   mode 2  long request with a wider cut: slices of about kTopkWideSlice entries leave their best
//           min(k, length) sorted, then pairwise merges in global memory, level by level.
struct TopkPlan { int mode, s, per; };
inline TopkPlan topk_plan(int n, int k)
{
    TopkPlan p = {0, 1, n};
    if (n < kTopkSliceMin || k == 0)
        return p;
    int kp = 1;
    while (kp < k)
        kp <<= 1;
    if (kp > kTopkMergeCap / 4) {
        int s = (n + kTopkWideSlice - 1) / kTopkWideSlice;
        if (s > kTopkWideMaxSlices)
            s = kTopkWideMaxSlices;
        if (s >= 2) {
            p.mode = 2;
            p.s = s;
            p.per = (((n + s - 1) / s) + 63) & ~63;
        }
        return p;
    }
    int s = kTopkMergeCap / kp;
    if (s > kTopkMaxSlices)
        s = kTopkMaxSlices;
    if (s > n / kTopkSliceEntries)
        s = n / kTopkSliceEntries;
    if (s >= 2) {
        p.mode = 1;
        p.s = s;
        p.per = (((n + s - 1) / s) + 63) & ~63;
    }
    return p;
}
int launch_topk_pairs(const TopkPairDesc *d_desc, int n_pairs, int max_entries, hipStream_t stream);
int launch_retile(const FamDesc *d_desc, int n_families, int total_blocks, hipStream_t stream);
int launch_pack_colblock64(const float *in, int64_t n_rows, int32_t n_features, float *out,
                           hipStream_t stream);

// ---- optional per-kernel timing (fs_profile_begin / fs_profile_end) ----------------------------
enum KernelClass { kKernTraverse = 0, kKernSegsum = 1, kKernTopk = 2, kKernPack = 3,
                   kKernTraverseGlobal = 4, kKernRankCode = 5, kKernTraverseRank = 6,
                   kKernTrainHist = 7, kKernTrainSplit = 8, kKernTrainOther = 9,
                   kKernClasses = 10 };
// Records an event pair around the launches made between prof_start and prof_stop when
// profiling is on; no-ops otherwise.  Both run under the API mutex.
void prof_start(int kernel_class, hipStream_t stream);
void prof_stop(hipStream_t stream);

// rank-coding kernel: most tiles handled by one workgroup, LDS bytes for threshold tables
constexpr int kBinTilesPerBlock = 256;
constexpr int kBinTableBytes = 64 * 1024;
constexpr int kRankWaves = 12;
constexpr int kRankLdsBytes = 160 * 1024;
constexpr int kRankPrefetchRegs = 6;     // 16-byte registers per thread for the next chunk

constexpr int kTravRowsPerBlock = 256;   // rows per block of the global-memory traversal
constexpr int kSegProgsPerBlock = 256;   // programs per block of the segmented sum

}  // namespace fs
#endif
