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

// ---- device-side model formats -------------------------------------------------------------

// Node of the reference device layout (global memory).  One entry per node, trees
// concatenated in the caller's numbering, child ids already offset to global node indices.
//   x: bits of threshold (internal) or of the leaf value (leaf)
//   y: split feature, or -1 at a leaf
//   z: global index of the left child    w: of the right child
typedef int4 GNode;

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
    int32_t trav_block0;   // first block of the traversal grid that belongs to this family
    int32_t seg_block0;    // first block of the segmented-sum grid
};

struct TopkDesc {
    const float *score;
    int32_t *out_idx;
    float *out_score;      // may be NULL
    int32_t n;
    int32_t k;
};

// ---- launchers (each returns FS_OK or records an error) ---------------------------------------
int launch_traverse_global(const FamDesc *d_desc, int n_families, int total_blocks,
                           hipStream_t stream);
int launch_segsum(const FamDesc *d_desc, int n_families, int total_blocks, hipStream_t stream);
int launch_topk(const TopkDesc *d_desc, int n_requests, int max_k, hipStream_t stream);
int launch_pack_colblock64(const float *in, int64_t n_rows, int32_t n_features, float *out,
                           hipStream_t stream);

// ---- optional per-kernel timing (fs_profile_begin / fs_profile_end) ----------------------------
enum KernelClass { kKernTraverse = 0, kKernSegsum = 1, kKernTopk = 2, kKernPack = 3, kKernClasses = 4 };
// Records an event pair around the launches made between prof_start and prof_stop when
// profiling is on; no-ops otherwise.  Both run under the API mutex.
void prof_start(int kernel_class, hipStream_t stream);
void prof_stop(hipStream_t stream);

constexpr int kTravRowsPerBlock = 256;   // rows per block of the global-memory traversal
constexpr int kSegProgsPerBlock = 256;   // programs per block of the segmented sum

}  // namespace fs
#endif
