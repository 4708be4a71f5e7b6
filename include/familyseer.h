/*
 * familyseer.h -- C ABI of the MI355X (gfx950) family cost-model scoring library.
 *
 * The auto-tuner of the paper keeps one gradient-boosted-tree cost model per subgraph
 * family (Section 4.2; Algorithm 1 initialises a model C[f] for every family f), lets
 * that model estimate every generated candidate program of the family's subgraphs
 * (Section 4.2, the tune step; Section 2 "Building the Cost Model"), and sends only the
 * best g candidates on to measurement (Section 3.2 "select the top-k"; Algorithm 1,
 * g = min(64, B / #subgraphs), g*p in the foresee step).  This library is that
 * estimate-then-cut step for many families at once:
 *
 *   fs_score_families   every family's model scores its own candidates:
 *                       tree traversal per (statement row, tree), per-row sum over the
 *                       ensemble, per-program sum over the program's statement rows
 *   fs_topk             per family, the k programs with the largest score
 *
 * Conventions (the paper leaves them open; both this library and its test oracle fix
 * them the same way):
 *   - larger score = better candidate; callers holding latencies negate them;
 *   - at an internal node a row goes LEFT iff x[split_feature] < threshold (strict),
 *     otherwise RIGHT; a NaN feature therefore goes right; no missing-value rule;
 *   - row_score[r]  = bias + sum of reached leaf values, fp32, trees in ascending order;
 *   - prog_score[p] = sum of its rows' scores, fp32, rows in ascending order, from +0;
 *     both sums are plain sequential additions (no FMA, no reassociation), so results
 *     are reproducible bit for bit;
 *   - top-k order: score descending, then program index ascending; -0 ties with +0;
 *     NaN scores order after every number.
 *
 * All functions return FS_OK (0) or a negative error code and never throw, abort or
 * print.  After an error, fs_last_error() gives a message for the calling thread.
 * "HOST" / "DEVICE" on a pointer says which memory it must point to.  Device pointers
 * must belong to the device that is current when the call is made.  Descriptor arrays
 * (fs_family[], fs_topk_req[]) are HOST memory and are only read during the call.
 * Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream)
 * and the call normally returns without waiting for it.  fs_score_families and fs_topk
 * block the host only in these cases:
 *   - the library scratch of the device must grow for this call: the device is
 *     synchronised, the old buffer freed and a larger one allocated.  A caller that has
 *     reserved enough (fs_workspace_bytes, fs_topk_workspace_bytes, fs_workspace_reserve)
 *     never gets here;
 *   - the call's descriptors (232 bytes per family, 56 per top-k workgroup) exceed 16 KB
 *     (about 70 families or 290 top-k workgroups).  Up to that size they travel as kernel
 *     arguments; beyond it they are staged through a ring of 8 pinned slots per device: a
 *     slot grows when it is too small, and the ninth such submission waits until the first
 *     has finished on the device.
 * A call that does neither only enqueues kernels on `stream`, so it may be recorded into a
 * HIP graph (stream capture), provided every kernel form it uses has been launched once
 * outside capture (a kernel's first launch on a device configures its LDS size).  A
 * replayed graph reads the buffers and uses the descriptors of the captured call; it shares
 * the library's descriptor buffers and scratch with later calls, so replays and other
 * library calls must not overlap in time on different streams.  The graph also holds the
 * address the scratch had at capture: reserve the largest scratch any later call on the
 * device will need before capturing, so that it is never re-allocated under the graph.
 * fs_model_create, fs_trainer_create and the fs_trainer_* read-back calls synchronise
 * (stated where they are declared).
 */
#ifndef FAMILYSEER_H
#define FAMILYSEER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    FS_OK = 0,
    FS_EINVAL = -1,       /* bad argument (NULL pointer, negative size, malformed model, ...) */
    FS_ENOMEM = -2,       /* host or device allocation failed                               */
    FS_EDEVICE = -3,      /* a HIP call failed; fs_last_error() holds the HIP message       */
    FS_EUNSUPPORTED = -4  /* valid request outside the implemented limits                   */
};

/* Feature matrix layouts. */
enum {
    FS_ROWMAJOR = 0,   /* x[r][j] at r*n_features + j.  Accepted everywhere.  The kernels that
                          first touch the features read it themselves where they can (rank-coded
                          models always; other LDS-staged models when n_features is a multiple
                          of 4): 10-20 % slower than FS_COLBLOCK64.  Otherwise the library
                          re-tiles the matrix into its scratch first (one extra pass)           */
    FS_COLBLOCK64 = 1  /* tiles of 64 rows, feature-major inside a tile:
                          x[r][j] at (r/64)*n_features*64 + j*64 + (r%64);
                          the last tile is padded to 64 rows (padding content is ignored);
                          the buffer holds ceil(n_rows/64)*n_features*64 floats            */
};

/* Limits. */
#define FS_MAX_FEATURES 4096     /* n_features per model                                    */
#define FS_MAX_TREE_NODES 65535  /* nodes in one tree (leaf ids fit uint16_t)               */
#define FS_MAX_TOPK 16384        /* k per request                                           */

/* Message for the last error on this thread; static storage, never NULL. */
const char *fs_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int fs_version(void);

/* ---- models: one per family (Section 4.2: an individual cost model per family) -------- */

typedef struct fs_model fs_model; /* opaque, owned by the library */

/*
 * Build a device-resident ensemble from HOST arrays (copied; the caller may free them
 * on return).  Trees are concatenated: tree t owns nodes [tree_off[t], tree_off[t+1]),
 * tree_off[0] = 0; node ids in `left`/`right` are LOCAL to the tree and the root is
 * local node 0.  split_feature[n] < 0 marks a leaf whose output is value[n] (its
 * threshold/left/right are ignored); otherwise 0 <= split_feature[n] < n_features and
 * the node sends a row left iff x[split_feature[n]] < threshold[n].  Child ids must be
 * greater than the parent's id and inside the tree (this rules out cycles); every tree
 * needs at least one node and at most FS_MAX_TREE_NODES.  n_trees may be 0 (every row
 * then scores `bias`).  `bias` is added once per row.
 * Errors: FS_EINVAL for NULL/negative/malformed input, FS_ENOMEM, FS_EDEVICE.
 * Synchronises with the device (plain hipMemcpy) before returning.
 */
int fs_model_create(fs_model **out, int32_t n_features, int32_t n_trees,
                    const int32_t *tree_off /* HOST, n_trees+1 */,
                    const int32_t *split_feature /* HOST, tree_off[n_trees] */,
                    const float *threshold /* HOST */, const int32_t *left /* HOST */,
                    const int32_t *right /* HOST */, const float *value /* HOST */,
                    float bias);

/* Free a model.  NULL is allowed.  The caller must make sure no enqueued work still
 * uses it (synchronise the streams first). */
void fs_model_destroy(fs_model *model);

/* ---- scoring -------------------------------------------------------------------------- */

/* One family: its model and its own candidates (Section 4.2: the family model estimates
 * the candidates generated for the family's subgraph). */
typedef struct fs_family {
    const fs_model *model;  /* this family's ensemble                                       */
    const float *features;  /* DEVICE, read-only, layout per `layout`; 16-byte aligned      */
    int32_t layout;         /* FS_ROWMAJOR or FS_COLBLOCK64                                 */
    int64_t n_rows;         /* statement rows, >= 0, < 2^31                                 */
    const int32_t *prog_off; /* DEVICE, n_programs+1 entries: program p owns rows
                                [prog_off[p], prog_off[p+1]); prog_off[0] = 0,
                                non-decreasing, prog_off[n_programs] = n_rows.  The content
                                is NOT validated on the device: a malformed array gives
                                undefined results (but reads stay inside n_rows).           */
    int32_t n_programs;     /* >= 0                                                         */
    float *prog_score;      /* DEVICE out, n_programs floats                                */
    float *row_score;       /* DEVICE out, n_rows floats, or NULL (library scratch is used) */
    uint16_t *leaf_idx;     /* DEVICE out, n_rows*n_trees, row-major [row][tree]: the local
                               id of the leaf reached; or NULL.  Verification aid: it adds
                               2*n_trees bytes of writes per row.                           */
} fs_family;

/*
 * Score all families in one batched submission (a fixed, small number of kernel
 * launches whatever n_families is).  Families are independent; buffers of different
 * families must not overlap.  Empty families (n_rows == 0 or n_programs == 0) are
 * allowed.  Errors are detected on the host before anything is enqueued: FS_EINVAL
 * (NULL pointers, negative sizes, unknown layout, misaligned features), FS_ENOMEM /
 * FS_EDEVICE (scratch growth, launch failure).
 * The library keeps one scoring scratch buffer per device (row scores of families that pass
 * row_score == NULL, rank tiles of models it rank-codes, re-tiled copies of row-major
 * input) which all fs_score_families calls on the device share: two such calls must not
 * overlap in time on different streams.  fs_topk has a scratch region of its own, so a
 * scoring call and a top-k call on unrelated data may overlap.
 */
int fs_score_families(int32_t n_families, const fs_family *fams /* HOST */, void *stream);

/* ---- top-k ---------------------------------------------------------------------------- */

typedef struct fs_topk_req {
    const float *score;  /* DEVICE in, n floats                                             */
    int32_t n;           /* >= 0                                                            */
    int32_t k;           /* 0 <= k <= FS_MAX_TOPK                                           */
    int32_t *out_idx;    /* DEVICE out, k entries: indices into score, best first; entries
                            past min(k,n) are -1                                            */
    float *out_score;    /* DEVICE out, k entries, or NULL: the selected scores; entries
                            past min(k,n) are -infinity                                     */
} fs_topk_req;

/*
 * For every request, the k entries with the largest score, ordered by (score descending,
 * index ascending) (Section 3.2: candidates are sorted by the model's estimate and the
 * top k are kept; Algorithm 1: k = g, or g*p in the foresee step).  One batched
 * submission for all requests.  Errors: FS_EINVAL, FS_EUNSUPPORTED (k > FS_MAX_TOPK),
 * FS_ENOMEM, FS_EDEVICE.  Requests of 8192 entries and more use the device's top-k scratch
 * region, which all fs_topk calls on the device share: two such calls must not overlap in
 * time on different streams.
 */
int fs_topk(int32_t n_requests, const fs_topk_req *reqs /* HOST */, void *stream);

/*
 * fs_topk for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result as fs_topk, but
 * the call allocates nothing and never waits: descriptors and the candidate lists of sliced
 * requests (8192 entries and more) live in a fixed 1 MiB array in device memory that the
 * library holds on every GPU it runs on until the process ends.  Limits (FS_EUNSUPPORTED
 * beyond them, nothing is enqueued): descriptors of at most 3584 bytes -- 56 per workgroup,
 * one workgroup per request below 8192 entries, up to 16 per longer request, plus 48 per
 * sliced request: about 60 workgroups; candidate lists (slices x k x 8 bytes per sliced
 * request) of at most 1 MiB - 3584 bytes; no cut wider than 4096 on a request of 8192 or more
 * entries.  All calls on a GPU share that GPU's array, which keeps the previous call's
 * contents (nothing in it needs clearing: every byte a call reads it has written first): calls
 * that overlap in time on one GPU, on whatever streams, race.  The array's device address is
 * looked up once per device, at the first call made with that device current.
 */
int fs_topk_noalloc(int32_t n_requests, const fs_topk_req *reqs /* HOST */, void *stream);

/* ---- library scratch ------------------------------------------------------------------- */

/*
 * Bytes of scoring scratch that fs_score_families(n_families, fams, ...) would use, and of
 * top-k scratch that fs_topk(n_requests, reqs, ...) would use.  Only sizes, layouts, models
 * and the NULL-ness of row_score are looked at; nothing is enqueued.  Return 0 for calls that
 * need none, and 0 with fs_last_error() set for descriptors the scoring / top-k call itself
 * would reject.
 */
size_t fs_workspace_bytes(int32_t n_families, const fs_family *fams /* HOST */);
size_t fs_topk_workspace_bytes(int32_t n_requests, const fs_topk_req *reqs /* HOST */);

/*
 * Grow the current device's scoring and top-k scratch to at least these sizes now (either may
 * be 0) and set up descriptor staging.  May synchronise the device and allocate.  Afterwards
 * calls whose needs stay within the reserved sizes neither allocate nor synchronise for
 * scratch.  Errors: FS_ENOMEM, FS_EDEVICE.
 */
int fs_workspace_reserve(size_t score_bytes, size_t topk_bytes);

/* ---- layout helper -------------------------------------------------------------------- */

/*
 * Re-tile a row-major feature matrix (DEVICE, n_rows x n_features floats) into
 * FS_COLBLOCK64 (DEVICE out, ceil(n_rows/64)*n_features*64 floats; padding rows are
 * written as 0).  in and out must not overlap.  Not part of the scoring path proper:
 * a producer that can emit FS_COLBLOCK64 directly never needs it.
 */
int fs_pack_colblock64(const float *rowmajor /* DEVICE */, int64_t n_rows, int32_t n_features,
                       float *out /* DEVICE */, void *stream);

/* Number of floats an FS_COLBLOCK64 buffer needs. */
int64_t fs_colblock64_floats(int64_t n_rows, int32_t n_features);

/* ---- population compaction ------------------------------------------------------------ */

/* One source of fs_gather_programs: a scored family in FS_COLBLOCK64 layout. */
typedef struct fs_gather_src {
    const float *features;   /* DEVICE, FS_COLBLOCK64                                      */
    const int32_t *prog_off; /* DEVICE, n_programs+1 (content not validated, as above)     */
    const float *score;      /* DEVICE, n_programs program scores, or NULL                 */
    int32_t n_programs;      /* >= 0                                                       */
} fs_gather_src;

/*
 * Carry selected programs over into a new family without leaving the device.  The search
 * that feeds the cost model keeps the best candidates from one generation to the next
 * (Section 2, the evolutionary search the tuner inherits; Section 3.2, pools of candidates):
 * survivors keep their feature rows and their scores, so only new candidates need scoring.
 * `keep` (DEVICE, n_keep <= FS_MAX_TOPK entries, e.g. the out_idx of fs_topk) indexes the
 * concatenation of the sources' programs (source 0 first; at most 8 sources); an entry of
 * -1 (the cut's padding) gives an empty program with score -infinity.  Output, in the order
 * of `keep`: out_prog_off (DEVICE, n_keep+1), out_features (DEVICE, FS_COLBLOCK64, room for
 * out_row_capacity rows rounded up to whole tiles; padding rows of the last tile are written
 * as 0), out_score (DEVICE, n_keep, or NULL; -infinity where the source has no scores).
 * The row count is only known on the device: it is out_prog_off[n_keep].  `status` (DEVICE,
 * one int32) receives 0, or 1 if the rows do not fit out_row_capacity (then every offset is
 * 0 and no row is copied), or 2 if `keep` holds an index outside the sources (such entries
 * are treated like -1).  Output buffers must not overlap the sources.
 * Errors (host side): FS_EINVAL, FS_EUNSUPPORTED (more than 8 sources, n_keep > FS_MAX_TOPK).
 */
int fs_gather_programs(int32_t n_features, int32_t n_sources, const fs_gather_src *src /* HOST */,
                       const int32_t *keep /* DEVICE */, int32_t n_keep, float *out_features,
                       int64_t out_row_capacity, int32_t *out_prog_off, float *out_score,
                       int32_t *status, void *stream);

/* ---- test and tuning hooks -------------------------------------------------------------- */

/*
 * Process-wide overrides of choices the library otherwise makes by itself.  They exist so
 * that tests can drive every kernel form on small inputs and so that tile / chunk shapes can
 * be swept; results never depend on them (every form is exact).  value < 0 restores the
 * automatic choice.  The model options are read by fs_model_create (models already built keep
 * their plan), the training options by fs_train_boost.  Nothing else -- no environment
 * variable -- changes which kernel a model or trainer takes.
 */
enum {
    FS_TUNE_LDS_TILES = 0,        /* 1..3: 64-row tiles per workgroup of the LDS-staged traversal  */
    FS_TUNE_LDS_MODE = 1,         /* 1: half-LDS workgroups (two per compute unit), 2: full         */
    FS_TUNE_RANK = 2,             /* 0: never rank-code a model, 1: whenever its trees allow        */
    FS_TUNE_RANK_TILES = 3,       /* 1, 2, 3, 4 or 6: tiles per workgroup of the rank traversal     */
    FS_TUNE_VERBOSE = 4,          /* 1: fs_model_create reports its plan on stderr                  */
    FS_TUNE_TRAIN_SLAB_ROWS = 5,  /* 64..65536: rows per histogram slab                             */
    FS_TUNE_TRAIN_SORT = 6,       /* 0: never regroup rows by node, 1: whenever possible            */
    FS_TUNE_TRAIN_PACKED = 7,     /* 0: separate 64-bit gradient / curvature sums only              */
    FS_TUNE_LDS_GROUPS = 8,       /* 1..16: tile groups a workgroup of the LDS traversal takes in a
                                     row (automatic: 1..4 by the length of the launch)             */
    FS_TUNE_OPTIONS = 9
};
int fs_tune_set(int32_t option, int32_t value);
int32_t fs_tune_get(int32_t option);   /* current override, -1 = automatic */

/* ---- per-kernel timing (measurement aid) ----------------------------------------------------- */

/* Kernel classes reported by fs_profile_end. */
enum { FS_KERNEL_TRAVERSE = 0,        /* LDS-staged traversal (the hot kernel)               */
       FS_KERNEL_SEGSUM = 1, FS_KERNEL_TOPK = 2, FS_KERNEL_PACK = 3,
       FS_KERNEL_TRAVERSE_GLOBAL = 4, /* traversal from global memory (models/layouts that
                                         the LDS kernel does not take)                       */
       FS_KERNEL_RANK_CODE = 5,       /* features -> 16-bit ranks (deep perfect-tree models)  */
       FS_KERNEL_TRAVERSE_RANK = 6,   /* LDS-staged traversal over rank-coded features        */
       FS_KERNEL_TRAIN_HIST = 7,      /* training: gradient histograms (familyseer_train.h)   */
       FS_KERNEL_TRAIN_SPLIT = 8,     /* training: best cut per (node, feature), node decision */
       FS_KERNEL_TRAIN_OTHER = 9,     /* training: gradients, row moves, output update, emit  */
       FS_KERNEL_CLASSES = 10 };

/*
 * Between fs_profile_begin and fs_profile_end the library brackets every kernel group it
 * launches with a pair of HIP events on the caller's stream (at most max_records groups;
 * later ones go untimed).  fs_profile_end waits for the recorded events and adds up, per
 * kernel class, the elapsed milliseconds (HOST out, FS_KERNEL_CLASSES doubles) and the
 * number of timed groups (HOST out, FS_KERNEL_CLASSES ints; either may be NULL).
 * The sections are the tuner's estimate step (traverse + segmented sum) and cut step
 * (top-k) of Section 4.2.  Process-wide switch; not meant for concurrent use.
 */
int fs_profile_begin(int32_t max_records);
int fs_profile_end(double *ms_by_kernel /* HOST */, int32_t *launches_by_kernel /* HOST */);

#ifdef __cplusplus
}
#endif
#endif /* FAMILYSEER_H */
