/*
 * familyseer_train.h -- C ABI for training family cost models on the MI355X (gfx950).
 *
 * After every tuning step the tuner of the paper retrains the family's cost model on the
 * candidates that were measured (Algorithm 1, train_cost_model; Section 4.2), and Section 4.3
 * moves that training to the GPU because it grows to dozens of seconds on the CPU once tens
 * of thousands of candidates have been measured.  The paper names the model class (XGBoost)
 * and no more; this library trains the published second-order boosting step of that method
 * (Chen & Guestrin 2016, Eq. 4-7: leaf weight -G/(H+lambda), gain GL^2/(HL+lambda) +
 * GR^2/(HR+lambda) - G^2/(H+lambda)) with histograms over pre-binned features.
 *
 * Setting (shared with the scoring path of familyseer.h): a program p owns the statement
 * rows [prog_off[p], prog_off[p+1]), the model's score of a program is the sum of its row
 * outputs, and there is one measured target per program.  Loss 1/2 sum_p (s_p - y_p)^2.
 * Per boosting round: s_p = row outputs added in row order (fp32); g_p = s_p - y_p; every
 * row of p carries gradient g_p and curvature h = rows of p; gradients are rounded to
 * integers q = rint(g * grad_scale) so that histogram sums are exact whatever the order of
 * the rows; the tree grows level by level, nodes numbered breadth-first; a candidate split
 * is (feature f, cut c of that feature's cut list): rows with x_f < c go left (NaN right);
 * it is admissible if both sides hold curvature >= max(min_child_weight, 1); the first
 * admissible split (features ascending, cuts ascending) with the largest gain wins and is
 * taken if gain > min_gain and the node is above max_depth; a leaf's value is
 * (float)(-eta * G / grad_scale / (H + lambda)); gains and leaf values are evaluated in
 * double.  The result is bit-for-bit reproducible and the trained arrays have the format
 * fs_model_create takes.
 *
 * Conventions as in familyseer.h: FS_OK or a negative code, fs_last_error() for the text,
 * HOST / DEVICE per pointer, work enqueued on `stream` unless stated.
 */
#ifndef FAMILYSEER_TRAIN_H
#define FAMILYSEER_TRAIN_H

#include "familyseer.h"

#ifdef __cplusplus
extern "C" {
#endif

#define FS_TRAIN_MAX_DEPTH 10  /* split levels per tree                                  */
#define FS_TRAIN_MAX_CUTS 255  /* cut points per feature (bins fit a byte)               */

typedef struct fs_trainer fs_trainer; /* opaque: one family's training set and model so far */

typedef struct fs_train_params {
    int32_t max_depth;        /* 0..FS_TRAIN_MAX_DEPTH and <= the trainer's own limit     */
    float eta;                /* learning rate, > 0                                       */
    float lambda;             /* L2 term on leaf values, >= 0                             */
    float min_gain;           /* a node is split only if the best gain exceeds this       */
    float min_child_weight;   /* least curvature on each side of a split                  */
    float grad_scale;         /* fixed-point scale of the gradients, a power of two > 0   */
} fs_train_params;

/*
 * Take over a training set: the features are binned against the cut lists (feature f owns
 * cuts[cut_off[f] .. cut_off[f+1]), ascending and distinct, at most FS_TRAIN_MAX_CUTS;
 * bin = number of cuts <= x, NaN takes the last bin) into the trainer's own device memory,
 * so `features` is not needed after the call's work has run; `prog_off` and `target` are
 * copied too.  Every row starts at `bias`.  max_depth / max_trees bound what fs_train_boost
 * may be asked for later (they size the buffers).  n_rows >= 1, n_programs >= 1.
 * The content of prog_off (DEVICE) is not validated: it must start at 0, be non-decreasing
 * and end at n_rows, as for fs_score_families; a malformed array gives undefined results.
 * The cut lists (HOST) are validated.  The call BLOCKS until its work on `stream` is done: the
 * binning kernels run there, then the length of the longest program is read back (it sizes
 * the curvature sums of the histograms); the small host arrays are copied with plain
 * (synchronising) copies.  Create trainers outside latency-critical sections.
 * Errors: FS_EINVAL, FS_EUNSUPPORTED (limits), FS_ENOMEM, FS_EDEVICE.
 */
int fs_trainer_create(fs_trainer **out, int32_t n_features, const float *features /* DEVICE */,
                      int32_t layout /* FS_ROWMAJOR | FS_COLBLOCK64 */, int64_t n_rows,
                      const int32_t *prog_off /* DEVICE, n_programs+1 */, int32_t n_programs,
                      const float *target /* DEVICE, n_programs */,
                      const int32_t *cut_off /* HOST, n_features+1 */, const float *cuts /* HOST */,
                      float bias, int32_t max_depth, int32_t max_trees, void *stream);

/* Free a trainer (NULL allowed).  Synchronise its streams first. */
void fs_trainer_destroy(fs_trainer *t);

/*
 * n_rounds boosting rounds for every trainer of the batch (families train independently; one
 * batched submission per step, no host synchronisation).  All trainers use `params`.
 * Calls that involve the same trainer, and all training calls on one device, must be issued
 * on one stream (or be ordered by the caller): the batch descriptors and each trainer's
 * state are shared between calls.
 * Errors: FS_EINVAL, FS_EUNSUPPORTED (a trainer's max_depth / max_trees would be exceeded).
 */
int fs_train_boost(int32_t n_trainers, fs_trainer *const *trainers /* HOST */, int32_t n_rounds,
                   const fs_train_params *params /* HOST */, void *stream);

/* Trees trained so far and their total node count.  Waits for `stream`. */
int fs_trainer_size(const fs_trainer *t, int32_t *n_trees /* HOST */, int64_t *n_nodes /* HOST */,
                    void *stream);

/*
 * The model so far in the arrays fs_model_create reads (HOST out; tree_off has n_trees+1
 * entries, the node arrays n_nodes; node ids local to the tree, root 0, children after their
 * parent; split_feature < 0 at leaves).  The model's bias is the trainer's.  Waits for
 * `stream`.
 */
int fs_trainer_export(const fs_trainer *t, int32_t *tree_off, int32_t *split_feature,
                      float *threshold, int32_t *left, int32_t *right, float *value, void *stream);

/*
 * Current outputs of the model on the training set: row outputs (DEVICE out, n_rows, or NULL)
 * and program sums (DEVICE out, n_programs, or NULL), bit-identical to scoring the exported
 * model with fs_score_families.
 */
int fs_trainer_predictions(const fs_trainer *t, float *row_pred, float *prog_pred, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FAMILYSEER_TRAIN_H */
