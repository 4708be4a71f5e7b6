/*
 * CPU oracle for family cost-model scoring.  TEST INFRASTRUCTURE ONLY: nothing on the
 * product path may call, link or load this file; it exists so that tests, the smoke
 * check and the benchmark's CPU-baseline leg have a plain definition to compare with.
 *
 * What is computed follows the paper's description of how a tuning round uses a cost
 * model: the family's gradient-boosted-tree model estimates every generated candidate
 * (Section 2, "Building the Cost Model"; Section 4.2, the tune step), the candidates
 * are ordered by the estimate and the best k go on to measurement (Section 3.2,
 * "select the top-k program candidates"; Section 4.2, the number is restricted to g).
 * A candidate program has several statements, each with its own feature row; the
 * program's score is the sum of the model's outputs over its rows.
 *
 * Everything is the definition written out, one step at a time, in float:
 *
 *   leaf(r,t)     walk tree t from its root; at an internal node go left iff
 *                 x[split_feature] < threshold (strict), else right; stop at a leaf.
 *   row_score[r]  acc = bias; for t = 0..T-1 ascending: acc = acc + value_t[leaf(r,t)]
 *   prog_score[p] acc = +0;  for r = off[p]..off[p+1]-1 ascending: acc = acc + row_score[r]
 *   topk          order all programs by (score descending, index ascending) with a full
 *                 stable merge sort; emit the first min(k,P); pad to k with (-1, -inf).
 *                 -0 equals +0; NaN orders after every number.
 *
 * Readings where the paper is silent: larger score = better; strict '<' goes left; a
 * NaN feature fails '<' and goes right; the bias is added once per row; sums are plain
 * sequential fp32 additions in the stated order (build with -ffp-contract=off, no
 * fast-math).  No blocking, fusion, vectorisation tricks or reordering.
 *
 * Parity pins for every function here are in tests/test_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Leaf reached by one feature row in one tree (node ids local to the tree). */
int32_t fso_leaf(const int32_t *split_feature, const float *threshold,
                 const int32_t *left, const int32_t *right, const float *x)
{
    int32_t n = 0;
    while (split_feature[n] >= 0) {
        if (x[split_feature[n]] < threshold[n])
            n = left[n];
        else
            n = right[n];
    }
    return n;
}

/* leaf_idx[r * n_trees + t] for rows [0, n_rows) of a row-major matrix X. */
void fso_leaf_indices(int32_t n_features, int32_t n_trees, const int32_t *tree_off,
                      const int32_t *split_feature, const float *threshold,
                      const int32_t *left, const int32_t *right,
                      const float *X, int64_t n_rows, int32_t *leaf_idx)
{
    for (int64_t r = 0; r < n_rows; ++r) {
        const float *x = X + r * (int64_t)n_features;
        for (int32_t t = 0; t < n_trees; ++t) {
            int32_t o = tree_off[t];
            leaf_idx[r * (int64_t)n_trees + t] =
                fso_leaf(split_feature + o, threshold + o, left + o, right + o, x);
        }
    }
}

/* row_score[r] = bias + sum over trees (ascending) of the reached leaf's value. */
void fso_row_scores(int32_t n_features, int32_t n_trees, const int32_t *tree_off,
                    const int32_t *split_feature, const float *threshold,
                    const int32_t *left, const int32_t *right, const float *value,
                    float bias, const float *X, int64_t n_rows, float *row_score)
{
    for (int64_t r = 0; r < n_rows; ++r) {
        const float *x = X + r * (int64_t)n_features;
        float acc = bias;
        for (int32_t t = 0; t < n_trees; ++t) {
            int32_t o = tree_off[t];
            int32_t leaf = fso_leaf(split_feature + o, threshold + o, left + o, right + o, x);
            acc = acc + value[o + leaf];
        }
        row_score[r] = acc;
    }
}

/* prog_score[p] = sum over the program's rows (ascending), starting from +0. */
void fso_program_scores(const float *row_score, const int32_t *prog_off, int32_t n_programs,
                        float *prog_score)
{
    for (int32_t p = 0; p < n_programs; ++p) {
        float acc = 0.0f;
        for (int32_t r = prog_off[p]; r < prog_off[p + 1]; ++r)
            acc = acc + row_score[r];
        prog_score[p] = acc;
    }
}

/* Rows straight to program scores for programs [p_begin, p_end): used to score a range
 * (or, called repeatedly, a sample) of programs without materialising all row scores. */
void fso_score_programs(int32_t n_features, int32_t n_trees, const int32_t *tree_off,
                        const int32_t *split_feature, const float *threshold,
                        const int32_t *left, const int32_t *right, const float *value,
                        float bias, const float *X, const int32_t *prog_off,
                        int32_t p_begin, int32_t p_end, float *prog_score)
{
    for (int32_t p = p_begin; p < p_end; ++p) {
        float acc = 0.0f;
        for (int32_t r = prog_off[p]; r < prog_off[p + 1]; ++r) {
            float rs;
            fso_row_scores(n_features, n_trees, tree_off, split_feature, threshold, left,
                           right, value, bias, X + (int64_t)r * n_features, 1, &rs);
            acc = acc + rs;
        }
        prog_score[p] = acc;
    }
}

/* 1 if program a orders before program b: higher score first, equal scores by lower
 * index (guaranteed by the stable sort), NaN after every number. */
static int fso_before(float a, float b)
{
    int an = isnan(a), bn = isnan(b);
    if (an || bn)
        return !an && bn;
    return a > b; /* -0 > +0 is false both ways: they tie */
}

static void fso_merge_sort(int32_t *idx, int32_t *tmp, const float *score, int32_t lo, int32_t hi)
{
    if (hi - lo < 2)
        return;
    int32_t mid = lo + (hi - lo) / 2;
    fso_merge_sort(idx, tmp, score, lo, mid);
    fso_merge_sort(idx, tmp, score, mid, hi);
    int32_t i = lo, j = mid, o = lo;
    while (i < mid && j < hi) {
        /* take from the right run only if it is strictly before: keeps the sort stable */
        if (fso_before(score[idx[j]], score[idx[i]]))
            tmp[o++] = idx[j++];
        else
            tmp[o++] = idx[i++];
    }
    while (i < mid)
        tmp[o++] = idx[i++];
    while (j < hi)
        tmp[o++] = idx[j++];
    memcpy(idx + lo, tmp + lo, (size_t)(hi - lo) * sizeof(int32_t));
}

/* Full sort, then cut.  Returns 0, or -1 if memory could not be obtained. */
int fso_topk(const float *score, int32_t n, int32_t k, int32_t *out_idx, float *out_score)
{
    int32_t *idx = NULL, *tmp = NULL;
    if (n > 0) {
        idx = (int32_t *)malloc((size_t)n * sizeof(int32_t));
        tmp = (int32_t *)malloc((size_t)n * sizeof(int32_t));
        if (!idx || !tmp) {
            free(idx);
            free(tmp);
            return -1;
        }
        for (int32_t i = 0; i < n; ++i)
            idx[i] = i;
        fso_merge_sort(idx, tmp, score, 0, n);
    }
    for (int32_t j = 0; j < k; ++j) {
        if (j < n) {
            out_idx[j] = idx[j];
            out_score[j] = score[idx[j]];
        } else {
            out_idx[j] = -1;
            out_score[j] = -INFINITY;
        }
    }
    free(idx);
    free(tmp);
    return 0;
}
