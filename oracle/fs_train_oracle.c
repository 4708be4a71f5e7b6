/*
 * CPU oracle for training a family's gradient-boosted-tree cost model.  TEST
 * INFRASTRUCTURE ONLY: nothing on the product path may call, link or load this file.
 *
 * The tuner of the paper retrains the family's cost model on the measured candidates after
 * every tuning step (Algorithm 1, train_cost_model; Section 4.2 "the evaluated candidates
 * are used to update the family cost model") and Section 4.3 moves that training to the GPU.
 * The paper names the model (XGBoost) and nothing else, so what is trained here is the
 * published second-order boosting step of that method (Chen & Guestrin 2016, Eq. 4-7) on
 * pre-binned features, under the readings listed below.
 *
 * Setting.  A program p owns the statement rows [off[p], off[p+1]); the model's score of a
 * program is the sum of its row outputs F(x_r) (as in scoring), and one measured target y_p
 * exists per program.  Loss: 1/2 * sum_p (s_p - y_p)^2 with s_p = sum_{r in p} F(x_r).
 *
 * One boosting round:
 *   s_p      = row outputs so far, added in row order from +0 (float)
 *   g_p      = s_p - y_p (float);  every row of p carries gradient g_p and curvature
 *              h_r = number of rows of p  (an upper bound of the loss curvature along any
 *              leaf, so a step with eta <= 1 never increases the loss)
 *   q_p      = (int32) rintf(clamp(g_p * grad_scale, +-2147483520)): gradients are summed as
 *              integers, so histogram sums do not depend on the order of the rows
 *   tree     grown level by level, nodes numbered breadth-first.  For a node with integer
 *            sums (G, H) over its rows, every feature f (ascending) and every cut
 *            j = 1..m_f (ascending) with c = cuts_f[j-1] splits it into the rows with
 *            x_f < c (left) and the others (right; NaN goes right).  In double:
 *              gain = gl*gl/(HL+lambda) + gr*gr/(HR+lambda) - g*g/(H+lambda),
 *              gl = GL/grad_scale etc.
 *            a split is admissible if HL, HR >= max(min_child_weight, 1); the first split
 *            with the largest gain wins; the node is split if that gain > min_gain and its
 *            depth < max_depth, else it is a leaf with
 *              value = (float)(-eta * g / (H + lambda))
 *   F(x_r)  += value of the leaf that holds r (float)
 *
 * Readings (the paper is silent on all of them): squared loss on program sums; diagonal
 * curvature h_r = rows of the program; fixed-point gradients; cut points are an input (any
 * ascending list of distinct floats per feature); strict '<' goes left as in scoring, so the
 * trained arrays can be handed to the scoring path unchanged.
 *
 * Pins: tests/test_train_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Number of cuts that are <= x; a NaN takes the last bin (it fails every '<'). */
static int32_t bin_of(const float *cuts, int32_t m, float x)
{
    if (x != x)
        return m;
    int32_t b = 0;
    while (b < m && cuts[b] <= x)
        ++b;
    return b;
}

static int32_t quantize(float g, float grad_scale)
{
    float t = g * grad_scale;
    t = fmaxf(t, -2147483520.0f);
    t = fminf(t, 2147483520.0f);
    return (int32_t)rintf(t);
}

static double split_gain(int64_t GL, int64_t HL, int64_t G, int64_t H, double inv_scale,
                         double lambda)
{
    const int64_t GR = G - GL, HR = H - HL;
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

/*
 * Train n_rounds trees.  X is row-major n_rows x n_features.  cuts of feature f are
 * cuts[cut_off[f] .. cut_off[f+1]).  Outputs: the trees in the flat arrays the scoring
 * oracle reads (tree_off has n_rounds+1 entries; node arrays hold up to node_cap nodes),
 * the final row outputs and program sums, and the loss before every round and after the
 * last (n_rounds+1 doubles).  Returns 0, or -1 on bad arguments / too small node_cap /
 * allocation failure.
 */
int fso_train(int32_t n_features, int64_t n_rows, const float *X, const int32_t *prog_off,
              int32_t n_programs, const float *target, const int32_t *cut_off,
              const float *cuts, float bias, int32_t n_rounds, int32_t max_depth, float eta,
              float lambda, float min_gain, float min_child_weight, float grad_scale,
              int32_t *tree_off, int32_t *split_feature, float *threshold, int32_t *left,
              int32_t *right, float *value, int64_t node_cap, float *row_pred,
              float *prog_pred, double *loss)
{
    if (n_rows < 1 || n_programs < 1 || n_features < 1 || max_depth < 0 || n_rounds < 0)
        return -1;
    const double inv_scale = 1.0 / (double)grad_scale;
    const double lam = (double)lambda, eta_d = (double)eta;
    int64_t mcw = (int64_t)ceil((double)min_child_weight);
    if (mcw < 1)
        mcw = 1;
    int32_t max_bins = 0;
    for (int32_t f = 0; f < n_features; ++f)
        if (cut_off[f + 1] - cut_off[f] + 1 > max_bins)
            max_bins = cut_off[f + 1] - cut_off[f] + 1;

    int32_t *q_row = malloc(sizeof(int32_t) * (size_t)n_rows);       /* gradient of the row   */
    int32_t *h_row = malloc(sizeof(int32_t) * (size_t)n_rows);       /* curvature of the row  */
    int64_t *rows = malloc(sizeof(int64_t) * (size_t)n_rows);        /* rows grouped by node  */
    int64_t *tmp = malloc(sizeof(int64_t) * (size_t)n_rows);
    int64_t *hist_g = malloc(sizeof(int64_t) * (size_t)max_bins);
    int64_t *hist_h = malloc(sizeof(int64_t) * (size_t)max_bins);
    /* per node of the tree being grown: its row range in `rows`, depth */
    const int64_t tree_cap = ((int64_t)1 << (max_depth + 1)) - 1;
    int64_t *node_begin = malloc(sizeof(int64_t) * (size_t)tree_cap);
    int64_t *node_end = malloc(sizeof(int64_t) * (size_t)tree_cap);
    int32_t *node_depth = malloc(sizeof(int32_t) * (size_t)tree_cap);
    if (!q_row || !h_row || !rows || !tmp || !hist_g || !hist_h || !node_begin || !node_end ||
        !node_depth)
        return -1;

    for (int64_t r = 0; r < n_rows; ++r)
        row_pred[r] = bias;
    for (int32_t p = 0; p < n_programs; ++p)
        for (int64_t r = prog_off[p]; r < prog_off[p + 1]; ++r)
            h_row[r] = prog_off[p + 1] - prog_off[p];

    int64_t n_nodes_total = 0;
    tree_off[0] = 0;
    for (int32_t round = 0; round <= n_rounds; ++round) {
        /* program sums, loss, gradients */
        double l = 0.0;
        for (int32_t p = 0; p < n_programs; ++p) {
            float s = 0.0f;
            for (int64_t r = prog_off[p]; r < prog_off[p + 1]; ++r)
                s = s + row_pred[r];
            prog_pred[p] = s;
            const float g = s - target[p];
            l += 0.5 * (double)g * (double)g;
            const int32_t q = quantize(g, grad_scale);
            for (int64_t r = prog_off[p]; r < prog_off[p + 1]; ++r)
                q_row[r] = q;
        }
        loss[round] = l;
        if (round == n_rounds)
            break;

        /* grow one tree, breadth-first */
        const int64_t base = n_nodes_total;
        int64_t n_nodes = 1;
        for (int64_t r = 0; r < n_rows; ++r)
            rows[r] = r;
        node_begin[0] = 0;
        node_end[0] = n_rows;
        node_depth[0] = 0;
        for (int64_t n = 0; n < n_nodes; ++n) {
            if (base + n >= node_cap)
                return -1;
            int64_t G = 0, H = 0;
            for (int64_t i = node_begin[n]; i < node_end[n]; ++i) {
                G += q_row[rows[i]];
                H += h_row[rows[i]];
            }
            double best = 0.0;
            int32_t best_f = -1, best_j = 0;
            if (node_depth[n] < max_depth) {
                for (int32_t f = 0; f < n_features; ++f) {
                    const float *cf = cuts + cut_off[f];
                    const int32_t m = cut_off[f + 1] - cut_off[f];
                    for (int32_t b = 0; b <= m; ++b)
                        hist_g[b] = hist_h[b] = 0;
                    for (int64_t i = node_begin[n]; i < node_end[n]; ++i) {
                        const int64_t r = rows[i];
                        const int32_t b = bin_of(cf, m, X[r * (int64_t)n_features + f]);
                        hist_g[b] += q_row[r];
                        hist_h[b] += h_row[r];
                    }
                    int64_t GL = 0, HL = 0;
                    for (int32_t j = 1; j <= m; ++j) {       /* left = bins 0..j-1 */
                        GL += hist_g[j - 1];
                        HL += hist_h[j - 1];
                        if (HL < mcw || H - HL < mcw)
                            continue;
                        const double gain = split_gain(GL, HL, G, H, inv_scale, lam);
                        if (best_f < 0 || gain > best) {
                            best = gain;
                            best_f = f;
                            best_j = j;
                        }
                    }
                }
            }
            const int64_t id = base + n;
            if (best_f >= 0 && best > (double)min_gain) {
                const float c = cuts[cut_off[best_f] + best_j - 1];
                int64_t nl = 0, nr = 0;
                for (int64_t i = node_begin[n]; i < node_end[n]; ++i) {
                    const int64_t r = rows[i];
                    if (X[r * (int64_t)n_features + best_f] < c)
                        rows[node_begin[n] + nl++] = r;      /* nl <= i - begin: no overwrite */
                    else
                        tmp[nr++] = r;
                }
                for (int64_t i = 0; i < nr; ++i)
                    rows[node_begin[n] + nl + i] = tmp[i];
                split_feature[id] = best_f;
                threshold[id] = c;
                left[id] = (int32_t)n_nodes;
                right[id] = (int32_t)n_nodes + 1;
                value[id] = 0.0f;
                node_begin[n_nodes] = node_begin[n];
                node_end[n_nodes] = node_begin[n] + nl;
                node_depth[n_nodes] = node_depth[n] + 1;
                node_begin[n_nodes + 1] = node_begin[n] + nl;
                node_end[n_nodes + 1] = node_end[n];
                node_depth[n_nodes + 1] = node_depth[n] + 1;
                n_nodes += 2;
            } else {
                const double g = (double)G * inv_scale;
                const float w = (float)(-eta_d * g / ((double)H + lam));
                split_feature[id] = -1;
                threshold[id] = 0.0f;
                left[id] = right[id] = -1;
                value[id] = w;
                for (int64_t i = node_begin[n]; i < node_end[n]; ++i)
                    row_pred[rows[i]] = row_pred[rows[i]] + w;
            }
        }
        n_nodes_total += n_nodes;
        tree_off[round + 1] = (int32_t)n_nodes_total;
    }
    free(q_row); free(h_row); free(rows); free(tmp); free(hist_g); free(hist_h);
    free(node_begin); free(node_end); free(node_depth);
    return 0;
}

/* Bin index of every entry of a row-major matrix (what the histogram counts). */
void fso_bins(int32_t n_features, int64_t n_rows, const float *X, const int32_t *cut_off,
              const float *cuts, int32_t *bins)
{
    for (int64_t r = 0; r < n_rows; ++r)
        for (int32_t f = 0; f < n_features; ++f)
            bins[r * (int64_t)n_features + f] =
                bin_of(cuts + cut_off[f], cut_off[f + 1] - cut_off[f], X[r * (int64_t)n_features + f]);
}
