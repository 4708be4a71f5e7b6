"""Pins for the CPU oracle: every check here compares `oracle/` with something that is
not the oracle -- a value worked out by hand, a closed form, a count, a library routine
that solves a special case, or an invariant of the definition (Section 2 "Building the
Cost Model": a boosted-tree model scores each candidate; Section 3.2: candidates are
ordered by the estimate and the top k are kept).  A dropped term, a flipped comparison,
a swapped child or an off-by-one in the CSR walk fails at least one of them.
"""
import itertools
import os

import numpy as np
import pytest

from paper_2201_00194_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def model_from_trees(trees, n_features, bias=0.0):
    """trees: list of lists of nodes; a node is ('s', f, thr, l, r) or ('l', value)."""
    tree_off = [0]
    sf, th, le, ri, va = [], [], [], [], []
    for t in trees:
        for n in t:
            if n[0] == "s":
                sf.append(n[1]); th.append(n[2]); le.append(n[3]); ri.append(n[4]); va.append(0.0)
            else:
                sf.append(-1); th.append(0.0); le.append(-1); ri.append(-1); va.append(n[1])
        tree_off.append(len(sf))
    return W.Model(n_features, np.array(tree_off, np.int32), np.array(sf, np.int32),
                   np.array(th, np.float32), np.array(le, np.int32), np.array(ri, np.int32),
                   np.array(va, np.float32), bias)


def hand_model():
    t0 = [("s", 0, 0.5, 1, 2), ("s", 1, 0.25, 3, 4), ("l", 1.0), ("l", -2.0),
          ("s", 2, 0.75, 5, 6), ("l", 4.0), ("l", 8.0)]
    t1 = [("s", 2, 0.0, 1, 2), ("l", 100.0), ("l", 0.125)]
    return model_from_trees([t0, t1], 3, bias=0.5)


def read_golden():
    rows, leaves, scores = [], [], []
    meta = {}
    with open(os.path.join(GOLDEN, "hand_tree_depth3.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, rest = line.split(None, 1)
            if key == "row":
                a, b, c, d = [s.strip() for s in rest.split("|")]
                rows.append([float(v) for v in a.split()])
                leaves.append([int(b), int(c)])
                scores.append(float(d))
            else:
                meta[key] = [float(v) for v in rest.split()]
    return (np.array(rows, np.float32), np.array(leaves, np.int32), np.array(scores, np.float32),
            np.array(meta["prog_off"], np.int32), np.array(meta["prog_score"], np.float32),
            np.array(meta["top3"], np.int32))


# ---- P1: hand-built trees, expected values typed in the fixture ---------------------

def test_hand_built_trees_match_values_worked_by_hand(oracle):
    X, leaves, scores, off, pscore, top3 = read_golden()
    m = hand_model()
    assert np.array_equal(oracle.leaf_indices(m, X), leaves)
    rs = oracle.row_scores(m, X)
    assert np.array_equal(rs, scores)
    ps = oracle.program_scores(rs, off)
    assert np.array_equal(ps, pscore)
    assert np.array_equal(oracle.score_programs(m, X, off), pscore)
    idx, val = oracle.topk(ps, 3)
    assert np.array_equal(idx, top3)
    assert np.array_equal(val, pscore[top3])


def test_brute_force_grid_depth3_full_tree(oracle):
    """Full depth-3 tree over 3 features on a grid of rows that includes values equal to
    the thresholds.  The expected leaf is written as a closed form: a full tree in heap
    order that splits on feature `level` at every node of that level ends in leaf
    7 + (b0 b1 b2) with b_level = [x_level >= thr of the node reached]."""
    thr = {0: 0.5, 1: 0.25, 2: 0.75, 3: 0.1, 4: 0.9, 5: 0.3, 6: 0.6}
    level_of = {0: 0, 1: 1, 2: 1, 3: 2, 4: 2, 5: 2, 6: 2}
    nodes = [("s", level_of[n], thr[n], 2 * n + 1, 2 * n + 2) for n in range(7)]
    leaf_vals = [float(1 << j) for j in range(8)]            # distinct powers of two
    nodes += [("l", v) for v in leaf_vals]
    m = model_from_trees([nodes], 3, bias=0.0)
    grid = sorted(set(thr.values()) | {0.0, 0.05, 0.2, 0.4, 0.55, 0.7, 0.8, 0.95})
    rows = np.array(list(itertools.product(grid, repeat=3)), np.float32)
    expect = []
    for x in rows:
        n = 0
        for _ in range(3):
            t = np.float32(thr[n])
            n = 2 * n + (2 if not (x[level_of[n]] < t) else 1)
        expect.append(n)
    expect = np.array(expect, np.int32)
    got = oracle.leaf_indices(m, rows)[:, 0]
    assert np.array_equal(got, expect)
    assert set(np.unique(got)) == set(range(7, 15))          # every leaf is reachable
    assert np.array_equal(oracle.row_scores(m, rows),
                          np.array([leaf_vals[n - 7] for n in expect], np.float32))


# ---- P2: depth-0 ensembles return the bias ------------------------------------------

def test_single_leaf_tree_returns_bias(oracle):
    m = model_from_trees([[("l", 0.0)]], 5, bias=0.3)
    X = np.random.default_rng(1).random((9, 5), dtype=np.float32)
    rs = oracle.row_scores(m, X)
    assert np.array_equal(rs, np.full(9, np.float32(0.3)))
    assert np.array_equal(oracle.leaf_indices(m, X), np.zeros((9, 1), np.int32))
    # one statement per program: the program score is the bias itself
    off1 = np.arange(10, dtype=np.int32)
    assert np.array_equal(oracle.program_scores(rs, off1), rs)
    # dyadic bias, s statements: s * bias exactly (the bias is per row)
    m2 = model_from_trees([[("l", 0.0)]], 5, bias=0.375)
    off = np.array([0, 1, 4, 9], np.int32)
    ps = oracle.score_programs(m2, X, off)
    assert np.array_equal(ps, np.array([0.375, 3 * 0.375, 5 * 0.375], np.float32))


# ---- P3: permutation of programs -----------------------------------------------------

def test_program_permutation_invariance(oracle):
    fam = W.make_small_family(seed=3, n_programs=200, stmts=(1, 9), n_trees=20, depth=5)
    ps = oracle.score_programs(fam.model, fam.features, fam.prog_off)
    rng = np.random.default_rng(5)
    perm = rng.permutation(fam.n_programs)            # new program j is old program perm[j]
    off = fam.prog_off
    rows = np.concatenate([np.arange(off[p], off[p + 1]) for p in perm])
    lens = (off[1:] - off[:-1])[perm]
    off2 = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ps2 = oracle.score_programs(fam.model, fam.features[rows], off2)
    assert np.array_equal(ps2, ps[perm])              # bit-identical: per-program order kept
    assert np.unique(ps).shape[0] == ps.shape[0]      # distinct scores => a unique ranking
    k = 17
    idx, val = oracle.topk(ps, k)
    idx2, val2 = oracle.topk(ps2, k)
    assert np.array_equal(perm[idx2], idx)
    assert np.array_equal(val2, val)


# ---- P4/P7: dyadic leaves, duplicate trees -------------------------------------------

def test_dyadic_leaves_sum_is_order_free_and_matches_integer_arithmetic(oracle):
    fam = W.make_small_family(seed=11, n_programs=64, stmts=(1, 12), n_trees=50, depth=4,
                              early_leaf_q=0.25, dyadic_leaves=True)
    m = fam.model
    li = oracle.leaf_indices(m, fam.features)
    # exact integer arithmetic on value*1024, gathered with numpy from the leaf ids
    iv = np.rint(m.value.astype(np.float64) * 1024).astype(np.int64)
    per_row = iv[(m.tree_off[:-1][None, :] + li)].sum(axis=1)
    rs = oracle.row_scores(m, fam.features)
    assert np.array_equal(rs.astype(np.float64) * 1024, per_row.astype(np.float64))
    off = fam.prog_off
    per_prog = np.array([per_row[off[p]:off[p + 1]].sum() for p in range(fam.n_programs)])
    ps = oracle.program_scores(rs, off)
    assert np.array_equal(ps.astype(np.float64) * 1024, per_prog.astype(np.float64))


def test_duplicate_tree_linearity(oracle):
    fam = W.make_small_family(seed=12, n_programs=30, stmts=(2, 2), n_trees=1, depth=5,
                              dyadic_leaves=True)
    m1 = fam.model
    T = 37
    n = m1.n_nodes
    mT = W.Model(m1.n_features, (np.arange(T + 1) * n).astype(np.int32),
                 np.tile(m1.split_feature, T), np.tile(m1.threshold, T), np.tile(m1.left, T),
                 np.tile(m1.right, T), np.tile(m1.value, T), 0.0)
    r1 = oracle.row_scores(m1, fam.features)
    rT = oracle.row_scores(mT, fam.features)
    assert np.array_equal(rT, np.float32(T) * r1)
    assert np.array_equal(oracle.leaf_indices(mT, fam.features),
                          np.repeat(oracle.leaf_indices(m1, fam.features), T, axis=1))


# ---- P5: a threshold chain is a binary search ----------------------------------------

def test_threshold_chain_tree_equals_searchsorted(oracle):
    d = 4
    n_int = (1 << d) - 1
    thr_sorted = np.sort(np.random.default_rng(2).random(n_int, dtype=np.float32))
    # in-order rank of heap node n in a full tree of depth d
    def inorder_rank(n):
        level = int(np.floor(np.log2(n + 1)))
        pos = n + 1 - (1 << level)
        span = 1 << (d - level)
        return pos * span + span // 2 - 1
    nodes = [("s", 1, float(thr_sorted[inorder_rank(n)]), 2 * n + 1, 2 * n + 2)
             for n in range(n_int)]
    nodes += [("l", float(j)) for j in range(1 << d)]       # leaf j outputs its bucket
    m = model_from_trees([nodes], 3)
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.random(300, dtype=np.float32), thr_sorted,       # equality cases
                        np.array([0.0, 1.0, -1.0], np.float32)])
    X = np.zeros((x.shape[0], 3), np.float32)
    X[:, 1] = x
    bucket = np.searchsorted(thr_sorted, x, side="right")   # #thresholds <= x
    assert np.array_equal(oracle.leaf_indices(m, X)[:, 0], n_int + bucket.astype(np.int32))
    assert np.array_equal(oracle.row_scores(m, X), bucket.astype(np.float32))


# ---- P6: a depth-1 tree counts -------------------------------------------------------

def test_depth1_tree_counts_rows_below_threshold(oracle):
    rng = np.random.default_rng(8)
    X = W.draw_features(rng, 500, 0.3, n_features=7)
    tau = np.float32(X[17, 4])
    a, b = 0.25, -3.0
    m = model_from_trees([[("s", 4, float(tau), 1, 2), ("l", a), ("l", b)]], 7)
    off = W.uniform_prog_off(rng, 60, 0, 14)
    X = X[: off[-1]]
    ps = oracle.score_programs(m, X, off)
    below = X[:, 4] < tau
    exp = np.array([a * below[off[p]:off[p + 1]].sum() + b * (~below[off[p]:off[p + 1]]).sum()
                    for p in range(60)], np.float32)
    assert np.array_equal(ps, exp)
    # rows equal to the threshold are NOT below it
    assert (X[:, 4] == tau).any()


# ---- P8: CSR identities --------------------------------------------------------------

def test_csr_identities(oracle):
    rs = (np.random.default_rng(9).integers(-500, 500, 1000) / 64.0).astype(np.float32)
    assert np.array_equal(oracle.program_scores(rs, np.arange(1001, dtype=np.int32)), rs)
    total = oracle.program_scores(rs, np.array([0, 1000], np.int32))
    acc = np.float32(0)
    for v in rs:
        acc = np.float32(acc + v)
    assert total[0] == acc
    ps = oracle.program_scores(rs, np.array([0, 0, 5, 5, 1000], np.int32))
    assert ps[0] == 0 and ps[2] == 0 and not np.signbit(ps[0])
    assert ps[1] == np.float32(rs[:5].astype(np.float64).sum())   # dyadic => exact
    # sequential fp32 order matters and is the ascending one
    tricky = np.array([1e8, 1.0, -1e8, 1.0], np.float32)
    assert oracle.program_scores(tricky, np.array([0, 4], np.int32))[0] == np.float32(1.0)


# ---- P9: power-of-two rescale of a column leaves every leaf unchanged ----------------

def test_power_of_two_column_rescale_keeps_leaves(oracle):
    fam = W.make_small_family(seed=21, n_programs=40, stmts=(3, 3), n_trees=30, depth=6,
                              early_leaf_q=0.2)
    m = fam.model
    li = oracle.leaf_indices(m, fam.features)
    X2 = fam.features.copy()
    thr2 = m.threshold.copy()
    for j, e in ((3, 5), (100, -7), (163, 12)):
        X2[:, j] = np.ldexp(X2[:, j], e)
        sel = m.split_feature == j
        thr2[sel] = np.ldexp(thr2[sel], e)
    m2 = W.Model(m.n_features, m.tree_off, m.split_feature, thr2, m.left, m.right, m.value, 0.0)
    assert np.array_equal(oracle.leaf_indices(m2, X2), li)


# ---- P10: top-k against library routines --------------------------------------------

def test_topk_reduces_to_library_routines(oracle):
    rng = np.random.default_rng(13)
    s = rng.standard_normal(777).astype(np.float32)
    s[rng.integers(0, 777, 200)] = s[rng.integers(0, 777, 200)]      # plant many ties
    idx, val = oracle.topk(s, 777)
    assert np.array_equal(idx, np.argsort(-s, kind="stable").astype(np.int32))
    assert np.array_equal(val, s[idx])
    i1, _ = oracle.topk(s, 1)
    assert i1[0] == int(np.argmax(s))                                 # first maximum
    ik, _ = oracle.topk(s, 50)
    assert np.array_equal(ik, idx[:50])
    same = np.full(40, np.float32(2.5))
    assert np.array_equal(oracle.topk(same, 12)[0], np.arange(12, dtype=np.int32))
    # ties across the cut: lower indices win
    t = np.array([1, 5, 3, 5, 3, 3, 0, 3], np.float32)
    assert np.array_equal(oracle.topk(t, 4)[0], np.array([1, 3, 2, 4], np.int32))
    # k > n pads with (-1, -inf); k = 0 and n = 0 are fine
    i, v = oracle.topk(t, 11)
    assert np.array_equal(i[8:], [-1, -1, -1]) and np.all(np.isneginf(v[8:]))
    assert oracle.topk(t, 0)[0].shape == (0,)
    i, v = oracle.topk(np.zeros(0, np.float32), 3)
    assert np.array_equal(i, [-1, -1, -1]) and np.all(np.isneginf(v))


def test_topk_signed_zero_nan_and_infinities(oracle):
    s = np.array([0.0, -0.0, np.nan, -np.inf, np.inf, -0.0, 0.0, np.nan, -1.0], np.float32)
    idx, val = oracle.topk(s, 9)
    assert np.array_equal(idx, np.array([4, 0, 1, 5, 6, 8, 3, 2, 7], np.int32))


# ---- P11: fp64 shadow sets the tolerance ---------------------------------------------

def test_fp32_scores_stay_within_tolerance_of_fp64_sum(oracle):
    fam = W.make_small_family(seed=31, n_programs=100, stmts=(1, 32), n_trees=300, depth=6)
    m = fam.model
    li = oracle.leaf_indices(m, fam.features)
    v64 = m.value.astype(np.float64)[(m.tree_off[:-1][None, :] + li)].sum(axis=1) + m.bias
    off = fam.prog_off
    p64 = np.array([v64[off[p]:off[p + 1]].sum() for p in range(fam.n_programs)])
    ps = oracle.score_programs(m, fam.features, off).astype(np.float64)
    assert np.all(np.abs(ps - p64) <= 1e-5 * np.abs(p64) + 1e-6 + 32 * 300 * 2.0 ** -24 * 0.05)


# ---- P12: thresholds at zero never send a non-negative feature left ------------------

def test_zero_threshold_left_subtrees_unreachable(oracle):
    fam = W.make_small_family(seed=41, n_programs=300, stmts=(4, 4), n_trees=40, depth=5,
                              zero_frac=0.5)
    m = fam.model
    li = oracle.leaf_indices(m, fam.features)
    assert (m.threshold[m.split_feature >= 0] == 0).any()
    for t in range(m.n_trees):
        o = m.tree_off[t]
        n_t = m.tree_off[t + 1] - o
        dead = set()
        for n in range(n_t):
            if m.split_feature[o + n] >= 0 and m.threshold[o + n] == 0:
                stack = [int(m.left[o + n])]
                while stack:
                    c = stack.pop()
                    dead.add(c)
                    if m.split_feature[o + c] >= 0:
                        stack += [int(m.left[o + c]), int(m.right[o + c])]
        assert not (set(np.unique(li[:, t]).tolist()) & dead)


def test_nan_feature_goes_right(oracle):
    m = model_from_trees([[("s", 0, 0.5, 1, 2), ("l", 1.0), ("l", 2.0)]], 1)
    X = np.array([[np.nan], [0.4], [0.5], [np.inf], [-np.inf]], np.float32)
    assert np.array_equal(oracle.leaf_indices(m, X)[:, 0], [2, 1, 2, 2, 1])


# ---- cross-checks of the oracle's own entry points and of the threaded driver --------

def test_entry_points_agree_and_threads_do_not_change_bits(oracle):
    fam = W.make_small_family(seed=51, n_programs=500, stmts=(1, 20), n_trees=25, depth=6,
                              early_leaf_q=0.2)
    rs = oracle.row_scores(fam.model, fam.features)
    ps = oracle.program_scores(rs, fam.prog_off)
    assert np.array_equal(oracle.score_programs(fam.model, fam.features, fam.prog_off), ps)
    assert np.array_equal(
        oracle.score_programs(fam.model, fam.features, fam.prog_off, threads=4), ps)
    sample = np.array([0, 7, 499, 250], np.int64)
    assert np.array_equal(
        oracle.score_program_sample(fam.model, fam.features, fam.prog_off, sample), ps[sample])
    # independent numpy walk of the definition on a few rows
    m = fam.model
    for r in (0, 13, fam.n_rows - 1):
        acc = np.float32(m.bias)
        for t in range(m.n_trees):
            o = m.tree_off[t]
            n = 0
            while m.split_feature[o + n] >= 0:
                go_left = fam.features[r, m.split_feature[o + n]] < m.threshold[o + n]
                n = m.left[o + n] if go_left else m.right[o + n]
            acc = np.float32(acc + m.value[o + n])
        assert rs[r] == acc


def test_gather_programs_is_plain_indexing(oracle):
    """With one row per program the gather is numpy's fancy indexing; with longer programs it
    is the concatenation of the selected row slices; -1 stands for an empty program."""
    rng = np.random.default_rng(9)
    X = rng.standard_normal((40, 6)).astype(np.float32)
    sc = rng.standard_normal(40).astype(np.float32)
    keep = rng.integers(0, 40, 25)
    f, off, s = oracle.gather_programs([(X, np.arange(41, dtype=np.int32), sc)], keep)
    assert np.array_equal(f, X[keep]) and np.array_equal(off, np.arange(26)) and np.array_equal(s, sc[keep])
    # two sources, ragged programs, by hand
    A = np.arange(12, dtype=np.float32).reshape(6, 2)
    B = 100 + np.arange(8, dtype=np.float32).reshape(4, 2)
    offA, offB = np.array([0, 1, 4, 6], np.int32), np.array([0, 0, 4], np.int32)
    f, off, s = oracle.gather_programs([(A, offA, np.array([1., 2., 3.], np.float32)), (B, offB, None)],
                                       [4, -1, 1, 3, 0])
    assert off.tolist() == [0, 4, 4, 7, 7, 8]
    assert np.array_equal(f, np.concatenate([B[0:4], A[1:4], A[0:1]]))
    assert s[2] == 2.0 and s[4] == 1.0 and np.isneginf(s[0]) and np.isneginf(s[1]) and np.isneginf(s[3])
