"""Pins for the training oracle (`oracle/fs_train_oracle.c`): every check compares it with
something other than itself -- a library routine, a closed form worked out by hand, a
numeric minimiser, the scoring oracle (an independent code path), or an invariant of the
method (Chen & Guestrin 2016, Eq. 4-7; the paper's Algorithm 1 only names the step,
train_cost_model).  All CPU."""
from fractions import Fraction

import numpy as np
import pytest
from scipy.optimize import minimize_scalar

from paper_2201_00194_amd import workloads as W

SCALE = float(1 << 20)


@pytest.fixture(scope="module")
def T():
    from oracle import train_oracle
    train_oracle.build()
    return train_oracle


def one_per_program(n):
    return np.arange(n + 1, dtype=np.int32)


def all_cuts(X):
    return W.draw_cuts(X, max_cuts=10**6)


def test_bins_are_searchsorted_right_and_nan_takes_the_last_bin(T):
    rng = np.random.default_rng(0)
    X = W.draw_features(rng, 300, 0.3, n_features=5)
    X[3, 1] = np.nan
    X[7, 2] = np.inf
    X[9, 0] = -0.0
    off, cuts = W.draw_cuts(X, 16)
    got = T.bins(X, off, cuts)
    for f in range(5):
        c = cuts[off[f]:off[f + 1]]
        exp = np.searchsorted(c, X[:, f], side="right")
        exp[np.isnan(X[:, f])] = c.shape[0]
        assert np.array_equal(got[:, f], exp)


def test_depth0_round_is_the_regularised_mean_residual(T):
    # one statement per program => h = 1; a single leaf: w = eta * sum(y - bias) / (P + lambda)
    y = np.array([0.5, -1.25, 2.0, 0.75, 3.0], np.float32)          # dyadic: quantisation exact
    X = np.zeros((5, 1), np.float32)
    off, cuts = all_cuts(X)
    r = T.train(X, one_per_program(5), y, off, cuts, bias=0.25, n_rounds=1, max_depth=0,
                eta=0.5, lam=3.0)
    w = Fraction(1, 2) * sum(Fraction(float(v)) - Fraction(1, 4) for v in y) / (5 + 3)
    assert r.split_feature.tolist() == [-1] and r.tree_off.tolist() == [0, 1]
    assert r.value[0] == np.float32(float(w))
    assert np.array_equal(r.row_pred, np.full(5, np.float32(0.25) + np.float32(float(w)), np.float32))
    # multi-statement programs: every row carries its program's residual and h = rows of the program
    offs = np.array([0, 2, 5], np.int32)
    y2 = np.array([1.0, -2.0], np.float32)
    X2 = np.zeros((5, 1), np.float32)
    r2 = T.train(X2, offs, y2, *all_cuts(X2), n_rounds=1, max_depth=0, eta=1.0, lam=0.0)
    G = 2 * (0 - 1.0) + 3 * (0 + 2.0)                                # sum over rows of s_p - y_p
    H = 2 * 2 + 3 * 3
    assert r2.value[0] == np.float32(-G / H)


def test_step_function_is_recovered_exactly(T):
    x = (np.arange(16, dtype=np.float32) / 16).reshape(-1, 1)
    y = np.where(x[:, 0] < 0.4375, np.float32(-1.5), np.float32(2.25)).astype(np.float32)
    r = T.train(x, one_per_program(16), y, *all_cuts(x), n_rounds=1, max_depth=1, eta=1.0, lam=0.0)
    assert r.split_feature.tolist() == [0, -1, -1]
    assert r.threshold[0] == np.float32(0.4375) and r.left[0] == 1 and r.right[0] == 2
    assert r.value[1] == np.float32(-1.5) and r.value[2] == np.float32(2.25)
    assert np.array_equal(r.prog_pred, y) and r.loss[1] == 0.0


def test_full_depth_tree_interpolates_distinct_points(T):
    rng = np.random.default_rng(3)
    # greedy splits may peel one point at a time: depth n-1 always suffices
    x = rng.permutation(9).astype(np.float32).reshape(-1, 1)
    y = (rng.permutation(64)[:9] / 8.0 - 4.0).astype(np.float32)     # distinct targets
    r = T.train(x, one_per_program(9), y, *all_cuts(x), n_rounds=1, max_depth=8, eta=1.0,
                lam=0.0, min_gain=-1.0)
    assert np.array_equal(r.prog_pred, y) and r.loss[1] == 0.0


def test_root_split_maximises_the_drop_of_the_second_order_objective(T):
    """For every admissible (feature, cut) the objective after the split is minimised
    numerically over the two leaf weights (no closed form); the oracle's root split must be the
    first one with the largest drop."""
    rng = np.random.default_rng(5)
    for trial in range(6):
        n = 14
        X = rng.integers(0, 5, size=(n, 3)).astype(np.float32)
        y = (rng.integers(-32, 32, n) / 4.0).astype(np.float32)
        lam = float(rng.choice([0.0, 0.5, 2.0]))
        off, cuts = all_cuts(X)
        r = T.train(X, one_per_program(n), y, off, cuts, n_rounds=1, max_depth=1, eta=1.0, lam=lam,
                    min_gain=-1e30)
        g = -y.astype(np.float64)                                   # s = 0, h = 1

        def best_obj(mask):
            gs = g[mask]
            f = lambda w: float(np.sum(gs * w + 0.5 * w * w) + 0.5 * lam * w * w)
            return minimize_scalar(f, bounds=(-100, 100), method="bounded",
                                   options={"xatol": 1e-12}).fun

        parent = best_obj(np.ones(n, bool))
        best = (None, None, -np.inf)
        for f in range(3):
            for c in cuts[off[f]:off[f + 1]]:
                L = X[:, f] < c
                if L.sum() == 0 or (~L).sum() == 0:
                    continue
                drop = parent - best_obj(L) - best_obj(~L)
                if drop > best[2] + 1e-9:
                    best = (f, float(c), drop)
        assert r.split_feature[0] == best[0] and float(r.threshold[0]) == best[1]


def test_loss_never_increases_with_multi_statement_programs(T):
    # eta = 1 and lambda = 0 is the most aggressive step; h = rows-of-program keeps it safe
    ts = W.make_train_set(7, 300, stmts=(1, 24), n_features=12, max_cuts=31)
    r = T.train(ts.features, ts.prog_off, ts.target, ts.cut_off, ts.cuts, n_rounds=25,
                max_depth=4, eta=1.0, lam=0.0)
    assert np.all(np.diff(r.loss) <= 1e-9 * r.loss[0])
    assert r.loss[-1] < 0.2 * r.loss[0]


def test_exported_trees_score_like_the_trainer_itself(T, oracle):
    """The scoring oracle walking the exported arrays (x < threshold) must land every row where
    the trainer put it (bin < cut): two independent code paths, bit-identical sums."""
    ts = W.make_train_set(11, 200, stmts=(1, 9), n_features=10, max_cuts=15)
    ts.features[5, 3] = np.nan                                       # goes right in both
    r = T.train(ts.features, ts.prog_off, ts.target, ts.cut_off, ts.cuts, bias=0.125,
                n_rounds=12, max_depth=5, eta=0.3, lam=1.0)
    m = W.Model(10, r.tree_off, r.split_feature, r.threshold, r.left, r.right, r.value, 0.125)
    rs = oracle.row_scores(m, ts.features)
    assert np.array_equal(rs.view(np.uint32), r.row_pred.view(np.uint32))
    ps = oracle.program_scores(rs, ts.prog_off)
    assert np.array_equal(ps.view(np.uint32), r.prog_pred.view(np.uint32))
    # children come after their parent and ids are local to the tree
    for t in range(12):
        a, b = r.tree_off[t], r.tree_off[t + 1]
        inner = np.nonzero(r.split_feature[a:b] >= 0)[0]
        assert np.all(r.left[a:b][inner] > inner) and np.all(r.right[a:b][inner] == r.left[a:b][inner] + 1)
        assert r.right[a:b].max(initial=0) < b - a


def test_program_order_does_not_change_the_trees(T):
    ts = W.make_train_set(13, 120, stmts=(2, 2), n_features=6, max_cuts=15)
    kw = dict(n_rounds=6, max_depth=3, eta=0.5, lam=1.0)
    a = T.train(ts.features, ts.prog_off, ts.target, ts.cut_off, ts.cuts, **kw)
    perm = np.random.default_rng(1).permutation(120)
    Xp = ts.features.reshape(120, 2, 6)[perm].reshape(240, 6)
    b = T.train(Xp, ts.prog_off, ts.target[perm], ts.cut_off, ts.cuts, **kw)
    for name in ("tree_off", "split_feature", "left", "right"):
        assert np.array_equal(getattr(a, name), getattr(b, name))
    assert np.array_equal(a.threshold.view(np.uint32), b.threshold.view(np.uint32))
    assert np.array_equal(a.value.view(np.uint32), b.value.view(np.uint32))
    assert np.array_equal(a.prog_pred[perm].view(np.uint32), b.prog_pred.view(np.uint32))


def test_ties_go_to_the_lowest_feature_then_the_lowest_cut(T):
    x = np.array([0, 1, 2, 3], np.float32)
    X = np.stack([x, x, x], axis=1)                                  # three identical columns
    y = np.array([1, -1, -1, 1], np.float32)                         # cuts 1 and 3 tie
    r = T.train(X, one_per_program(4), y, *all_cuts(X), n_rounds=1, max_depth=1, eta=1.0, lam=0.0)
    assert r.split_feature[0] == 0 and r.threshold[0] == np.float32(1.0)


def test_min_child_weight_and_min_gain_stop_splits(T):
    ts = W.make_train_set(17, 64, stmts=(1, 1), n_features=4, max_cuts=7)
    kw = dict(n_rounds=1, max_depth=3, eta=1.0, lam=0.0)
    r = T.train(ts.features, ts.prog_off, ts.target, ts.cut_off, ts.cuts, min_child_weight=33.0, **kw)
    assert r.split_feature.tolist() == [-1]                          # no child can hold 33 of 64 rows
    r = T.train(ts.features, ts.prog_off, ts.target, ts.cut_off, ts.cuts, min_gain=1e30, **kw)
    assert r.split_feature.tolist() == [-1]
    r = T.train(ts.features, ts.prog_off, ts.target, ts.cut_off, ts.cuts, min_child_weight=8.0, **kw)
    m = W.Model(4, r.tree_off, r.split_feature, r.threshold, r.left, r.right, r.value, 0.0)
    from oracle import oracle as O
    leaves = O.leaf_indices(m, ts.features)[:, 0]
    assert np.bincount(leaves).max() >= 8 and min(c for c in np.bincount(leaves) if c) >= 8


def test_root_split_weighs_rows_by_their_programs_length_hand_worked(T):
    """Multi-statement programs: the curvature of a row is the number of rows of its program,
    not 1.  Worked by hand (lambda = 0, s = 0 so g = -y on every row of the program):

        program   rows (x)   y    per row (g, h)
        0         1          1    (-1, 1)
        1         2, 1      -1    (+1, 2), (+1, 2)
        2         3         -2    (+2, 1)

    G = 3, H = 6.  Cut x < 2: left = {x=1 rows} GL = 0, HL = 3; right GR = 3, HR = 3:
    gain = 0 + 9/3 - 9/6 = 3/2.  Cut x < 3: GL = 1, HL = 5; GR = 2, HR = 1:
    gain = 1/5 + 4 - 3/2 = 27/10.  So the root splits at 3 with leaves -1/5 and -2.
    Counting rows instead of curvature (h = 1: H = 4) would give 9/4 for the cut at 2 and
    25/12 for the cut at 3 and so split at 2 with leaves 0 and -3/2."""
    X = np.array([[1], [2], [1], [3]], np.float32)
    off = np.array([0, 1, 3, 4], np.int32)
    y = np.array([1, -1, -2], np.float32)
    r = T.train(X, off, y, *all_cuts(X), n_rounds=1, max_depth=1, eta=1.0, lam=0.0)
    assert r.split_feature.tolist() == [0, -1, -1]
    assert r.threshold[0] == np.float32(3.0)
    assert r.value[1] == np.float32(float(Fraction(-1, 5))) and r.value[2] == np.float32(-2.0)
    # the two hand-worked gains really order the other way round under row counting
    assert Fraction(27, 10) > Fraction(3, 2) and Fraction(9, 4) > Fraction(25, 12)


def test_root_split_with_multi_statement_programs_minimises_the_weighted_objective(T):
    """As the single-statement pin above, with programs of 1..4 rows: every row of program p
    carries g = -y_p and curvature h = rows of p, and the objective of a leaf with weight w is
    sum_r (g_r w + h_r w^2 / 2) + lambda w^2 / 2, minimised numerically."""
    rng = np.random.default_rng(9)
    for trial in range(6):
        lens = rng.integers(1, 5, size=8)
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        n = int(off[-1])
        X = rng.integers(0, 5, size=(n, 2)).astype(np.float32)
        y = (rng.integers(-32, 32, 8) / 4.0).astype(np.float32)
        lam = float(rng.choice([0.0, 0.5, 2.0]))
        co, cuts = all_cuts(X)
        r = T.train(X, off, y, co, cuts, n_rounds=1, max_depth=1, eta=1.0, lam=lam, min_gain=-1e30)
        g = np.repeat(-y.astype(np.float64), lens)
        h = np.repeat(lens.astype(np.float64), lens)

        def best_obj(mask):
            gs, hs = g[mask], h[mask]
            f = lambda w: float(np.sum(gs * w + 0.5 * hs * w * w) + 0.5 * lam * w * w)
            return minimize_scalar(f, bounds=(-100, 100), method="bounded",
                                   options={"xatol": 1e-12}).fun

        parent = best_obj(np.ones(n, bool))
        best = (None, None, -np.inf)
        for f in range(2):
            for c in cuts[co[f]:co[f + 1]]:
                L = X[:, f] < c
                if L.sum() == 0 or (~L).sum() == 0:
                    continue
                drop = parent - best_obj(L) - best_obj(~L)
                if drop > best[2] + 1e-9:
                    best = (f, float(c), drop)
        assert r.split_feature[0] == best[0] and float(r.threshold[0]) == best[1]


def test_gradients_beyond_the_fixed_point_range_are_clamped_hand_worked(T):
    """Fixed-point gradients q = rint(g * 2^20) are clamped to +-2147483520 (= 2^31 - 128, the
    largest float below 2^31).  One row per program, a single leaf (depth 0), bias 0, so
    g = -y and H = number of programs.  Worked by hand:

      y = -4096:  g * 2^20 = 2^32 -> q = 2147483520; eta = 1, lambda = 1:
                  value = -(2147483520 / 2^20) / (1 + 1) = -(1024 - 2^-14)   (not -2048)
      y = +4096:  the mirror image, +(1024 - 2^-14)
      y = (-4096, -8192, 3), eta = 1/2, lambda = 1:  q = 2147483520, 2147483520, -3 * 2^20;
                  G / 2^20 = 2 * (2048 - 2^-13) - 3 = 4093 - 2^-12;
                  value = -(4093 - 2^-12) / 2 / (3 + 1) = -(511.625 - 2^-15)
    All three values are exact in float32."""
    X1 = np.zeros((1, 1), np.float32)
    for yv, exp in ((-4096.0, -(1024.0 - 2.0 ** -14)), (4096.0, 1024.0 - 2.0 ** -14)):
        r = T.train(X1, one_per_program(1), np.array([yv], np.float32), *all_cuts(X1), n_rounds=1,
                    max_depth=0, eta=1.0, lam=1.0)
        assert r.value.tolist() == [exp] and r.value.dtype == np.float32
    X3 = np.zeros((3, 1), np.float32)
    r = T.train(X3, one_per_program(3), np.array([-4096.0, -8192.0, 3.0], np.float32),
                *all_cuts(X3), n_rounds=1, max_depth=0, eta=0.5, lam=1.0)
    assert r.value.tolist() == [-(511.625 - 2.0 ** -15)]
    # just inside the range nothing is clamped: y = -2047 -> q = 2047 * 2^20, value = -2047 / 2
    r = T.train(X1, one_per_program(1), np.array([-2047.0], np.float32), *all_cuts(X1), n_rounds=1,
                max_depth=0, eta=1.0, lam=1.0)
    assert r.value.tolist() == [-1023.5]
