"""GPU training of family cost models against the training oracle: the trees (every array,
bit for bit) and the predictions on the training set, through the C ABI
(`fs_trainer_create`, `fs_train_boost`, `fs_trainer_export`, `fs_trainer_predictions`)."""
import numpy as np
import pytest

from paper_2201_00194_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2201_00194_amd import api as A
    return A


@pytest.fixture(scope="module")
def T():
    from oracle import train_oracle
    train_oracle.build()
    return train_oracle


def same_trees(got, exp):
    to, sf, th, le, ri, va = got
    assert np.array_equal(to, exp.tree_off)
    assert np.array_equal(sf, exp.split_feature)
    assert np.array_equal(le, exp.left) and np.array_equal(ri, exp.right)
    assert np.array_equal(th.view(np.uint32), exp.threshold.view(np.uint32))
    assert np.array_equal(va.view(np.uint32), exp.value.view(np.uint32))


def check(api, T, ts, rounds, layout=1, bias=0.0, **kw):
    import torch
    p = api.train_params(**kw)
    tr = api.fs_trainer.from_train_set(ts, layout=layout, bias=bias, max_depth=p.max_depth,
                                       max_trees=rounds)
    api.fs_train_boost([tr], rounds, p)
    torch.cuda.synchronize()
    exp = T.train(ts.features, ts.prog_off, ts.target, ts.cut_off, ts.cuts, bias=bias,
                  n_rounds=rounds, max_depth=p.max_depth, eta=p.eta, lam=p.lam, min_gain=p.min_gain,
                  min_child_weight=p.min_child_weight, grad_scale=p.grad_scale)
    same_trees(tr.export(), exp)
    rows, progs = tr.predictions()
    torch.cuda.synchronize()
    assert np.array_equal(rows.cpu().numpy().view(np.uint32), exp.row_pred.view(np.uint32))
    assert np.array_equal(progs.cpu().numpy().view(np.uint32), exp.prog_pred.view(np.uint32))
    return tr, exp


@pytest.mark.parametrize("layout", [0, 1])
def test_small_family_all_depths(api, T, layout):
    ts = W.make_train_set(21, 700, stmts=(1, 12), n_features=23, max_cuts=40)
    for depth in (0, 1, 3, 6):
        check(api, T, ts, rounds=4, layout=layout, max_depth=depth, eta=0.5, lam=1.0)


def test_full_width_features_255_cuts_depth8(api, T):
    ts = W.make_train_set(22, 1500, stmts=(1, 16), max_cuts=255)
    ts.features[17, 5] = np.nan
    ts.features[99, 0] = np.inf
    check(api, T, ts, rounds=3, max_depth=8, eta=0.3, lam=0.5, bias=0.25)


def test_deepest_trees(api, T):
    ts = W.make_train_set(24, 3000, stmts=(1, 6), n_features=12, max_cuts=255)
    tr, exp = check(api, T, ts, rounds=2, max_depth=api.FS_TRAIN_MAX_DEPTH, eta=0.5, lam=0.0)
    depth = 0                                    # the oracle's first tree really is that deep
    a, b = exp.tree_off[0], exp.tree_off[1]
    level = {0: 0}
    for n in range(b - a):
        if exp.split_feature[a + n] >= 0:
            level[int(exp.left[a + n])] = level[int(exp.right[a + n])] = level[n] + 1
            depth = max(depth, level[n] + 1)
    assert depth == api.FS_TRAIN_MAX_DEPTH
    check(api, T, ts, rounds=1, max_depth=9, eta=0.5, lam=1.0)


def test_regularisation_and_stopping_rules(api, T):
    ts = W.make_train_set(23, 400, stmts=(1, 5), n_features=9, max_cuts=15)
    check(api, T, ts, rounds=3, max_depth=4, eta=1.0, lam=0.0)
    check(api, T, ts, rounds=3, max_depth=4, eta=0.2, lam=10.0, min_child_weight=40.0)
    check(api, T, ts, rounds=2, max_depth=4, eta=0.2, lam=1.0, min_gain=5.0)
    check(api, T, ts, rounds=2, max_depth=3, eta=0.2, lam=1.0, grad_scale=float(1 << 10))


def test_families_spanning_several_row_slabs(api, T, tune):
    """Families with more rows than one histogram workgroup takes add their partial
    histograms into the global buffer and a separate kernel searches the cuts; forced here by
    shrinking the slab (a full slab is 65536 rows)."""
    tune(api.FS_TUNE_TRAIN_SLAB_ROWS, 1000)
    ts = W.make_train_set(27, 900, stmts=(1, 12), n_features=21, max_cuts=100)
    assert ts.n_rows > 4000
    check(api, T, ts, rounds=4, max_depth=6, eta=0.5, lam=1.0)
    tune(api.FS_TUNE_TRAIN_SLAB_ROWS, -1)
    check(api, T, ts, rounds=2, max_depth=6, eta=0.5, lam=1.0)


def test_family_larger_than_one_slab_at_its_natural_size(api, T):
    """The same path with nothing forced: a family of more than 65536 rows spans two slabs of its
    own accord (two workgroups per feature group add into the global histograms, the split
    kernel searches there)."""
    ts = W.make_train_set(29, 12_000, stmts=(4, 9), n_features=12, max_cuts=63)
    assert 65_536 < ts.n_rows < 131_072
    check(api, T, ts, rounds=2, max_depth=4, eta=0.3, lam=1.0)


def test_batched_families_train_independently(api, T):
    import torch
    sets = [W.make_train_set(30 + i, n, stmts=(1, 8), n_features=nf, max_cuts=mc)
            for i, (n, nf, mc) in enumerate([(300, 12, 20), (1200, 30, 63), (50, 5, 4), (2000, 12, 255)])]
    p = api.train_params(max_depth=5, eta=0.4, lam=1.0)
    trs = [api.fs_trainer.from_train_set(ts, max_depth=5, max_trees=8) for ts in sets]
    api.fs_train_boost(trs, 3, p)
    api.fs_train_boost(trs[:2], 2, p)                 # the first two get two more rounds
    torch.cuda.synchronize()
    for i, (ts, tr) in enumerate(zip(sets, trs)):
        exp = T.train(ts.features, ts.prog_off, ts.target, ts.cut_off, ts.cuts,
                      n_rounds=5 if i < 2 else 3, max_depth=5, eta=0.4, lam=1.0)
        same_trees(tr.export(), exp)
        assert tr.size()[0] == (5 if i < 2 else 3)


def test_trained_model_scores_identically_through_the_scoring_path(api, T, oracle):
    import torch
    ts = W.make_train_set(41, 900, stmts=(1, 10), n_features=40, max_cuts=31)
    tr, exp = check(api, T, ts, rounds=10, max_depth=5, eta=0.3, lam=1.0, bias=0.5)
    to, sf, th, le, ri, va = tr.export()
    host = W.Model(40, to, sf, th, le, ri, va, 0.5)
    fam = W.Family(host, ts.features, ts.prog_off, 16)
    dev = api.DeviceFamily(fam, want_row_score=True)
    api.fs_score_families([dev.family()])
    torch.cuda.synchronize()
    rows, progs = tr.predictions()
    assert torch.equal(dev.row_score[: ts.n_rows], rows)
    assert torch.equal(dev.prog_score[: ts.n_programs], progs)
    assert exp.loss[-1] < 0.5 * exp.loss[0]


def test_errors(api):
    import torch
    ts = W.make_train_set(51, 40, stmts=(1, 3), n_features=4, max_cuts=7)
    tr = api.fs_trainer.from_train_set(ts, max_depth=3, max_trees=2)
    with pytest.raises(api.FsError):
        api.fs_train_boost([tr], 1, api.train_params(max_depth=4))          # deeper than created for
    with pytest.raises(api.FsError):
        api.fs_train_boost([tr], 3, api.train_params(max_depth=3))          # more trees than room
    with pytest.raises(api.FsError):
        api.fs_train_boost([tr], 1, api.train_params(max_depth=3, grad_scale=3.0))
    with pytest.raises(api.FsError):
        api.fs_train_boost([tr, tr], 1, api.train_params(max_depth=3))
    bad = W.make_train_set(52, 40, stmts=(1, 3), n_features=4, max_cuts=7)
    bad.cuts = bad.cuts[::-1].copy()
    with pytest.raises(api.FsError):
        api.fs_trainer.from_train_set(bad, max_depth=3, max_trees=2)
    api.fs_train_boost([tr], 2, api.train_params(max_depth=3))              # still works
    torch.cuda.synchronize()
    assert tr.size()[0] == 2


@pytest.mark.parametrize("seed", range(30))
def test_random_training_shapes_and_parameters(api, T, tune, seed):
    rng = np.random.default_rng([seed, 777])
    if seed >= 10:                # the later seeds also vary the histogram form and the row slabs
        tune(api.FS_TUNE_TRAIN_SLAB_ROWS, int(rng.choice([-1, 512, 3000])))
        tune(api.FS_TUNE_TRAIN_PACKED, int(rng.choice([-1, 0])))
        tune(api.FS_TUNE_TRAIN_SORT, int(rng.choice([-1, 0, 1])))
    nf = int(rng.choice([1, 2, 3, 5, 17, 33, 64]))
    ts = W.make_train_set(100 + seed, int(rng.integers(2, 1500)), stmts=(1, int(rng.integers(1, 30))),
                          n_features=nf, max_cuts=int(rng.choice([1, 2, 7, 64, 255])),
                          zero_frac=float(rng.choice([0.0, 0.3, 0.95])))
    check(api, T, ts, rounds=int(rng.integers(1, 6)), layout=int(rng.integers(0, 2)),
          bias=float(rng.choice([0.0, 1.5])), max_depth=int(rng.integers(0, 11)),
          eta=float(rng.choice([0.1, 0.5, 1.0])), lam=float(rng.choice([0.0, 1.0, 7.5])),
          min_child_weight=float(rng.choice([0.0, 1.0, 20.0])),
          min_gain=float(rng.choice([0.0, 0.0, 0.01])))


def test_one_very_long_program_does_not_overflow_the_curvature_sums(api, T):
    """Curvature of a row = rows of its program, so one program of 66 000 rows puts
    66 000 x 66 000 > 2^32 into a single histogram bin; also more rows than one slab."""
    rng = np.random.default_rng(5)
    lens = np.concatenate([[66_000], rng.integers(1, 9, 60)]).astype(np.int64)
    off = np.zeros(lens.shape[0] + 1, np.int64)
    np.cumsum(lens, out=off[1:])
    X = W.draw_features(rng, int(off[-1]), 0.5, n_features=4)
    y = rng.standard_normal(lens.shape[0]).astype(np.float32)
    cut_off, cuts = W.draw_cuts(X, 7)
    ts = W.TrainSet(X, off.astype(np.int32), y, cut_off, cuts)
    check(api, T, ts, rounds=2, max_depth=2, eta=0.5, lam=1.0)


def test_many_tied_and_near_tied_cuts(api, T):
    """Small integer features in duplicated columns and coarse targets make many cuts tie
    exactly or differ in the last bits: the choice must still be the oracle's first largest."""
    rng = np.random.default_rng(8)
    base = rng.integers(0, 6, size=(600, 3)).astype(np.float32)
    X = np.concatenate([base, base, base[:, ::-1]], axis=1)          # 9 columns, 3 distinct twice
    off = np.arange(601, dtype=np.int32)
    y = rng.integers(-2, 3, 600).astype(np.float32)
    cut_off, cuts = W.draw_cuts(X, 255)
    ts = W.TrainSet(X, off, y, cut_off, cuts)
    check(api, T, ts, rounds=6, max_depth=6, eta=1.0, lam=0.0)
    check(api, T, ts, rounds=3, max_depth=5, eta=0.3, lam=2.0, grad_scale=float(1 << 4))
    big = W.TrainSet(X * np.float32(3e4), off, (y * np.float32(1000)).astype(np.float32),
                     *W.draw_cuts(X * np.float32(3e4), 255))
    check(api, T, big, rounds=3, max_depth=4, eta=0.5, lam=0.0, grad_scale=float(1 << 20))


def test_histogram_forms_packed_wide_and_fallback(api, T, tune):
    """The histogram kernel keeps (G, H) of a bin packed in one 64-bit word while the round's
    gradients leave room for it, and falls back inside the kernel to separate 64-bit sums when
    they do not; the override FS_TUNE_TRAIN_PACKED = 0 launches the separate sums outright.  All three must
    give the oracle's trees.  Huge targets make the fixed-point gradients hit their clamp
    (+-2^31), so that their sum over the rows passes what the packed form can hold."""
    ts = W.make_train_set(41, 2500, stmts=(1, 40), n_features=30, max_cuts=120)
    assert 40_000 < ts.n_rows <= 65_536
    kw = dict(rounds=3, max_depth=6, eta=0.5, lam=1.0)
    check(api, T, ts, **kw)                                          # packed
    tune(api.FS_TUNE_TRAIN_PACKED, 0)
    check(api, T, ts, **kw)                                          # wide
    tune(api.FS_TUNE_TRAIN_PACKED, -1)
    huge = W.TrainSet(ts.features, ts.prog_off, (ts.target * np.float32(1e7)).astype(np.float32),
                      ts.cut_off, ts.cuts)
    # the packed form has 63 - 21 bits for gradient sums here (rows x longest program < 2^21);
    # the clamped gradients add up to about rows x 2^31
    assert np.sum(np.abs(huge.target) > 4096) > 0.9 * huge.target.shape[0]
    assert 0.9 * huge.n_rows * float(1 << 31) > 2.0 ** 44
    check(api, T, huge, rounds=2, max_depth=5, eta=0.5, lam=1.0)      # fallback in the first round
    check(api, T, huge, rounds=2, max_depth=0, eta=0.5, lam=1.0)
    tune(api.FS_TUNE_TRAIN_SLAB_ROWS, 20000)
    check(api, T, ts, **kw)                                          # packed, several slabs
    check(api, T, huge, rounds=2, max_depth=5, eta=0.5, lam=1.0)      # fallback, several slabs
    tune(api.FS_TUNE_TRAIN_SLAB_ROWS, -1)


def test_rows_regrouped_by_node_for_deep_trees(api, T, tune):
    """From depth 7 on the rows are regrouped once per tree by their node of level 5 and the
    deeper histograms read only their ancestors' segments; the trees must not change.  Forced on
    at depth 6, forced off at depth 9, and run with early leaves above level 5 (rows that stay
    behind) and with several families of different sizes in one batch."""
    import torch
    ts = W.make_train_set(43, 3000, stmts=(1, 9), n_features=17, max_cuts=200)
    tune(api.FS_TUNE_TRAIN_SORT, 1)
    check(api, T, ts, rounds=3, max_depth=6, eta=0.5, lam=1.0)
    check(api, T, ts, rounds=2, max_depth=9, eta=0.5, lam=0.0, min_child_weight=40.0)   # leaves above level 5
    tune(api.FS_TUNE_TRAIN_PACKED, 0)
    check(api, T, ts, rounds=2, max_depth=8, eta=0.5, lam=1.0)                          # 8 nodes per pass
    tune(api.FS_TUNE_TRAIN_PACKED, -1)
    tune(api.FS_TUNE_TRAIN_SORT, 0)
    check(api, T, ts, rounds=2, max_depth=9, eta=0.5, lam=1.0)
    tune(api.FS_TUNE_TRAIN_SORT, -1)
    sets = [W.make_train_set(50 + i, n, stmts=(1, 6), n_features=9, max_cuts=60) for i, n in enumerate((400, 2500, 60))]
    p = api.train_params(max_depth=8, eta=0.4, lam=1.0)
    trs = [api.fs_trainer.from_train_set(s, max_depth=8, max_trees=3) for s in sets]
    api.fs_train_boost(trs, 3, p)
    torch.cuda.synchronize()
    for s, tr in zip(sets, trs):
        exp = T.train(s.features, s.prog_off, s.target, s.cut_off, s.cuts, bias=0.0, n_rounds=3, max_depth=8,
                      eta=p.eta, lam=p.lam, min_gain=p.min_gain, min_child_weight=p.min_child_weight,
                      grad_scale=p.grad_scale)
        same_trees(tr.export(), exp)
        rows, progs = tr.predictions()
        torch.cuda.synchronize()
        assert np.array_equal(rows.cpu().numpy().view(np.uint32), exp.row_pred.view(np.uint32))


def test_family_of_the_benchmark_workloads_own_size(api, T):
    """One family of the workload `bench.py --train` times, at its own size: the largest of the
    eight (164 features, 255 cuts, tens of thousands of rows in one histogram slab), two rounds
    at the benchmark's depth and parameters."""
    sets = W.make_train_case(seed=0)
    ts = max(sets, key=lambda s: s.n_rows)
    assert ts.features.shape[1] == 164 and 30_000 < ts.n_rows <= 65_536
    check(api, T, ts, rounds=2, max_depth=6, eta=0.2, lam=1.0)
