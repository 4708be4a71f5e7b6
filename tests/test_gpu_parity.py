"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI.

Bar: leaf indices and top-k indices bit-exact; fp32 scores within 1e-5 relative /
1e-6 absolute.  The library reproduces the oracle's order of additions, so scores are in
fact expected to be bit-identical and the tests also assert that.
"""
import numpy as np
import pytest

from paper_2201_00194_amd import workloads as W

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-5, 1e-6


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2201_00194_amd import api as A
    return A


def run_families(api, fams, layout, want_rows=True, want_leaves=True):
    import torch
    devs = [api.DeviceFamily(f, layout=layout, want_row_score=want_rows, want_leaf_idx=want_leaves)
            for f in fams]
    api.fs_score_families([d.family() for d in devs])
    api.fs_topk([d.topk_request() for d in devs])
    torch.cuda.synchronize()
    return devs


def check_family(oracle, fam, dev, check_leaves=True, check_rows=True):
    m = fam.model
    rs = oracle.row_scores(m, fam.features)
    ps = oracle.program_scores(rs, fam.prog_off)
    if check_leaves and dev.leaf_idx is not None and fam.n_rows * m.n_trees > 0:
        li = oracle.leaf_indices(m, fam.features)
        got = dev.leaf_idx.cpu().numpy().view(np.uint16)[: fam.n_rows * m.n_trees]
        assert np.array_equal(got.reshape(fam.n_rows, m.n_trees).astype(np.int32), li)
    if check_rows and dev.row_score is not None and fam.n_rows > 0:
        got = dev.row_score.cpu().numpy()[: fam.n_rows]
        np.testing.assert_allclose(got, rs, rtol=RTOL, atol=ATOL)
        assert np.array_equal(got.view(np.uint32), rs.view(np.uint32))
    if fam.n_programs > 0:
        got = dev.prog_score.cpu().numpy()[: fam.n_programs]
        np.testing.assert_allclose(got, ps, rtol=RTOL, atol=ATOL)
        assert np.array_equal(got.view(np.uint32), ps.view(np.uint32))
    if fam.k > 0:
        idx, val = oracle.topk(ps, fam.k)
        gi = dev.topk_idx.cpu().numpy()[: fam.k]
        gv = dev.topk_score.cpu().numpy()[: fam.k]
        assert np.array_equal(gi, idx)
        assert np.array_equal(gv.view(np.uint32), val.view(np.uint32))
        # decoupled check: the oracle's cut applied to the device's own scores
        if fam.n_programs > 0:
            own = dev.prog_score.cpu().numpy()[: fam.n_programs]
            idx2, _ = oracle.topk(own, fam.k)
            assert np.array_equal(gi, idx2)


LAYOUTS = [0, 1]


@pytest.mark.parametrize("layout", LAYOUTS)
def test_cfg0_full_size(api, oracle, layout):
    case = W.make_case(0, seed=0)
    devs = run_families(api, case.families, layout)
    for f, d in zip(case.families, devs):
        check_family(oracle, f, d)


@pytest.mark.parametrize("cfg,scale,trees", [(1, 0.05, 60), (2, 0.004, 40), (3, 0.02, 50),
                                              (4, 0.03, 40)])
def test_scaled_configs_all_outputs(api, oracle, cfg, scale, trees):
    case = W.make_case(cfg, seed=1, scale=scale, trees=trees)
    devs = run_families(api, case.families, api.FS_COLBLOCK64)
    for f, d in zip(case.families, devs):
        check_family(oracle, f, d)


def test_scaled_configs_rowmajor(api, oracle):
    case = W.make_case(3, seed=2, scale=0.01, trees=30)
    devs = run_families(api, case.families, api.FS_ROWMAJOR)
    for f, d in zip(case.families, devs):
        check_family(oracle, f, d)


def test_ragged_tails_and_tiny_shapes(api, oracle):
    fams = []
    for i, (P, stm, T, dep, q) in enumerate([(1, (1, 1), 1, 0, 0.0), (3, (1, 1), 2, 1, 0.0),
                                              (65, (1, 3), 7, 3, 0.3), (130, (0, 5), 9, 5, 0.2),
                                              (257, (63, 64), 3, 2, 0.0), (64, (1, 1), 33, 4, 0.0),
                                              (1000, (0, 2), 5, 12, 0.3)]):
        fams.append(W.make_small_family(seed=100 + i, n_programs=P, stmts=stm, n_trees=T, depth=dep,
                                        early_leaf_q=q, k=[1, 5, 64, 200, 17, 64, 1000][i],
                                        bias=[0.0, 0.5, -1.25, 3.0, 0.0, 1e-3, 0.0][i]))
    for layout in LAYOUTS:
        devs = run_families(api, fams, layout)
        for f, d in zip(fams, devs):
            check_family(oracle, f, d)


def test_empty_families_zero_trees_and_k_edges(api, oracle):
    import torch
    empty = W.make_small_family(seed=7, n_programs=0, stmts=(1, 1), n_trees=3, depth=2, k=4)
    assert empty.n_rows == 0 and empty.n_programs == 0
    no_rows = W.make_small_family(seed=8, n_programs=5, stmts=(0, 0), n_trees=3, depth=2, k=3)
    assert no_rows.n_rows == 0 and no_rows.n_programs == 5
    no_trees = W.make_small_family(seed=9, n_programs=20, stmts=(1, 4), n_trees=0, depth=0, k=50,
                                   bias=0.75)
    k0 = W.make_small_family(seed=10, n_programs=20, stmts=(2, 2), n_trees=4, depth=3, k=0)
    fams = [empty, no_rows, no_trees, k0]
    devs = run_families(api, fams, api.FS_COLBLOCK64)
    for f, d in zip(fams, devs):
        check_family(oracle, f, d)
    # empty family: k entries of (-1, -inf)
    assert np.array_equal(devs[0].topk_idx.cpu().numpy(), [-1] * 4)
    assert np.all(np.isneginf(devs[0].topk_score.cpu().numpy()))
    # programs without rows score +0 and rank by index
    assert np.array_equal(devs[1].topk_idx.cpu().numpy(), [0, 1, 2])
    # k = 0 leaves the output buffer untouched
    assert devs[3].topk_idx.cpu().numpy()[0] == -7


def test_special_values_in_features_and_thresholds(api, oracle):
    fam = W.make_small_family(seed=21, n_programs=300, stmts=(1, 6), n_trees=40, depth=6,
                              early_leaf_q=0.1, k=32)
    X = fam.features
    rng = np.random.default_rng(3)
    for val in (np.nan, np.inf, -np.inf, -0.0, 1e-42, -1e-42):
        r = rng.integers(0, X.shape[0], 200)
        c = rng.integers(0, X.shape[1], 200)
        X[r, c] = val
    internal = np.flatnonzero(fam.model.split_feature >= 0)
    pick = rng.choice(internal, 40, replace=False)
    fam.model.threshold[pick[:10]] = np.inf
    fam.model.threshold[pick[10:20]] = -0.0
    fam.model.threshold[pick[20:30]] = np.nan
    fam.model.threshold[pick[30:]] = 1e-42
    for layout in LAYOUTS:
        devs = run_families(api, [fam], layout)
        check_family(oracle, fam, devs[0])


def test_topk_standalone_ties_signed_zero_nan(api, oracle):
    import torch
    rng = np.random.default_rng(5)
    cases = []
    s = rng.standard_normal(5000).astype(np.float32)
    s[rng.integers(0, 5000, 2500)] = s[rng.integers(0, 5000, 2500)]
    cases.append((s, 100))
    cases.append((s, 5000))
    cases.append((s, 6000))
    cases.append((np.full(3000, 1.5, np.float32), 77))
    z = np.zeros(2000, np.float32)
    z[::3] = -0.0
    z[5::7] = np.nan
    z[1::11] = -np.inf
    z[2::13] = np.inf
    cases.append((z, 1500))
    cases.append((z, 2000))
    cases.append((np.array([3.0], np.float32), 1))
    cases.append((rng.standard_normal(70000).astype(np.float32), 16384))
    q = (rng.integers(-8, 8, 100000) / 4.0).astype(np.float32)       # few distinct values
    cases.append((q, 1024))
    reqs, outs = [], []
    for sc, k in cases:
        t = torch.from_numpy(sc).cuda()
        oi = torch.full((k,), -7, dtype=torch.int32, device="cuda")
        ov = torch.full((k,), float("nan"), dtype=torch.float32, device="cuda")
        reqs.append(api.TopkRequest(t, sc.shape[0], k, oi, ov))
        outs.append((oi, ov))
    api.fs_topk(reqs)
    torch.cuda.synchronize()
    for (sc, k), (oi, ov) in zip(cases, outs):
        idx, val = oracle.topk(sc, k)
        assert np.array_equal(oi.cpu().numpy(), idx)
        assert np.array_equal(ov.cpu().numpy().view(np.uint32), val.view(np.uint32))
    # out_score may be NULL
    sc, k = cases[0]
    oi = torch.full((k,), -7, dtype=torch.int32, device="cuda")
    api.fs_topk([api.TopkRequest(reqs[0].score, sc.shape[0], k, oi, None)])
    torch.cuda.synchronize()
    assert np.array_equal(oi.cpu().numpy(), oracle.topk(sc, k)[0])


def test_topk_long_requests_are_sliced_and_merged(api, oracle):
    """Requests of 8192 entries or more take several workgroups plus a merge; mixed in one
    submission with short ones.  Ties, NaN and constant scores must still come out in the
    oracle's order (Section 3.2: sort by estimate, keep the top k)."""
    import torch
    rng = np.random.default_rng(11)
    cases = []
    cases.append((rng.standard_normal(32768).astype(np.float32), 64))
    cases.append((rng.standard_normal(40001).astype(np.float32), 5000))      # 3 ragged slices
    cases.append((np.full(50000, -2.25, np.float32), 3000))                  # all tie: lowest indices
    q = (rng.integers(-3, 3, 262144) / 2.0).astype(np.float32)
    q[rng.integers(0, 262144, 1000)] = np.nan
    q[rng.integers(0, 262144, 1000)] = -0.0
    cases.append((q, 1024))
    cases.append((rng.standard_normal(1000).astype(np.float32), 10))         # short, same launch
    cases.append((rng.standard_normal(8192).astype(np.float32), 64))         # 4 slices
    cases.append((rng.standard_normal(9000).astype(np.float32), 3000))       # 4 slices, k above a slice's length
    step = np.zeros(65536, np.float32)
    step[60000:] = 1.0                                                       # best entries all in the last slice
    cases.append((step, 8192))
    cases.append((rng.standard_normal(33000).astype(np.float32), 16384))     # k too large to slice
    cases.append((rng.standard_normal(100000).astype(np.float32), 1))
    nanall = np.full(40000, np.nan, np.float32)
    cases.append((nanall, 100))
    reqs, outs = [], []
    for sc, k in cases:
        t = torch.from_numpy(sc).cuda()
        oi = torch.full((k,), -7, dtype=torch.int32, device="cuda")
        ov = torch.full((k,), float("nan"), dtype=torch.float32, device="cuda")
        reqs.append(api.TopkRequest(t, sc.shape[0], k, oi, ov))
        outs.append((oi, ov))
    for _ in range(2):      # the second call reuses the candidate scratch
        api.fs_topk(reqs)
        torch.cuda.synchronize()
        for (sc, k), (oi, ov) in zip(cases, outs):
            idx, val = oracle.topk(sc, k)
            assert np.array_equal(oi.cpu().numpy(), idx)
            assert np.array_equal(ov.cpu().numpy().view(np.uint32), val.view(np.uint32))


def test_topk_wide_cuts_merge_in_global_memory(api, oracle):
    """Cuts above 4096 of long requests: slices sorted per workgroup, then pairwise merges level
    by level.  Odd slice counts, a last slice shorter than the others, k above the request's
    length, ties that straddle slices, NaN and signed zeros; mixed with other kinds of request
    in one submission and repeated so that the scratch is reused."""
    import torch
    rng = np.random.default_rng(23)
    cases = []
    cases.append((rng.standard_normal(65536).astype(np.float32), 16384))     # 32 slices, 5 levels
    cases.append((rng.standard_normal(8192).astype(np.float32), 4097))       # 4 slices
    cases.append((rng.standard_normal(8193).astype(np.float32), 4097))       # 5 slices, the last one shorter
    cases.append((rng.standard_normal(24577).astype(np.float32), 5000))      # 13 slices, ragged
    cases.append((rng.standard_normal(20000).astype(np.float32), 16384))     # 10 slices: odd counts carry one list up
    cases.append((rng.standard_normal(12000).astype(np.float32), 16000))     # k above n: -1 padding
    cases.append((np.full(70000, 0.5, np.float32), 9000))                    # all tie: lowest indices
    q = (rng.integers(-2, 3, 300000) / 2.0).astype(np.float32)               # 5 values, 128 slices (the cap)
    q[rng.integers(0, 300000, 3000)] = np.nan
    q[rng.integers(0, 300000, 3000)] = -0.0
    cases.append((q, 12345))
    step = np.zeros(100000, np.float32)
    step[93000:] = 2.0                                                       # best entries in the last slices
    cases.append((step, 8000))
    cases.append((rng.standard_normal(700000).astype(np.float32), 16384))    # 128 slices of 5504 (cap)
    cases.append((rng.standard_normal(3_000_000).astype(np.float32), 16384))  # slices longer than the cut
    cases.append((np.full(9000, np.nan, np.float32), 6000))
    cases.append((rng.standard_normal(30000).astype(np.float32), 100))       # LDS merge, same launch
    cases.append((rng.standard_normal(500).astype(np.float32), 20))          # short, same launch
    reqs, outs = [], []
    for sc, k in cases:
        t = torch.from_numpy(sc).cuda()
        oi = torch.full((k,), -7, dtype=torch.int32, device="cuda")
        ov = torch.full((k,), float("nan"), dtype=torch.float32, device="cuda")
        reqs.append(api.TopkRequest(t, sc.shape[0], k, oi, ov))
        outs.append((oi, ov))
    for _ in range(2):
        api.fs_topk(reqs)
        torch.cuda.synchronize()
        for (sc, k), (oi, ov) in zip(cases, outs):
            idx, val = oracle.topk(sc, k)
            assert np.array_equal(oi.cpu().numpy(), idx), (sc.shape[0], k)
            assert np.array_equal(ov.cpu().numpy().view(np.uint32), val.view(np.uint32)), (sc.shape[0], k)
        for oi, ov in outs:
            oi.fill_(-7)
            ov.fill_(float("nan"))
    # out_score may be NULL on this path too
    sc, k = cases[0]
    oi = torch.full((k,), -7, dtype=torch.int32, device="cuda")
    api.fs_topk([api.TopkRequest(reqs[0].score, sc.shape[0], k, oi, None)])
    torch.cuda.synchronize()
    assert np.array_equal(oi.cpu().numpy(), oracle.topk(sc, k)[0])


def test_repeat_calls_are_bit_identical_and_scratch_row_scores_work(api, oracle):
    import torch
    case = W.make_case(3, seed=4, scale=0.01, trees=25)
    devs = [api.DeviceFamily(f, layout=api.FS_COLBLOCK64) for f in case.families]  # no row_score
    prepared = api.PreparedFamilies([d.family() for d in devs])
    api.fs_score_families(prepared)
    torch.cuda.synchronize()
    first = [d.prog_score.clone() for d in devs]
    for d in devs:
        d.prog_score.fill_(float("nan"))
    api.fs_score_families(prepared)
    api.fs_topk([d.topk_request() for d in devs])
    torch.cuda.synchronize()
    for f, d, a in zip(case.families, devs, first):
        assert torch.equal(d.prog_score.view(torch.int32), a.view(torch.int32))
        check_family(oracle, f, d)


def test_pack_colblock64_layout(api):
    import torch
    for R, D in ((1, 164), (64, 164), (200, 164), (130, 7), (70, 300)):
        x = torch.arange(R * D, dtype=torch.float32, device="cuda").reshape(R, D)
        out = api.fs_pack_colblock64(x, R, D)
        torch.cuda.synchronize()
        tiles = (R + 63) // 64
        o = out.cpu().numpy().reshape(tiles, D, 64)
        xp = np.zeros((tiles * 64, D), np.float32)
        xp[:R] = x.cpu().numpy()
        assert np.array_equal(o, xp.reshape(tiles, 64, D).transpose(0, 2, 1))


def test_errors_are_reported_not_raised_as_faults(api):
    import torch
    fam = W.make_small_family(seed=31, n_programs=10, stmts=(2, 2), n_trees=2, depth=2, k=4)
    d = api.DeviceFamily(fam)
    bad = d.family()
    bad.layout = 9
    with pytest.raises(api.FsError) as e:
        api.fs_score_families([bad])
    assert e.value.code == api.FS_EINVAL and "layout" in str(e.value)
    bad = d.family()
    bad.prog_score = None
    with pytest.raises(api.FsError):
        api.fs_score_families([bad])
    bad = d.family()
    bad.features = None
    with pytest.raises(api.FsError):
        api.fs_score_families([bad])
    with pytest.raises(api.FsError) as e:
        api.fs_topk([api.TopkRequest(d.prog_score, 10, api.FS_MAX_TOPK + 1, d.topk_idx, None)])
    assert e.value.code == api.FS_EUNSUPPORTED
    with pytest.raises(api.FsError):
        api.fs_topk([api.TopkRequest(d.prog_score, -1, 2, d.topk_idx, None)])
    # the library still works afterwards
    api.fs_score_families([d.family()])
    torch.cuda.synchronize()


def test_rank_coded_path_special_values_and_shallow_trees(api, oracle, tune):
    """Deep perfect-tree models are walked over 16-bit ranks of the features among the model's
    own thresholds; the leaves must be the same as over the fp32 values, also for NaN, inf,
    signed zeros and denormals in features and thresholds.  Forced here for shallow trees too."""
    tune(api.FS_TUNE_RANK, 1)
    fams = []
    for i, (P, stm, T, dep, k) in enumerate([(700, (1, 5), 60, 10, 100), (300, (2, 2), 25, 9, 40),
                                              (500, (1, 9), 70, 6, 64), (90, (3, 3), 10, 1, 8),
                                              (65, (1, 2), 33, 11, 70)]):
        fam = W.make_small_family(seed=200 + i, n_programs=P, stmts=stm, n_trees=T, depth=dep, k=k,
                                  bias=[0.0, 0.25, -1.0, 0.0, 2.0][i])
        rng = np.random.default_rng(300 + i)
        X = fam.features
        for val in (np.nan, np.inf, -np.inf, -0.0, 1e-42, -1e-42, -0.5):
            r = rng.integers(0, X.shape[0], 150)
            c = rng.integers(0, X.shape[1], 150)
            X[r, c] = val
        internal = np.flatnonzero(fam.model.split_feature >= 0)
        pick = rng.choice(internal, min(40, internal.shape[0]), replace=False)
        q = max(1, pick.shape[0] // 5)
        fam.model.threshold[pick[:q]] = np.inf
        fam.model.threshold[pick[q:2 * q]] = -0.0
        fam.model.threshold[pick[2 * q:3 * q]] = np.nan
        fam.model.threshold[pick[3 * q:4 * q]] = 1e-42
        fam.model.threshold[pick[4 * q:]] = -np.inf
        fams.append(fam)
    devs = run_families(api, fams, api.FS_COLBLOCK64)
    for f, d in zip(fams, devs):
        check_family(oracle, f, d)
    # same families without the optional outputs (the timed configuration)
    devs = run_families(api, fams, api.FS_COLBLOCK64, want_rows=False, want_leaves=False)
    for f, d in zip(fams, devs):
        check_family(oracle, f, d)


def test_trees_of_mixed_depth_walked_in_runs_of_their_own_depth(api, oracle):
    """The LDS kernel walks a chunk's trees in runs, each to the depth of its deepest tree; with
    many shallow trees the runs are formed by depth and dealt to the wavefronts by cost, with
    few they stay in tree order.  Leaf ids, row scores and the sums (in tree order whatever the
    walk order) must not notice: ensembles that mix stumps, single leaves and deep trees, a
    chunk with more trees than one round of runs holds, and a model of single leaves only."""
    def mixed(seed, n_trees, depths, n_features=164):
        fam = W.make_small_family(seed=seed, n_programs=260, stmts=(1, 5), n_trees=n_trees, depth=1,
                                  n_features=n_features, k=32, bias=0.125)
        rng = np.random.default_rng(seed)
        parts = [W.draw_model(rng, fam.features, 1, int(d), early_leaf_q=0.25 if d > 1 else 0.0)
                 for d in rng.choice(depths, size=n_trees)]
        off = np.concatenate([[0], np.cumsum([p.n_nodes for p in parts])]).astype(np.int32)
        cat = lambda name: np.concatenate([getattr(p, name) for p in parts])
        fam.model = W.Model(n_features, off, cat("split_feature"), cat("threshold"), cat("left"),
                            cat("right"), cat("value"), 0.125)
        return fam
    fams = [mixed(701, 90, [0, 1, 1, 2, 9]),          # mostly shallow: runs formed by depth
            mixed(702, 70, [7, 8, 8, 8, 8, 8, 1]),    # mostly deep: runs in tree order
            mixed(703, 200, [1, 2, 3], 40),           # many small trees per chunk: several runs per wavefront
            mixed(704, 30, [0])]                      # single leaves only
    for layout in LAYOUTS:
        devs = run_families(api, fams, layout)
        for f, d in zip(fams, devs):
            check_family(oracle, f, d)
    devs = run_families(api, fams, api.FS_COLBLOCK64, want_rows=False, want_leaves=False)
    for f, d in zip(fams, devs):
        check_family(oracle, f, d)


@pytest.mark.parametrize("groups", [2, 3, 4, 16])
def test_workgroups_that_take_several_tile_groups(api, oracle, tune, groups):
    """In a long launch a workgroup of the LDS kernel walks several consecutive groups of tiles
    and receives all but the first through registers while it is still walking.  Forced here on
    small inputs: group counts that the workgroups do not divide evenly, a last group with a
    single tile and a ragged last tile, one-chunk and many-chunk models, a family shorter than
    one workgroup's share, leaf ids on and off, and row-major input beside it (one group per
    workgroup there).  Every output must equal the oracle's, as with one group per workgroup."""
    tune(api.FS_TUNE_LDS_GROUPS, groups)
    fams = [W.make_small_family(seed=811, n_programs=700, stmts=(1, 7), n_trees=24, depth=4,
                                early_leaf_q=0.3, k=40, bias=-0.25),       # one chunk
            W.make_small_family(seed=812, n_programs=523, stmts=(2, 6), n_trees=150, depth=6,
                                early_leaf_q=0.25, k=64),                   # several chunks
            W.make_small_family(seed=813, n_programs=40, stmts=(1, 4), n_trees=150, depth=6,
                                early_leaf_q=0.25, k=8),                    # fewer groups than a share
            W.make_small_family(seed=814, n_programs=301, stmts=(3, 3), n_trees=9, depth=2, k=301)]
    assert any(((f.n_rows + 63) // 64) % 2 == 1 for f in fams)     # a last group of one tile
    for layout in LAYOUTS:
        devs = run_families(api, fams, layout)
        for f, d in zip(fams, devs):
            check_family(oracle, f, d)
    devs = run_families(api, fams, api.FS_COLBLOCK64, want_rows=False, want_leaves=False)
    for f, d in zip(fams, devs):
        check_family(oracle, f, d)
    case = W.make_case(3, seed=2, scale=0.02, trees=50)
    devs = run_families(api, case.families, api.FS_COLBLOCK64, want_leaves=False)
    for f, d in zip(case.families, devs):
        check_family(oracle, f, d, check_leaves=False)
    # both layouts in one call: the workgroups of the row-major families take one group each,
    # the others several, and the workgroup counts of the launch have to add up
    import torch
    devs = [api.DeviceFamily(f, layout=i % 2, want_row_score=True, want_leaf_idx=i % 3 == 0)
            for i, f in enumerate(fams)]
    api.fs_score_families([d.family() for d in devs])
    api.fs_topk([d.topk_request() for d in devs])
    torch.cuda.synchronize()
    for f, d in zip(fams, devs):
        check_family(oracle, f, d)


def test_models_outside_the_lds_formats_take_the_global_kernel(api, oracle):
    """More than 255 features, or trees too large for an LDS chunk: walked from global memory,
    in either layout."""
    wide = W.make_small_family(seed=401, n_programs=150, stmts=(1, 6), n_trees=12, depth=5,
                               early_leaf_q=0.2, n_features=300, k=20)
    deep = W.make_small_family(seed=402, n_programs=90, stmts=(2, 3), n_trees=3, depth=13, k=10)
    for layout in LAYOUTS:
        devs = run_families(api, [wide, deep], layout)
        for f, d in zip([wide, deep], devs):
            check_family(oracle, f, d)
    api.fs_profile_begin(16)
    run_families(api, [wide, deep], api.FS_COLBLOCK64)
    prof = api.fs_profile_end()
    assert prof["traverse_global"][1] >= 1 and prof["traverse"][1] == 0


def test_rowmajor_input_goes_straight_into_the_fast_kernels(api, oracle):
    case = W.make_case(1, seed=5, scale=0.02, trees=30)       # perfect depth-8 trees: rank path
    irregular = W.make_case(4, seed=5, scale=0.02, trees=20)  # 8-byte-node LDS path
    fams = case.families[:3] + irregular.families[:3]
    api.fs_profile_begin(32)
    devs = run_families(api, fams, api.FS_ROWMAJOR)
    prof = api.fs_profile_end()
    for f, d in zip(fams, devs):
        check_family(oracle, f, d)
    # the rank-coding kernel and the LDS kernel read the row-major matrices themselves
    assert prof["pack"][1] == 0 and prof["traverse_global"][1] == 0
    assert prof["traverse"][1] == 1 and prof["traverse_rank"][1] == 1


def test_rowmajor_input_transposed_inside_the_lds_kernel(api, oracle):
    """Row-major families whose model takes an LDS kernel and whose feature count is a multiple
    of four are read as they are (no re-tiling pass): ragged last tile, a one-row family, special
    values, 164 and 64 features (two and three tiles per workgroup).  A 30-feature family in the
    same call still goes through the re-tiling pass."""
    import torch
    fams = [W.make_small_family(seed=91, n_programs=333, stmts=(1, 9), n_trees=60, depth=7,
                                early_leaf_q=0.2, k=16),
            W.make_small_family(seed=92, n_programs=1, stmts=(1, 1), n_trees=5, depth=3, k=1),
            W.make_small_family(seed=93, n_programs=200, stmts=(2, 5), n_trees=40, depth=6,
                                n_features=64, k=9, bias=0.5),
            W.make_small_family(seed=94, n_programs=90, stmts=(1, 4), n_trees=25, depth=5,
                                n_features=30, k=5)]
    x = fams[0].features
    x[3, 7], x[64, 0], x[65, 163], x[130, 5] = np.nan, np.inf, -np.inf, -0.0
    api.fs_profile_begin(32)
    devs = run_families(api, fams[:3], api.FS_ROWMAJOR)
    prof = api.fs_profile_end()
    for f, d in zip(fams[:3], devs):
        check_family(oracle, f, d)
    assert prof["pack"][1] == 0 and prof["traverse"][1] == 1 and prof["traverse_global"][1] == 0
    api.fs_profile_begin(32)
    devs = run_families(api, fams, api.FS_ROWMAJOR)
    prof = api.fs_profile_end()
    for f, d in zip(fams, devs):
        check_family(oracle, f, d)
    assert prof["pack"][1] == 1


def test_foresee_step_shape_many_small_pools_sharing_a_family_model(api, oracle):
    """The family-scoped step of the paper's Algorithm 1: the family's one model estimates the
    candidates of several member subgraphs, and g*p = 16 candidates per subgraph go on
    (Section 4.2; p = 0.25, g = 64).  Here: 5 families, 3-6 subgraph pools each, pools of
    320..4288 programs (the paper's Section 3.2 example sizes), one batched call for all."""
    import torch
    rng = np.random.default_rng(77)
    host, devs = [], []
    models = {}
    for fam in range(5):
        base = W.make_small_family(seed=500 + fam, n_programs=8, stmts=(1, 8), n_trees=30,
                                   depth=7, early_leaf_q=0.0 if fam % 2 else 0.25, k=16)
        for sub in range(int(rng.integers(3, 7))):
            n_prog = int(rng.choice([320, 1024, 2048, 2304, 4288]))
            pool = W.make_small_family(seed=1000 * fam + sub, n_programs=n_prog, stmts=(1, 8),
                                       n_trees=1, depth=1, k=16)
            pool.model = base.model                      # the family's model, shared
            host.append(pool)
    shared = {}
    for f in host:
        key = id(f.model)
        if key not in shared:
            shared[key] = api.fs_model.from_arrays(f.model)
        tmp = api.DeviceFamily(f, want_row_score=True, want_leaf_idx=True)
        tmp.model.destroy()
        tmp.model = shared[key]                          # one fs_model per family
        devs.append(tmp)
    api.fs_score_families([d.family() for d in devs])
    api.fs_topk([d.topk_request() for d in devs])
    torch.cuda.synchronize()
    for f, d in zip(host, devs):
        check_family(oracle, f, d)
    assert len(shared) == 5 and len(devs) >= 15


def test_maximum_sizes_of_the_interface(api, oracle):
    """The documented limits themselves: FS_MAX_FEATURES columns, a tree of FS_MAX_TREE_NODES
    nodes (leaf ids up to 65534), one program holding 100 000 rows next to one-row programs,
    and just past each limit an error instead of a launch."""
    import torch
    wide = W.make_small_family(seed=61, n_programs=40, stmts=(1, 5), n_trees=6, depth=5,
                               n_features=api.FS_MAX_FEATURES, k=7)
    deep = W.make_small_family(seed=62, n_programs=300, stmts=(1, 3), n_trees=2, depth=15,
                               n_features=20, k=11)
    assert int(np.diff(deep.model.tree_off).max()) == api.FS_MAX_TREE_NODES
    long_ = W.make_small_family(seed=63, n_programs=3, stmts=(1, 1), n_trees=9, depth=4,
                                n_features=32, k=3)
    rng = np.random.default_rng(64)
    long_.features = W.draw_features(rng, 100_002, 0.3, n_features=32)
    long_.prog_off = np.array([0, 1, 100_001, 100_002], np.int32)
    fams = [wide, deep, long_]
    for layout in LAYOUTS:
        devs = [api.DeviceFamily(f, layout=layout, want_row_score=True, want_leaf_idx=True)
                for f in fams]
        api.fs_score_families([d.family() for d in devs])
        api.fs_topk([d.topk_request() for d in devs])
        torch.cuda.synchronize()
        for f, d in zip(fams, devs):
            check_family(oracle, f, d)
    # one past the limits
    m = wide.model
    with pytest.raises(api.FsError):
        api.fs_model.from_arrays(W.Model(api.FS_MAX_FEATURES + 1, m.tree_off, m.split_feature,
                                         m.threshold, m.left, m.right, m.value, 0.0))
    big = W.make_small_family(seed=65, n_programs=1, stmts=(1, 1), n_trees=1, depth=16,
                              n_features=8, k=1)
    with pytest.raises(api.FsError):
        api.fs_model.from_arrays(big.model)


@pytest.mark.parametrize("seed", range(48))
def test_random_shapes_across_the_kernel_choices(api, oracle, tune, seed):
    """Seeded random families: feature counts on both sides of the LDS formats' limit, depths
    0..12 perfect or irregular (so the compact, 8-byte-node, rank-coded and global-memory
    kernels all get picked somewhere), ragged program lengths, both layouts; everything the
    library returns is compared, three families per submission."""
    import torch
    rng = np.random.default_rng([seed, 31337])
    if seed >= 16:                # the later seeds also force several tile groups per workgroup
        tune(api.FS_TUNE_LDS_GROUPS, int(rng.choice([2, 3, 4, 16])))
    fams = []
    for i in range(3):
        depth = int(rng.integers(0, 13))
        q = float(rng.choice([0.0, 0.0, 0.15, 0.35]))
        nf = int(rng.choice([1, 7, 64, 164, 255, 256, 300]))
        n_trees = int(rng.integers(1, 40 if depth > 9 else 90))
        n_prog = int(rng.integers(1, 400))
        hi = int(rng.integers(1, 20))
        fams.append(W.make_small_family(seed=1000 * seed + i, n_programs=n_prog, stmts=(1, hi),
                                        n_trees=n_trees, depth=depth, early_leaf_q=q,
                                        n_features=nf, k=int(rng.integers(1, 80)),
                                        bias=float(rng.choice([0.0, -0.5, 0.125])),
                                        zero_frac=float(rng.choice([0.0, 0.3, 0.9]))))
    layouts = [int(rng.integers(0, 2)) for _ in fams]
    devs = [api.DeviceFamily(f, layout=l, want_row_score=True, want_leaf_idx=True)
            for f, l in zip(fams, layouts)]
    api.fs_score_families([d.family() for d in devs])
    api.fs_topk([d.topk_request() for d in devs])
    torch.cuda.synchronize()
    for f, d in zip(fams, devs):
        check_family(oracle, f, d)
