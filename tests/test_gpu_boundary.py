"""Boundary behaviour of the C ABI beyond plain parity: work on a stream that is not the
default one, scoring and the cut overlapping on two streams (they have separate scratch),
and scratch reserved ahead of the calls (fs_workspace_bytes, fs_topk_workspace_bytes,
fs_workspace_reserve)."""
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


def expect(oracle, fam):
    ps = oracle.score_programs(fam.model, fam.features, fam.prog_off)
    return (ps,) + tuple(oracle.topk(ps, fam.k))


def same(dev, fam, ps, idx, val):
    assert np.array_equal(dev.prog_score.cpu().numpy()[: fam.n_programs].view(np.uint32), ps.view(np.uint32))
    assert np.array_equal(dev.topk_idx.cpu().numpy()[: fam.k], idx)
    assert np.array_equal(dev.topk_score.cpu().numpy()[: fam.k].view(np.uint32), val.view(np.uint32))


def families():
    # an LDS-staged irregular model, a rank-coded deep one, and a cut long enough to be sliced
    return [W.make_small_family(seed=61, n_programs=9000, stmts=(1, 3), n_trees=30, depth=8,
                                early_leaf_q=0.2, k=64),
            W.make_small_family(seed=62, n_programs=500, stmts=(2, 6), n_trees=20, depth=9, k=16),
            W.make_small_family(seed=63, n_programs=700, stmts=(1, 1), n_trees=12, depth=4, k=700)]


def test_score_then_cut_on_a_side_stream(api, oracle):
    import torch
    fams = families()
    devs = [api.DeviceFamily(f) for f in fams]
    torch.cuda.synchronize()                      # uploads were made on the default stream
    side = torch.cuda.Stream()                    # plain stream, default priority
    api.fs_score_families([d.family() for d in devs], stream=side)
    api.fs_topk([d.topk_request() for d in devs], stream=side)
    side.synchronize()
    for f, d in zip(fams, devs):
        same(d, f, *expect(oracle, f))


def test_scoring_and_cut_of_other_data_overlap_on_two_streams(api, oracle):
    """The scoring scratch and the top-k scratch are separate regions: a scoring call on one
    stream and a sliced cut of unrelated scores on another may run at the same time."""
    import torch
    fams = families()
    devs = [api.DeviceFamily(f) for f in fams]
    rng = np.random.default_rng(5)
    other = rng.standard_normal(300000).astype(np.float32)
    d_other = torch.from_numpy(other).cuda()
    o_idx = torch.zeros(2048, dtype=torch.int32, device="cuda")
    o_val = torch.zeros(2048, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    a, b = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(3):                            # several rounds in flight, no sync in between
        api.fs_score_families([d.family() for d in devs], stream=a)
        api.fs_topk([api.TopkRequest(d_other, other.shape[0], 2048, o_idx, o_val)], stream=b)
    a.synchronize()
    b.synchronize()
    api.fs_topk([d.topk_request() for d in devs], stream=a)
    a.synchronize()
    for f, d in zip(fams, devs):
        same(d, f, *expect(oracle, f))
    idx, val = oracle.topk(other, 2048)
    assert np.array_equal(o_idx.cpu().numpy(), idx)
    assert np.array_equal(o_val.cpu().numpy().view(np.uint32), val.view(np.uint32))


def test_workspace_sizes_and_reservation(api, oracle):
    import torch
    fams = families()
    devs = [api.DeviceFamily(f) for f in fams]
    prepared = api.PreparedFamilies([d.family() for d in devs])
    reqs = api.PreparedTopk([d.topk_request() for d in devs])
    need = api.fs_workspace_bytes(prepared)
    # row scores of every family (none passes its own buffer) and the rank tiles of the deep model
    rows = sum(f.n_rows for f in fams)
    rank_tiles = ((fams[1].n_rows + 63) // 64) * 64 * 164 * 2
    assert 4 * rows + rank_tiles <= need <= 4 * rows + rank_tiles + 64
    # family 0's cut is sliced (9000 programs): slices x k composites of 8 bytes
    assert api.fs_topk_workspace_bytes(reqs) == 4 * 64 * 8
    # a family that brings its own row-score buffer and has no rank-coded model needs nothing
    own = api.DeviceFamily(fams[2], want_row_score=True)
    assert api.fs_workspace_bytes([own.family()]) == 0
    assert api.fs_topk_workspace_bytes([own.topk_request()]) == 0
    api.fs_workspace_reserve(need, api.fs_topk_workspace_bytes(reqs))
    api.fs_score_families(prepared)
    api.fs_topk(reqs)
    torch.cuda.synchronize()
    for f, d in zip(fams, devs):
        same(d, f, *expect(oracle, f))
    # descriptors the scoring call would reject give 0 and a message
    bad = api.Family(devs[0].model, devs[0].features, 7, fams[0].n_rows, devs[0].prog_off,
                     devs[0].prog_score)
    assert api.fs_workspace_bytes([bad]) == 0 and "layout" in api.fs_last_error()


def test_tuning_overrides_are_explicit_and_reset(api, tune):
    assert api.fs_tune_get(api.FS_TUNE_RANK) == -1
    tune(api.FS_TUNE_RANK, 0)
    assert api.fs_tune_get(api.FS_TUNE_RANK) == 0
    tune(api.FS_TUNE_RANK, -5)
    assert api.fs_tune_get(api.FS_TUNE_RANK) == -1
    with pytest.raises(api.FsError):
        api.fs_tune_set(99, 1)


def test_small_calls_replay_from_a_hip_graph(api, oracle):
    """A scoring call and a cut whose descriptors travel as kernel arguments and whose scratch was
    reserved only enqueue kernels, so they can be captured into a graph.  The graph is replayed
    several times on changed features, with eager library work and synchronisations in between,
    and every replay is checked against the oracle."""
    import torch
    fams = families()
    devs = [api.DeviceFamily(f) for f in fams]
    prepared = api.PreparedFamilies([d.family() for d in devs])
    reqs = api.PreparedTopk([d.topk_request() for d in devs])
    rng = np.random.default_rng(17)
    other = torch.from_numpy(rng.standard_normal(50000).astype(np.float32)).cuda()
    o_idx = torch.zeros(100, dtype=torch.int32, device="cuda")
    other_req = api.PreparedTopk([api.TopkRequest(other, 50000, 100, o_idx, None)])
    # a graph keeps the scratch addresses it was captured with: reserve what any later call needs
    api.fs_workspace_reserve(api.fs_workspace_bytes(prepared),
                             max(api.fs_topk_workspace_bytes(reqs), api.fs_topk_workspace_bytes(other_req)))
    api.fs_score_families(prepared)               # every kernel form once outside capture
    api.fs_topk(reqs)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.fs_score_families(prepared)
        api.fs_topk(reqs)
    for replay in range(4):
        for f, d in zip(fams, devs):              # new candidates in the same buffers
            f.features[:] = W.draw_features(rng, f.n_rows, 0.3, n_features=f.features.shape[1])
            x = torch.from_numpy(f.features).cuda()
            api.fs_pack_colblock64(x, f.n_rows, f.features.shape[1], out=d.features)
            d.prog_score.fill_(float("nan"))
            d.topk_idx.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for f, d in zip(fams, devs):
            same(d, f, *expect(oracle, f))
        # eager work between the replays: another cut (its descriptors overwrite the graph's)
        api.fs_topk(other_req)
        torch.cuda.synchronize()
        assert np.array_equal(o_idx.cpu().numpy(), oracle.topk(other.cpu().numpy(), 100)[0])
