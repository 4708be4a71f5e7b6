"""fs_gather_programs: survivors of a cut carried into a new family on the device, against the
plain gather in the oracle module; and the property that makes it useful -- the carried scores
are the scores the library gives the new family when it scores it again."""
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


def gather(api, devs, keep, capacity, with_scores=True):
    import torch
    nf = devs[0].host.model.n_features
    k = torch.from_numpy(np.asarray(keep, np.int32)).cuda()
    tiles = (capacity + 63) // 64
    out_x = torch.full((max(1, tiles * nf * 64),), float("nan"), dtype=torch.float32, device="cuda")
    out_off = torch.full((len(keep) + 1,), -9, dtype=torch.int32, device="cuda")
    out_sc = torch.full((max(1, len(keep)),), float("nan"), dtype=torch.float32, device="cuda")
    status = torch.full((1,), -9, dtype=torch.int32, device="cuda")
    src = [(d.features, d.prog_off, d.prog_score if with_scores else None, d.n_programs) for d in devs]
    api.fs_gather_programs(nf, src, k, len(keep), out_x, capacity, out_off, out_sc, status)
    torch.cuda.synchronize()
    return out_x, out_off.cpu().numpy(), out_sc.cpu().numpy()[: len(keep)], int(status.item())


def test_gather_from_two_scored_families_matches_the_plain_gather(api, oracle):
    import torch
    fams = [W.make_small_family(seed=71, n_programs=300, stmts=(1, 9), n_trees=20, depth=5, k=16),
            W.make_small_family(seed=72, n_programs=120, stmts=(3, 3), n_trees=20, depth=5, k=16)]
    fams[1].model = fams[0].model
    devs = api.upload_case(W.Case("two", 0, fams))
    api.fs_score_families([d.family() for d in devs])
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    keep = rng.permutation(420)[:150].astype(np.int32)
    keep[10] = -1
    keep[77] = -1
    keep[5] = keep[6]                                             # a program may be kept twice
    scores = [d.prog_score.cpu().numpy()[: d.n_programs] for d in devs]
    ex, eoff, esc = oracle.gather_programs(
        [(f.features, f.prog_off, s) for f, s in zip(fams, scores)], keep)
    out_x, off, sc, status = gather(api, devs, keep, capacity=int(eoff[-1]) + 5)
    assert status == 0 and np.array_equal(off, eoff)
    assert np.array_equal(sc.view(np.uint32), esc.view(np.uint32))
    got = api.unpack_colblock64(out_x, int(eoff[-1]), 164)
    assert np.array_equal(got.view(np.uint32), ex.view(np.uint32))
    # padding rows of the last tile are zero
    tiles = (int(eoff[-1]) + 63) // 64
    full = out_x[: tiles * 164 * 64].cpu().numpy().reshape(tiles, 164, 64)
    pad = int(eoff[-1]) % 64
    if pad:
        assert np.all(full[-1, :, pad:] == 0)
    # scoring the gathered family again gives the carried scores, bit for bit
    n_keep = len(keep)
    new_ps = torch.full((n_keep,), float("nan"), dtype=torch.float32, device="cuda")
    off_dev = torch.from_numpy(off).cuda()
    fam = api.Family(devs[0].model, out_x, api.FS_COLBLOCK64, int(eoff[-1]), off_dev, new_ps, None, None)
    api.fs_score_families([fam])
    torch.cuda.synchronize()
    again = new_ps.cpu().numpy()
    real = keep >= 0
    assert np.array_equal(again[real].view(np.uint32), sc[real].view(np.uint32))
    assert np.all(again[~real] == 0) and np.all(np.isneginf(sc[~real]))


def test_gather_capacity_bad_indices_and_empty_requests(api, oracle):
    fam = W.make_small_family(seed=73, n_programs=50, stmts=(2, 6), n_trees=3, depth=2, k=4)
    devs = api.upload_case(W.Case("one", 0, [fam]))
    keep = np.arange(50, dtype=np.int32)
    total = int(fam.prog_off[-1])
    _, off, _, status = gather(api, devs, keep, capacity=total - 1, with_scores=False)
    assert status == 1 and np.all(off == 0)
    _, off, sc, status = gather(api, devs, keep, capacity=total, with_scores=False)
    assert status == 0 and off[-1] == total and np.all(np.isneginf(sc))
    bad = np.array([0, 50, 7, -3], np.int32)
    _, off, _, status = gather(api, devs, bad, capacity=64)
    ex, eoff, _ = oracle.gather_programs([(fam.features, fam.prog_off, None)], [0, -1, 7, -1])
    assert status == 2 and np.array_equal(off, eoff)
    _, off, _, status = gather(api, devs, np.zeros(0, np.int32), capacity=0)
    assert status == 0 and off.tolist() == [0]
    with pytest.raises(api.FsError):
        gather(api, devs, np.zeros(api.FS_MAX_TOPK + 1, np.int32), capacity=64)


@pytest.mark.parametrize("order", ["long_first", "short_first", "random", "max_keep"])
def test_gather_with_very_uneven_program_lengths(api, oracle, order):
    """The row copy finds the owner of every output row by a search that starts from a
    proportional guess: programs sorted by length (rows bunched at one end), many empty
    programs and repeated indices put that guess far off on either side."""
    fam = W.make_small_family(seed=75, n_programs=700, stmts=(0, 40), n_trees=2, depth=2, k=4)
    devs = api.upload_case(W.Case("one", 0, [fam]))
    lens = np.diff(fam.prog_off)
    rng = np.random.default_rng(6)
    if order == "long_first":
        keep = np.argsort(-lens, kind="stable").astype(np.int32)
    elif order == "short_first":
        keep = np.argsort(lens, kind="stable").astype(np.int32)
        keep[::5] = -1
    elif order == "random":
        keep = rng.integers(0, 700, 1500).astype(np.int32)            # repeats are allowed
        keep[rng.integers(0, 1500, 400)] = -1
    else:
        short = np.flatnonzero(lens <= 2)
        keep = short[rng.integers(0, short.shape[0], api.FS_MAX_TOPK)].astype(np.int32)
        keep[-3:] = np.argsort(-lens)[:3]                              # the long ones last
    ex, eoff, esc = oracle.gather_programs([(fam.features, fam.prog_off, None)], keep.tolist())
    out_x, off, sc, status = gather(api, devs, keep, capacity=int(eoff[-1]), with_scores=False)
    assert status == 0
    assert np.array_equal(off, eoff)
    got = api.unpack_colblock64(out_x, int(eoff[-1]), 164)
    assert np.array_equal(got.view(np.uint32), ex.view(np.uint32))


def test_generations_with_a_resident_population_match_rescoring_everything(api, oracle):
    """Three generations of: score only the new candidates, cut (old scores + new scores) to the
    population size, gather the survivors from (population, new) into the next population --
    no host round trip in between.  The oracle scores everything from scratch every generation;
    programs, order and scores of the final population must be identical."""
    import torch
    n_pop, nf = 96, 164
    base = W.make_small_family(seed=81, n_programs=n_pop, stmts=(1, 7), n_trees=30, depth=6,
                               early_leaf_q=0.2, k=n_pop)
    news = [W.make_small_family(seed=82 + g, n_programs=150, stmts=(1, 7), n_trees=1, depth=1, k=1)
            for g in range(3)]
    model = base.model
    handle = api.fs_model.from_arrays(model)
    cap_rows = 7 * n_pop
    # device: two population buffers, one score buffer [n_pop + n_new]
    pops = []
    for _ in range(2):
        pops.append(dict(x=torch.zeros(((cap_rows + 63) // 64) * nf * 64, dtype=torch.float32, device="cuda"),
                         off=torch.zeros(n_pop + 1, dtype=torch.int32, device="cuda")))
    sbuf = [torch.zeros(n_pop + 150, dtype=torch.float32, device="cuda") for _ in range(2)]
    scores = sbuf[0]
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    keep = torch.zeros(n_pop, dtype=torch.int32, device="cuda")
    d0 = api.DeviceFamily(base, model=handle)
    pops[0]["x"][: d0.features.numel()] = d0.features
    pops[0]["off"].copy_(d0.prog_off)
    api.fs_score_families([api.Family(handle, pops[0]["x"], api.FS_COLBLOCK64, base.n_rows,
                                      pops[0]["off"], scores[:n_pop], None, None)])
    # host twin
    hX, hoff = base.features, base.prog_off
    hs = oracle.program_scores(oracle.row_scores(model, hX), hoff)
    cur = 0
    for g, nw in enumerate(news):
        dn = api.DeviceFamily(nw, model=handle)
        api.fs_score_families([api.Family(handle, dn.features, api.FS_COLBLOCK64, nw.n_rows, dn.prog_off,
                                          scores[n_pop:], None, None)])
        api.fs_topk([api.TopkRequest(scores, n_pop + 150, n_pop, keep, None)])
        nxt = 1 - cur
        api.fs_gather_programs(nf, [(pops[cur]["x"], pops[cur]["off"], scores[:n_pop], n_pop),
                                    (dn.features, dn.prog_off, scores[n_pop:], 150)],
                               keep, n_pop, pops[nxt]["x"], cap_rows, pops[nxt]["off"],
                               sbuf[nxt][:n_pop], status)          # outputs never overlap sources
        cur = nxt
        scores = sbuf[cur]
        # oracle: everything again
        ns = oracle.program_scores(oracle.row_scores(model, nw.features), nw.prog_off)
        idx, _ = oracle.topk(np.concatenate([hs, ns]), n_pop)
        hX, hoff, hs = oracle.gather_programs([(hX, hoff, hs), (nw.features, nw.prog_off, ns)], idx)
        again = oracle.program_scores(oracle.row_scores(model, hX), hoff)
        assert np.array_equal(again.view(np.uint32), hs.view(np.uint32))
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    off = pops[cur]["off"].cpu().numpy()
    assert np.array_equal(off, hoff)
    assert np.array_equal(scores[:n_pop].cpu().numpy().view(np.uint32), hs.view(np.uint32))
    got = api.unpack_colblock64(pops[cur]["x"], int(hoff[-1]), nf)
    assert np.array_equal(got.view(np.uint32), hX.view(np.uint32))
