"""Parity at the full sizes of the five workloads, in the launch configuration the benchmark
times (column-blocked features, no optional outputs).  Where scoring every program with the
CPU oracle takes too long, a seeded sample of programs is scored one by one; the top-k cut
is always checked in full against the oracle's cut of the device's own scores, and against
the oracle end to end where the oracle scores everything.
"""
import os

import numpy as np
import pytest

from paper_2201_00194_amd import workloads as W

pytestmark = pytest.mark.gpu
RTOL, ATOL = 1e-5, 1e-6
THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2201_00194_amd import api as A
    return A


def run_case(api, case):
    import torch
    devs = api.upload_case(case, layout=api.FS_COLBLOCK64)
    api.fs_score_families(api.PreparedFamilies([d.family() for d in devs]))
    api.fs_topk(api.PreparedTopk([d.topk_request() for d in devs]))
    torch.cuda.synchronize()
    return devs


def check_cut_properties(oracle, fam, dev):
    """Checks of the cut that hold at any size."""
    own = dev.prog_score.cpu().numpy()[: fam.n_programs]
    gi = dev.topk_idx.cpu().numpy()[: fam.k]
    gv = dev.topk_score.cpu().numpy()[: fam.k]
    idx, val = oracle.topk(own, fam.k)                   # oracle's cut of the device's scores
    assert np.array_equal(gi, idx)
    assert np.array_equal(gv.view(np.uint32), val.view(np.uint32))
    kk = min(fam.k, fam.n_programs)
    assert len(set(gi[:kk].tolist())) == kk
    assert np.all(np.diff(gv[:kk]) <= 0)                 # best first
    if kk < fam.n_programs:
        rest = np.ones(fam.n_programs, bool)
        rest[gi[:kk]] = False
        assert own[rest].max() <= gv[kk - 1]             # nothing better was left out
    return own


def check_sample(oracle, fam, own, n_sample, seed):
    rng = np.random.default_rng(seed)
    n = min(n_sample, fam.n_programs)
    sample = np.unique(np.concatenate([rng.integers(0, fam.n_programs, n),
                                       [0, fam.n_programs - 1]]))
    exp = oracle.score_program_sample(fam.model, fam.features, fam.prog_off, sample)
    np.testing.assert_allclose(own[sample], exp, rtol=RTOL, atol=ATOL)
    assert np.array_equal(own[sample].view(np.uint32), exp.view(np.uint32))


def check_full(oracle, fam, dev):
    ps = oracle.score_programs(fam.model, fam.features, fam.prog_off, threads=THREADS)
    own = dev.prog_score.cpu().numpy()[: fam.n_programs]
    np.testing.assert_allclose(own, ps, rtol=RTOL, atol=ATOL)
    assert np.array_equal(own.view(np.uint32), ps.view(np.uint32))
    idx, val = oracle.topk(ps, fam.k)
    assert np.array_equal(dev.topk_idx.cpu().numpy()[: fam.k], idx)
    assert np.array_equal(dev.topk_score.cpu().numpy()[: fam.k].view(np.uint32), val.view(np.uint32))


def test_cfg1_full_size_every_program(api, oracle):
    case = W.make_case(1, seed=0)
    assert case.n_rows == 1_280_000
    devs = run_case(api, case)
    for f, d in zip(case.families, devs):
        check_cut_properties(oracle, f, d)
    for f, d in list(zip(case.families, devs))[:3]:      # three families end to end
        check_full(oracle, f, d)
    for i, (f, d) in enumerate(list(zip(case.families, devs))[3:]):
        check_sample(oracle, f, d.prog_score.cpu().numpy()[: f.n_programs], 200, 10 + i)


def test_cfg2_full_size_sampled(api, oracle):
    case = W.make_case(2, seed=0)
    assert case.n_rows == 2_097_152 and case.families[0].k == 1024
    devs = run_case(api, case)
    f, d = case.families[0], devs[0]
    own = check_cut_properties(oracle, f, d)
    check_sample(oracle, f, own, 1500, 20)
    # the 64 best programs, recomputed one by one, really have the scores reported
    best = d.topk_idx.cpu().numpy()[:64].astype(np.int64)
    exp = oracle.score_program_sample(f.model, f.features, f.prog_off, best)
    assert np.array_equal(d.topk_score.cpu().numpy()[:64].view(np.uint32), exp.view(np.uint32))


def test_cfg3_full_size_sampled(api, oracle):
    case = W.make_case(3, seed=0)
    assert len(case.families) == 30 and case.n_programs == 201029
    devs = run_case(api, case)
    for i, (f, d) in enumerate(zip(case.families, devs)):
        own = check_cut_properties(oracle, f, d)
        check_sample(oracle, f, own, 120, 30 + i)
    # the smallest families end to end
    small = sorted(range(30), key=lambda i: case.families[i].n_rows)[:6]
    for i in small:
        check_full(oracle, case.families[i], devs[i])


def test_cfg4_full_size_every_program(api, oracle):
    case = W.make_case(4, seed=0)
    assert len(case.families) == 64 and case.n_rows == 2_000_000
    devs = run_case(api, case)
    for i, (f, d) in enumerate(zip(case.families, devs)):
        check_cut_properties(oracle, f, d)
        if i % 4 == 0:
            check_full(oracle, f, d)
        else:
            check_sample(oracle, f, d.prog_score.cpu().numpy()[: f.n_programs], 60, 40 + i)


def test_foresee_step_full_size_every_program(api, oracle):
    """The family-scoped step of Algorithm 1 at the size `bench.py --foresee` times: every
    pool of every family scored by the family's shared model and cut to 16, all compared with
    the oracle (about 0.9 M rows)."""
    case = W.make_foresee_case(seed=0)
    assert len({id(f.model) for f in case.families}) == 12
    devs = run_case(api, case)
    assert len({id(d.model) for d in devs}) == 12        # one fs_model per family
    for fam, dev in zip(case.families, devs):
        check_cut_properties(oracle, fam, dev)
        check_full(oracle, fam, dev)
