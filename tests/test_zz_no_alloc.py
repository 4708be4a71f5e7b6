"""fs_topk_noalloc (the cut for callers that cannot allocate) against fs_topk: same indices,
same score bits, on two calls in a row, the second with a smaller input -- the fixed device
array keeps the first call's contents, which must not leak into the second."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2201_00194_amd import api as A
    return A


def both_cuts(api, scores, ks):
    """[(idx, score) by fs_topk], [(idx, score) by fs_topk_noalloc] for one batch of requests."""
    import torch
    out = []
    for fn in (api.fs_topk, api.fs_topk_noalloc):
        dev = [torch.from_numpy(s).cuda() for s in scores]
        idx = [torch.full((max(1, k),), -7, dtype=torch.int32, device="cuda") for k in ks]
        val = [torch.full((max(1, k),), float("nan"), dtype=torch.float32, device="cuda") for k in ks]
        torch.cuda.synchronize()
        fn([api.TopkRequest(d, d.shape[0], k, i, v) for d, k, i, v in zip(dev, ks, idx, val)])
        torch.cuda.synchronize()
        out.append([(i.cpu().numpy(), v.cpu().numpy()) for i, v in zip(idx, val)])
    return out


def assert_same(a, b):
    for (ia, va), (ib, vb) in zip(a, b):
        assert np.array_equal(ia, ib)
        assert np.array_equal(va.view(np.uint32), vb.view(np.uint32))


def test_noalloc_cut_equals_the_allocating_cut_twice_in_a_row(api, oracle):
    rng = np.random.default_rng(77)
    # first call: a long request (16 slices, candidate lists in the fixed array), a medium sliced
    # one with ties across the cut, and a short one served by a single workgroup
    big = rng.standard_normal(262144).astype(np.float32)
    tied = np.round(rng.standard_normal(20000) * 4).astype(np.float32) / 4
    small = rng.standard_normal(300).astype(np.float32)
    small[5] = np.nan
    small[7] = -0.0
    first = both_cuts(api, [big, tied, small], [1024, 64, 500])
    assert_same(*first)
    # second call, smaller input: fewer and shorter lists than the array still holds
    mid = rng.standard_normal(9000).astype(np.float32)
    tiny = rng.standard_normal(40).astype(np.float32)
    second = both_cuts(api, [mid, tiny], [33, 16])
    assert_same(*second)
    # and both agree with the oracle's full sort
    for s, k, (gi, gv) in zip([big, tied, small], [1024, 64, 500], first[1]):
        idx, val = oracle.topk(s, k)
        assert np.array_equal(gi[:k], idx) and np.array_equal(gv[:k].view(np.uint32), val.view(np.uint32))
    for s, k, (gi, gv) in zip([mid, tiny], [33, 16], second[1]):
        idx, val = oracle.topk(s, k)
        assert np.array_equal(gi[:k], idx) and np.array_equal(gv[:k].view(np.uint32), val.view(np.uint32))


def test_noalloc_rejects_what_does_not_fit(api):
    import torch
    s = torch.zeros(70000, dtype=torch.float32, device="cuda")
    out = torch.zeros(8192, dtype=torch.int32, device="cuda")
    with pytest.raises(api.FsError) as e:                      # wide cut of a long request
        api.fs_topk_noalloc([api.TopkRequest(s, 70000, 8192, out, None)])
    assert e.value.code == api.FS_EUNSUPPORTED
    with pytest.raises(api.FsError) as e:                      # too many workgroups
        api.fs_topk_noalloc([api.TopkRequest(s, 100, 4, out, None)] * 80)
    assert e.value.code == api.FS_EUNSUPPORTED and "descriptors" in str(e.value)
    with pytest.raises(api.FsError) as e:                      # candidate lists beyond the array
        api.fs_topk_noalloc([api.TopkRequest(s, 70000, 4096, out, None)] * 8)
    assert e.value.code == api.FS_EUNSUPPORTED
    api.fs_topk_noalloc([api.TopkRequest(s, 70000, 16, out, None)])   # still works afterwards
    torch.cuda.synchronize()
    assert out[:16].cpu().numpy().tolist() == list(range(16))
