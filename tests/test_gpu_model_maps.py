"""Monolithic / per-family / per-subgraph model maps (Section 3.1, Fig. 1 and 2 of the paper;
Section 4.2) through the library: every model of every map is trained on the device and must
equal the training oracle's model for the same pooled samples; every (model, validation pool)
score must equal the scoring oracle's."""
import numpy as np
import pytest

from paper_2201_00194_amd import model_maps as MM
from paper_2201_00194_amd import workloads as W

@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2201_00194_amd import api as A
    return A


@pytest.mark.gpu
def test_three_maps_train_and_score_like_the_oracles(api, oracle):
    from oracle import train_oracle as TO
    TO.build()
    subs = W.make_network(seed=5, n_subgraphs=6, n_families=2, samples=96, val=64, n_features=16,
                          max_cuts=31)
    prm = api.train_params(max_depth=3, eta=0.4, lam=1.0)
    for name, mapping in MM.maps_for(subs).items():
        models, groups = MM.train_map(api, subs, mapping, 5, prm)
        assert len(models) == {"monolithic": 1, "family": 2, "individual": 6}[name]
        for m, g in zip(models, groups):
            ts = W.pool_train_sets([subs[s].train for s in g])
            exp = TO.train(ts.features, ts.prog_off, ts.target, ts.cut_off, ts.cuts, n_rounds=5,
                           max_depth=3, eta=0.4, lam=1.0)
            assert np.array_equal(m.tree_off, exp.tree_off)
            assert np.array_equal(m.split_feature, exp.split_feature)
            assert np.array_equal(m.threshold.view(np.uint32), exp.threshold.view(np.uint32))
            assert np.array_equal(m.value.view(np.uint32), exp.value.view(np.uint32))
        sc = MM.cross_scores(api, models, subs)
        for i, m in enumerate(models):
            for j, sg in enumerate(subs):
                ps = oracle.program_scores(oracle.row_scores(m, sg.val_features), sg.val_prog_off)
                assert np.array_equal(sc[i][j].view(np.uint32), ps.view(np.uint32))


def test_pairwise_accuracy_against_hand_counts():
    t = np.array([1.0, 2.0, 3.0, 3.0], np.float32)
    assert MM.pairwise_accuracy(np.array([1.0, 2.0, 3.0, 4.0]), t) == 1.0          # the tie is skipped
    assert MM.pairwise_accuracy(np.array([4.0, 3.0, 2.0, 1.0]), t) == 0.0
    assert MM.pairwise_accuracy(np.array([1.0, 3.0, 2.0, 2.0]), t) == pytest.approx(3 / 5)
