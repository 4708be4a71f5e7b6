"""The seeded generator: shapes, structure and distributions of the five workloads."""
import numpy as np

from paper_2201_00194_amd import workloads as W


def check_model_structure(m):
    assert m.tree_off[0] == 0 and m.tree_off[-1] == m.n_nodes
    for t in range(m.n_trees):
        o, e = m.tree_off[t], m.tree_off[t + 1]
        sf, l, r = m.split_feature[o:e], m.left[o:e], m.right[o:e]
        internal = sf >= 0
        ids = np.arange(e - o)
        assert np.all(l[internal] > ids[internal]) and np.all(r[internal] > ids[internal])
        assert np.all(l[~internal] == -1) and np.all(r[~internal] == -1)
        assert np.all(sf[internal] < m.n_features)
        # every non-root node is the child of exactly one parent
        kids = np.concatenate([l[internal], r[internal]])
        assert np.array_equal(np.sort(kids), np.arange(1, e - o))
        assert np.all(m.value[o:e][internal] == 0)


def test_cfg0_full_size_shape_and_distributions():
    c = W.make_case(0, seed=0)
    f = c.families[0]
    assert f.features.shape == (32768, 164) and f.features.dtype == np.float32
    assert f.n_programs == 4096 and f.k == 64
    assert np.array_equal(np.diff(f.prog_off), np.full(4096, 8))
    m = f.model
    assert m.n_trees == 100 and m.n_nodes == 100 * 127 and m.bias == 0.0
    check_model_structure(m)
    z = (f.features == 0).mean()
    assert abs(z - 0.30) < 0.005
    nz = f.features[f.features != 0]
    assert nz.min() > 0 and nz.max() < 1 and abs(nz.mean() - 0.5) < 0.005
    leaf = m.split_feature < 0
    assert abs(m.value[leaf].std() - 0.1) < 0.005 and abs(m.value[leaf].mean()) < 0.005
    thr = m.threshold[~leaf]
    assert abs((thr == 0).mean() - 0.30) < 0.02          # thresholds follow the column's values
    # heap order
    o = m.tree_off[3]
    assert m.left[o + 5] == 11 and m.right[o + 5] == 12


def test_same_seed_same_case_and_different_seed_differs():
    a = W.make_case(3, seed=5, scale=0.01, trees=8)
    b = W.make_case(3, seed=5, scale=0.01, trees=8)
    c = W.make_case(3, seed=6, scale=0.01, trees=8)
    for fa, fb in zip(a.families, b.families):
        assert np.array_equal(fa.features, fb.features)
        assert np.array_equal(fa.model.threshold, fb.model.threshold)
        assert np.array_equal(fa.prog_off, fb.prog_off)
    assert not np.array_equal(a.families[0].prog_off, c.families[0].prog_off)


def test_cfg3_power_law_and_irregular_trees():
    counts = W.zipf_program_counts(30, 65536, 256, 1.2)
    assert counts[0] == 65536 and counts[1] == 28526 and counts[-1] == 1106
    assert sum(counts) == 201029
    c = W.make_case(3, seed=0, scale=0.02, trees=40)
    assert len(c.families) == 30
    lens = np.concatenate([np.diff(f.prog_off) for f in c.families])
    assert lens.min() >= 1 and lens.max() <= 64 and abs(lens.mean() - 32.5) < 2.0
    sizes = []
    for f in c.families[:4]:
        check_model_structure(f.model)
        sizes.append(np.diff(f.model.tree_off))
        assert abs((f.features == 0).mean() - 0.5) < 0.02
    sizes = np.concatenate(sizes)
    assert 100 < sizes.mean() < 190                      # E[nodes] ~ 141 for q=0.2, depth<=8
    assert sizes.max() <= 511


def test_cfg4_row_budget_and_column_scales():
    c = W.make_case(4, seed=0, scale=0.02, trees=10)
    assert len(c.families) == 64 and c.n_rows == 40000
    lens = np.concatenate([np.diff(f.prog_off) for f in c.families])
    assert lens.min() >= 1 and lens.max() <= 32
    f = c.families[0]
    colmax = f.features.max(axis=0)
    assert colmax.min() < 0.05 and colmax.max() > 20      # scales spread over decades
    check_model_structure(f.model)


def test_cfg1_cfg2_scaled_shapes():
    c1 = W.make_case(1, seed=0, scale=0.01, trees=5)
    assert len(c1.families) == 8 and all(f.n_programs == 100 for f in c1.families)
    assert all(f.n_rows == 1600 and f.k == 128 for f in c1.families)
    assert c1.families[0].model.n_nodes == 5 * 511
    c2 = W.make_case(2, seed=0, scale=0.001, trees=3)
    assert c2.families[0].n_rows == 262 * 8 and c2.families[0].model.n_nodes == 3 * 2047


def test_foresee_case_shape_and_shared_models():
    case = W.make_foresee_case(seed=3, scale=0.05, trees=5)
    models = {id(f.model) for f in case.families}
    assert len(models) == 12 and 24 <= len(case.families) <= 72
    for f in case.families:
        assert f.k == 16 and f.prog_off[0] == 0 and f.prog_off[-1] == f.n_rows
        assert np.all(np.diff(f.prog_off) >= 1) and np.all(np.diff(f.prog_off) <= 32)
        assert f.features.shape == (f.n_rows, 164) and f.model.n_trees == 5
    again = W.make_foresee_case(seed=3, scale=0.05, trees=5)
    assert all(np.array_equal(a.features, b.features) for a, b in zip(case.families, again.families))


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
