"""Which samples train which cost model: monolithic, per family, per subgraph.

Section 3.1 of the paper compares one monolithic cost model for all subgraphs of a network with
an individual model per subgraph (Fig. 1) and shows how well the model of subgraph X predicts
the candidates of subgraph Y (Fig. 2); Section 4.2 settles on one model per subgraph family.
A *map* here assigns every subgraph to the model that estimates it.  All models of a map are
trained in one `fs_train_boost` batch on the pooled measured programs of their subgraphs, and
all (model, validation pool) pairs are scored in one `fs_score_families` call -- the library
does the arithmetic; this module only arranges the inputs and, for reporting, compares the
resulting rankings with the true ones on the host.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

from . import workloads as W


def maps_for(subgraphs: Sequence[W.Subgraph]) -> Dict[str, List[int]]:
    """model index per subgraph for the three arrangements the paper discusses."""
    n = len(subgraphs)
    return {"monolithic": [0] * n,
            "family": [s.family for s in subgraphs],
            "individual": list(range(n))}


def groups_of(mapping: Sequence[int]) -> List[List[int]]:
    out: Dict[int, List[int]] = {}
    for s, m in enumerate(mapping):
        out.setdefault(m, []).append(s)
    return [out[k] for k in sorted(out)]


def train_map(api, subgraphs: Sequence[W.Subgraph], mapping: Sequence[int], rounds: int, params,
              bias: float = 0.0):
    """One model per group of the map, trained on the device in one batch.  Returns
    (host `Model` per group, groups)."""
    import torch
    groups = groups_of(mapping)
    sets = [W.pool_train_sets([subgraphs[s].train for s in g]) for g in groups]
    trs = [api.fs_trainer.from_train_set(ts, bias=bias, max_depth=params.max_depth, max_trees=rounds)
           for ts in sets]
    api.fs_train_boost(trs, rounds, params)
    torch.cuda.synchronize()
    nf = subgraphs[0].train.features.shape[1]
    models = []
    for tr in trs:
        to, sf, th, le, ri, va = tr.export()
        models.append(W.Model(nf, to, sf, th, le, ri, va, bias))
        tr.destroy()
    return models, groups


def cross_scores(api, models: Sequence[W.Model], subgraphs: Sequence[W.Subgraph]):
    """scores[m][s] = program scores of subgraph s's validation pool under model m (numpy),
    all pairs in one batched call."""
    import torch
    handles = [api.fs_model.from_arrays(m) for m in models]
    devs = []
    for m, h in zip(models, handles):
        for sg in subgraphs:
            fam = W.Family(m, sg.val_features, sg.val_prog_off, 1)
            devs.append(api.DeviceFamily(fam, model=h))
    api.fs_score_families([d.family() for d in devs])
    torch.cuda.synchronize()
    n = len(subgraphs)
    return [[devs[i * n + j].prog_score.cpu().numpy()[: devs[i * n + j].n_programs]
             for j in range(n)] for i in range(len(models))]


def pairwise_accuracy(score: np.ndarray, truth: np.ndarray) -> float:
    """Share of candidate pairs the scores order like the true values (ties in truth skipped)."""
    ds = np.sign(score[:, None] - score[None, :])
    dt = np.sign(truth[:, None] - truth[None, :])
    mask = np.triu(dt != 0, k=1)
    return float((ds[mask] == dt[mask]).mean()) if mask.any() else 1.0


def study(api, subgraphs: Sequence[W.Subgraph], rounds: int = 40, params=None):
    """Accuracy per subgraph under the three maps, and the model-X-on-subgraph-Y table of the
    individual models."""
    params = params or api.train_params(max_depth=4, eta=0.3, lam=1.0)
    out = {}
    heat = None
    for name, mapping in maps_for(subgraphs).items():
        models, groups = train_map(api, subgraphs, mapping, rounds, params)
        model_of = {s: gi for gi, g in enumerate(groups) for s in g}
        sc = cross_scores(api, models, subgraphs)
        out[name] = [pairwise_accuracy(sc[model_of[s]][s], sg.val_target)
                     for s, sg in enumerate(subgraphs)]
        if name == "individual":
            heat = [[pairwise_accuracy(sc[x][y], subgraphs[y].val_target)
                     for y in range(len(subgraphs))] for x in range(len(subgraphs))]
    return out, heat


def main():
    from . import api
    subgraphs = W.make_network(seed=0)
    acc, heat = study(api, subgraphs)
    print("families:", [s.family for s in subgraphs])
    for name, a in acc.items():
        print("%-11s mean %.3f  per subgraph %s" % (name, float(np.mean(a)), " ".join("%.2f" % v for v in a)))
    print("model X (row) on subgraph Y (column):")
    for row in heat:
        print(" ".join("%.2f" % v for v in row))


if __name__ == "__main__":
    main()
