"""Benchmark of the scoring hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C] [--seed S]

A step is one pass of the whole path over one batch: fs_score_families (tree traversal,
per-row ensemble sum, per-program segmented sum) for every family of the workload, then
fs_topk for every family.  Inputs (column-blocked features, CSR offsets, models) are
resident in HBM before the timed region.  Prints one JSON line.

The default workload is configs[3] (30 families of power-law size, irregular trees): the
workload list numbers its entries from 0 ("same distributions as config 0"), so this is
the "config 3" its throughput target names.  --config selects any of the five.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def measured_ceilings() -> dict:
    """The JSON line of profiles/ceilings_mi355x.txt (output of fs_ceilings.bin on an MI355X):
    measured HBM read stream, LDS read rates and the synthetic visit loop.  {} if absent."""
    path = os.path.join(ROOT, "profiles", "ceilings_mi355x.txt")
    try:
        for line in open(path):
            if line.startswith("JSON "):
                return json.loads(line[5:])
    except (OSError, ValueError):
        pass
    return {}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="workload 0..4")
    ap.add_argument("--foresee", action="store_true",
                    help="instead of --config: the family-scoped step of Algorithm 1 (many small "
                         "pools per family model, k = 16)")
    ap.add_argument("--train", action="store_true",
                    help="instead of scoring: boosting rounds of the family models on synthetic "
                         "measured programs (train_cost_model of Algorithm 1); a step is one round "
                         "for all families")
    ap.add_argument("--depth", type=int, default=6, help="--train: tree depth")
    ap.add_argument("--evolve", action="store_true",
                    help="instead of scoring a fixed pool: generations of a search with a resident "
                         "population (score only the new candidates, cut, carry the survivors over "
                         "on the device); a step is one generation")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debug only)")
    ap.add_argument("--trees", type=int, default=None, help="override trees per family (debug only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also capture one step (score + cut) into a HIP graph and time its replays "
                         "(`graph_replay`): what a caller of a launch-bound workload would do")
    ap.add_argument("--also", type=str, default=None,
                    help="comma-separated workloads (0..4) to time briefly after the main one and "
                         "report under `other_workloads` (default: 2 when the main one is configs[3], "
                         "since configs[2] calls itself the bandwidth-roofline config; 'none' = skip)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for HBM counters)")
    return ap.parse_args()


TRAVERSAL_SOURCES = ("fs_internal.h", "fs_lds.h", "fs_model.hip", "fs_rank.hip",
                     "fs_traverse_lds.hip")


def source_digest() -> str:
    """Digest of the sources that make the traversal kernels and the model image they walk:
    counter-derived traffic is only quoted while it matches."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2201_00194_amd", "csrc")
    for name in TRAVERSAL_SOURCES:
        h.update(name.encode())
        h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(config: int):
    """HBM bytes per launch of the traversal kernel from the committed counter summary, or
    None if there is none for this workload or the kernels changed since it was taken."""
    path = os.path.join(ROOT, "profiles", "traverse_hbm_traffic.txt")
    try:
        rec = json.load(open(path))
    except (OSError, ValueError):
        return None
    ent = rec.get("configs", {}).get(str(config))
    if not ent or rec.get("source_digest") != source_digest():
        return None
    return ent.get("hbm_bytes_per_launch")


def mean_path_length(case, devs, api, torch, sample_rows: int = 512):
    """(mean splits per (row, tree) on a row sample, from the leaf ids the library itself reports
    for the first rows of every family; walked levels per (row, tree) in a lock-step walk to the
    deepest leaf; (row, tree) pairs of the workload)."""
    import numpy as np
    tot, cnt, lock = 0.0, 0, 0.0
    for f, d in zip(case.families, devs):
        m = f.model
        if m.n_trees == 0 or f.n_rows == 0:
            continue
        # depth of every node: children have larger ids, so repeated relaxation settles in
        # at most max-depth passes
        sizes = np.diff(m.tree_off)
        node_off = np.repeat(m.tree_off[:-1], sizes).astype(np.int64)
        internal = np.flatnonzero(m.split_feature >= 0)
        gl = node_off[internal] + m.left[internal]
        gr = node_off[internal] + m.right[internal]
        depth = np.zeros(m.n_nodes, np.int32)
        for _ in range(64):
            before = depth.copy()
            depth[gl] = depth[internal] + 1
            depth[gr] = depth[internal] + 1
            if np.array_equal(before, depth):
                break
        nr = min(sample_rows, f.n_rows)
        leaf = torch.zeros(nr * m.n_trees, dtype=torch.int16, device="cuda")
        off = torch.tensor([0, nr], dtype=torch.int32, device="cuda")
        ps = torch.zeros(1, dtype=torch.float32, device="cuda")
        api.fs_score_families([api.Family(d.model, d.features, api.FS_COLBLOCK64, nr, off, ps, None, leaf)])
        li = leaf.cpu().numpy().view(np.uint16).reshape(nr, m.n_trees).astype(np.int64)
        dl = depth[m.tree_off[:-1][None, :] + li]
        tot += float(dl.mean()) * f.n_rows * m.n_trees
        cnt += f.n_rows * m.n_trees
        lock += float(depth.max()) * f.n_rows * m.n_trees
    return (tot / max(1, cnt), lock / max(1, cnt), cnt)


def quick_measure(cfg: int, seed: int, np, torch, api, W, steps: int = 10, warmup: int = 3) -> dict:
    """A short timing of another workload with the same step (score + cut) and the same
    accounting as the main one: ms per step, rows/s, traversal kernel time and HBM fraction."""
    case = W.make_case(cfg, seed=seed)
    devs = api.upload_case(case, layout=api.FS_COLBLOCK64)
    fams = api.PreparedFamilies([d.family() for d in devs])
    reqs = api.PreparedTopk([d.topk_request() for d in devs])
    for _ in range(warmup):
        api.fs_score_families(fams)
        api.fs_topk(reqs)
    torch.cuda.synchronize()
    api.fs_profile_begin(8 * steps + 8)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        api.fs_score_families(fams)
        api.fs_topk(reqs)
    e1.record()
    torch.cuda.synchronize()
    prof = api.fs_profile_end()
    ms = e0.elapsed_time(e1) / steps
    trav_ms = max(prof["traverse"][0], prof["rank_code"][0] + prof["traverse_rank"][0],
                  prof["traverse_global"][0]) / steps
    model_bytes = sum(8 * m.n_nodes for m in {id(f.model): f.model for f in case.families}.values())
    alg_bytes = sum(f.n_rows * (f.model.n_features * 4 + 4) for f in case.families) + model_bytes
    achieved = alg_bytes / (trav_ms * 1e-3) / 1e9 if trav_ms > 0 else 0.0
    out = {"workload": "configs[%d] %s" % (cfg, case.name), "rows": case.n_rows, "steps": steps,
           "ms_per_step": round(ms, 5), "rows_per_s": round(case.n_rows / (ms * 1e-3), 1),
           "traverse_ms": round(trav_ms, 5), "achieved_gbs": round(achieved, 2),
           "frac_of_hbm_peak": round(achieved / HBM_PEAK_GBS, 5),
           "topk_us_per_family": round(prof["topk"][0] / steps * 1e3 / max(1, len(case.families)), 3)}
    del devs, fams, reqs, case
    torch.cuda.empty_cache()
    return out


def train_main(args, np, torch, api, W):
    """Boosting rounds for all families of a synthetic tuning job.  value = statement rows
    taken through one boosting round per second."""
    t0 = time.time()
    sets = W.make_train_case(seed=args.seed, scale=args.scale)
    gen_s = time.time() - t0
    total = args.warmup + args.steps
    prm = api.train_params(max_depth=args.depth, eta=0.2, lam=1.0)
    trs = [api.fs_trainer.from_train_set(ts, max_depth=args.depth, max_trees=total) for ts in sets]
    n_rows = sum(ts.n_rows for ts in sets)
    n_prog = sum(ts.n_programs for ts in sets)
    n_feat = sets[0].features.shape[1]
    if args.warmup:
        api.fs_train_boost(trs, args.warmup, prm)
    torch.cuda.synchronize()
    api.fs_profile_begin(16 * args.depth * args.steps + 64)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    w0 = time.perf_counter()
    e0.record()
    api.fs_train_boost(trs, args.steps, prm)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - w0) * 1e3
    prof = api.fs_profile_end()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    # dominant kernel: the histogram build.  Algorithmic bytes per launch (one level): every
    # bin once (1 B per row and feature) plus gradient, curvature and node of every row once.
    hist_ms, hist_n = prof["train_hist"]
    alg_bytes = n_rows * (n_feat + 10)
    hist_avg = hist_ms / max(1, hist_n)
    achieved = alg_bytes / (hist_avg * 1e-3) / 1e9 if hist_avg > 0 else 0.0
    out = {
        "metric": "statement-rows per boosting round per second (family cost-model training)",
        "value": round(n_rows / (ms_per_step * 1e-3), 1), "unit": "rows/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64+f64",
        "data": "synthetic",
        "config": {"workload": "training: %d families, depth %d, 255 cuts per feature" %
                               (len(sets), args.depth), "seed": args.seed, "scale": args.scale,
                   "rows": n_rows, "programs": n_prog, "features": n_feat},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": None,
                     "kernel": "train_hist_kernel (one level)",
                     "kernel_avg_ms": round(hist_avg, 5),
                     "algorithmic_bytes_per_launch": int(alg_bytes)},
        "kernels_ms_per_step": {k: round(v[0] / max(1, args.steps), 5) for k, v in prof.items()
                                if k.startswith("train")},
        "host_wall_ms_per_step": round(wall_ms / args.steps, 5),
        "workload_gen_s": round(gen_s, 2),
    }
    if not args.no_cpu_baseline:
        from oracle import train_oracle as TO
        TO.build()
        ts = min(sets, key=lambda s: s.n_rows)
        rounds = 2
        c0 = time.perf_counter()
        TO.train(ts.features, ts.prog_off, ts.target, ts.cut_off, ts.cuts, n_rounds=rounds,
                 max_depth=args.depth, eta=0.2, lam=1.0)
        t_cpu = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": round(ts.n_rows * rounds / t_cpu, 1), "unit": "rows/s",
                               "cores": 1, "kind": "oracle",
                               "sample": "smallest family (%d rows), %d rounds in %.2f s wall"
                                         % (ts.n_rows, rounds, t_cpu)}
    print(json.dumps(out))


def evolve_main(args, np, torch, api, W):
    """Generations of one family's search: population of 16384 programs resident on the device,
    49152 new candidates per generation (8 statements each), irregular 200-tree model as in the
    power-law workload.  Per generation: fs_score_families on the new candidates only, fs_topk
    over old + new scores, fs_gather_programs into the next population buffer."""
    n_pop, n_new, stmts, nf = 16384, int(49152 * args.scale), 8, 164
    t0 = time.time()
    rng = np.random.default_rng([args.seed, 5005])
    probe = W.draw_features(rng, 4096, 0.5)
    model = W.draw_model(rng, probe, args.trees or 200, 8, early_leaf_q=0.2)
    pool = W.Family(model, W.draw_features(rng, (n_pop + n_new) * stmts, 0.5),
                    W.fixed_prog_off(n_pop + n_new, stmts), n_pop)
    gen_s = time.time() - t0
    handle = api.fs_model.from_arrays(model)
    first = W.Family(model, pool.features[: n_pop * stmts], W.fixed_prog_off(n_pop, stmts), n_pop)
    new = W.Family(model, pool.features[n_pop * stmts:], W.fixed_prog_off(n_new, stmts), n_pop)
    d_first = api.DeviceFamily(first, model=handle)
    d_new = api.DeviceFamily(new, model=handle)            # the same candidates every generation
    cap = n_pop * stmts
    pops = [dict(x=torch.zeros(((cap + 63) // 64) * nf * 64, dtype=torch.float32, device="cuda"),
                 off=torch.zeros(n_pop + 1, dtype=torch.int32, device="cuda"),
                 sc=torch.zeros(n_pop + n_new, dtype=torch.float32, device="cuda")) for _ in range(2)]
    pops[0]["x"].copy_(d_first.features[: pops[0]["x"].numel()])
    pops[0]["off"].copy_(d_first.prog_off)
    keep = torch.zeros(n_pop, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    api.fs_score_families([api.Family(handle, pops[0]["x"], api.FS_COLBLOCK64, cap, pops[0]["off"],
                                      pops[0]["sc"][:n_pop], None, None)])
    state = {"cur": 0}

    def step():
        c = pops[state["cur"]]
        n = pops[1 - state["cur"]]
        api.fs_score_families([api.Family(handle, d_new.features, api.FS_COLBLOCK64, new.n_rows,
                                          d_new.prog_off, c["sc"][n_pop:], None, None)])
        api.fs_topk([api.TopkRequest(c["sc"], n_pop + n_new, n_pop, keep, None)])
        api.fs_gather_programs(nf, [(c["x"], c["off"], c["sc"][:n_pop], n_pop),
                                    (d_new.features, d_new.prog_off, c["sc"][n_pop:], n_new)],
                               keep, n_pop, n["x"], cap, n["off"], n["sc"][:n_pop], status)
        state["cur"] = 1 - state["cur"]

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    api.fs_profile_begin(8 * args.steps + 8)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    prof = api.fs_profile_end()
    assert int(status.item()) == 0
    ms = e0.elapsed_time(e1) / args.steps
    trav_ms, trav_n = prof["traverse"]
    alg_bytes = new.n_rows * (nf * 4 + 4) + 8 * model.n_nodes
    trav_avg = trav_ms / max(1, trav_n)
    achieved = alg_bytes / (trav_avg * 1e-3) / 1e9 if trav_avg > 0 else 0.0
    out = {"metric": "candidate statement-rows per second through one search generation "
                     "(score new, cut, carry survivors over)",
           "value": round(new.n_rows / (ms * 1e-3), 1), "unit": "rows/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": "evolutionary generation: population %d, %d new candidates x %d "
                                  "statements, %d trees" % (n_pop, n_new, stmts, model.n_trees),
                      "seed": args.seed, "scale": args.scale},
           "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": None,
                        "kernel": "traverse_lds_kernel", "kernel_avg_ms": round(trav_avg, 5),
                        "algorithmic_bytes_per_launch": int(alg_bytes)},
           "kernels_ms_per_step": {k: round(v[0] / max(1, args.steps), 5) for k, v in prof.items()
                                   if v[1]},
           "workload_gen_s": round(gen_s, 2)}
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only; --gpus %d is not supported "
              "(no collectives, no sharding in this library)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2201_00194_amd import api, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.train:
        return train_main(args, np, torch, api, W)
    if args.evolve:
        return evolve_main(args, np, torch, api, W)

    t0 = time.time()
    if args.foresee:
        case = W.make_foresee_case(seed=args.seed, scale=args.scale,
                                   **({"trees": args.trees} if args.trees else {}))
    else:
        case = W.make_case(args.config, seed=args.seed, scale=args.scale, trees=args.trees)
    gen_s = time.time() - t0
    devs = api.upload_case(case, layout=api.FS_COLBLOCK64)
    fams = api.PreparedFamilies([d.family() for d in devs])
    reqs = api.PreparedTopk([d.topk_request() for d in devs])
    n_rows, n_prog = case.n_rows, case.n_programs
    torch.cuda.synchronize()

    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        b = torch.empty_like(a)
        a.fill_(1.0)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    def step():
        api.fs_score_families(fams)
        api.fs_topk(reqs)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    api.fs_profile_begin(4 * args.steps + 8)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    w0 = time.perf_counter()
    e0.record()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - w0) * 1e3
    prof = api.fs_profile_end()
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = max(ev_ms, 0.0) / args.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    rows_per_s = n_rows / (ms_per_step * 1e-3)

    # ---- roofline of the dominant kernel (LDS-staged traversal) --------------------------------
    # Algorithmic bytes per launch: every feature once (n_features * 4 B per row), one fp32 row
    # score written per row, each family's packed model read once.
    # The traversal is one of: LDS kernel; rank coding + rank kernel (deep perfect trees);
    # global-memory kernel.  Whichever carried the rows is the dominant kernel (group).
    cands = {"traverse_lds_kernel": prof["traverse"],
             "rank_code_kernel+traverse_rank_kernel":
                 (prof["rank_code"][0] + prof["traverse_rank"][0], prof["traverse_rank"][1]),
             "traverse_global_kernel": prof["traverse_global"]}
    kname = max(cands, key=lambda k: cands[k][0])
    trav_ms, trav_n = cands[kname]
    model_bytes = sum(8 * m.n_nodes for m in {id(f.model): f.model for f in case.families}.values())
    alg_bytes = sum(f.n_rows * (f.model.n_features * 4 + 4) for f in case.families) + model_bytes
    trav_avg_ms = trav_ms / max(1, trav_n)
    achieved = alg_bytes / (trav_avg_ms * 1e-3) / 1e9 if trav_avg_ms > 0 else 0.0
    ceil = measured_ceilings()
    stream = ceil.get("hbm_read_stream_gbs")
    roofline = {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": None if args.foresee else recorded_traffic(args.config),
                "kernel": kname, "kernel_avg_ms": round(trav_avg_ms, 5),
                "algorithmic_bytes_per_launch": int(alg_bytes),
                "measured_read_stream": stream,
                "frac_of_measured_stream": round(achieved / stream, 5) if stream else None}

    out = {
        "metric": "statement-rows scored/sec + achieved HBM GB/s (% of peak); per-family top-k us",
        "value": round(rows_per_s, 1),
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": ("foresee step (Algorithm 1, family scope) %s" % case.name) if args.foresee
                   else "configs[%d] %s" % (args.config, case.name), "seed": args.seed,
                   "scale": args.scale, "trees_override": args.trees, "families": len(case.families), "rows": n_rows,
                   "programs": n_prog, "feature_layout": "colblock64",
                   "feature_bytes": int(case.feature_bytes)},
        "roofline": roofline,
        "kernels_ms_per_step": {k: round(v[0] / max(1, args.steps), 5) for k, v in prof.items()},
        "topk_us_per_family": round(prof["topk"][0] / max(1, prof["topk"][1]) * 1e3
                                    / max(1, len(case.families)), 3),
        "ms_per_step_median": round(per_step[len(per_step) // 2], 5),
        "ms_per_step_min": round(per_step[0], 5),
        "host_wall_ms_per_step": round(wall_ms / args.steps, 5),
        "workload_gen_s": round(gen_s, 2),
    }

    # ---- what actually binds the kernel: LDS instruction issue of the visit loop ---------------
    mean_path, lock_path, pairs = mean_path_length(case, devs, api, torch)
    visits_alg = mean_path * pairs
    visits_walked = lock_path * pairs
    # peak: one node read + one feature read per visit at the measured conflict-free LDS rate;
    # synthetic_loop: what a lock-step walk with nothing else around it reaches on this chip
    vpeak, vloop = ceil.get("visit_peak_conflict_free"), ceil.get("visit_loop_measured")
    walked_rate = visits_walked / (trav_avg_ms * 1e-3)
    out["visit_roofline"] = {
        "bound": "lds-issue", "unit": "node visits/s",
        "achieved_algorithmic": round(visits_alg / (trav_avg_ms * 1e-3), 1),
        "achieved_walked": round(walked_rate, 1),
        "peak": vpeak, "frac_walked": round(walked_rate / vpeak, 4) if vpeak else None,
        "synthetic_loop": vloop,
        "frac_walked_of_synthetic_loop": round(walked_rate / vloop, 4) if vloop else None,
        "mean_path": round(mean_path, 3), "walked_levels": round(lock_path, 3)}

    if args.graph:
        api.fs_workspace_reserve(api.fs_workspace_bytes(fams), api.fs_topk_workspace_bytes(reqs))
        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        g0 = torch.cuda.Event(enable_timing=True)
        g1 = torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(args.steps):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        g_ms = g0.elapsed_time(g1) / args.steps
        out["graph_replay"] = {"ms_per_step": round(g_ms, 5), "rows_per_s": round(n_rows / (g_ms * 1e-3), 1)}
        del graph

    also = args.also
    if also is None:
        also = "2" if (args.config == 3 and not args.foresee and args.scale == 1.0 and args.trees is None) else "none"
    if also != "none":
        del devs, fams, reqs
        torch.cuda.empty_cache()
        out["other_workloads"] = [quick_measure(int(c), args.seed, np, torch, api, W)
                                  for c in also.split(",") if c.strip() != ""]

    if not args.no_cpu_baseline:
        from oracle import oracle as O
        O.build()
        # ---- CPU baseline: the oracle as it stands, on a bounded sample --------------------------
        threads = min(16, os.cpu_count() or 1)
        budget = 2.0e10                     # node visits: roughly 30 core-seconds of the oracle
        remaining = budget
        sample_rows, t_cpu, desc, whole = 0, 0.0, [], 0
        for fi, f in enumerate(case.families):
            if remaining <= 0 or f.n_rows == 0 or f.n_programs == 0:
                continue
            per_row = f.model.n_trees * max(1.0, mean_path)
            want_rows = int(remaining / max(1.0, per_row))
            p_end = int(np.searchsorted(f.prog_off, want_rows, side="right")) - 1
            p_end = max(1, min(f.n_programs, p_end))
            sub_off = f.prog_off[: p_end + 1]
            rows = int(sub_off[-1])
            if rows == 0:
                continue
            c0 = time.perf_counter()
            ps = O.score_programs(f.model, f.features[:rows], sub_off, threads=threads)
            O.topk(ps, min(f.k, p_end))
            t_cpu += time.perf_counter() - c0
            sample_rows += rows
            remaining -= rows * per_row
            if p_end == f.n_programs:
                whole += 1
            else:
                desc.append("family %d programs [0,%d) = %d rows" % (fi, p_end, rows))
        if whole:
            desc.insert(0, "%d whole families" % whole)
        # the same oracle on one thread, on the first 1/16 of the first sampled family
        f0 = next(f for f in case.families if f.n_rows > 0 and f.n_programs > 0)
        p1 = max(1, min(f0.n_programs, int(2.0e10 / 16 / max(1.0, f0.model.n_trees * max(1.0, mean_path)
                                                                 * max(1.0, f0.n_rows / f0.n_programs)))))
        c0 = time.perf_counter()
        O.score_programs(f0.model, f0.features[: int(f0.prog_off[p1])], f0.prog_off[: p1 + 1], threads=1)
        t1 = time.perf_counter() - c0
        out["cpu_baseline"] = {
            "value": round(sample_rows / t_cpu, 1) if t_cpu > 0 else None, "unit": "rows/s",
            "cores": threads, "kind": "oracle",
            "value_1_thread": round(int(f0.prog_off[p1]) / t1, 1) if t1 > 0 else None,
            "sample": "; ".join(desc) + " (%d rows); scored + cut in %.2f s wall" % (sample_rows, t_cpu)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
