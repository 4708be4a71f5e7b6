"""Seeded synthetic workloads: families of candidate programs and their cost models.

This module only *draws inputs*.  It holds none of the method's arithmetic (no tree
traversal, no sums of model outputs, no ranking, no training step) so that both the CPU
oracle's tests and the HIP path's tests can take their inputs from it without sharing any
of the method.  Training targets are drawn from a hidden closed-form response of the
statements (step and product terms, `draw_response`) totalled per program: data for the
trainers to fit, evaluated with whole-column numpy comparisons, never through a tree.

The tuner the paper describes keeps one gradient-boosted-tree cost model per
subgraph family (Section 4.2, Algorithm 1: one model initialised per family) and
uses it to estimate every generated candidate of the family's subgraphs before the
best `g` go on to measurement (Section 4.2; `g = min(64, B / #subgraphs)`).  The
real candidates' feature vectors come out of a tensor compiler that is not
available here, so each workload below is a synthetic stand-in with the structure
such a tuning round has: a few to a few dozen families (the paper's Table 1 lists
9-38 subgraphs per network), each with its own ensemble, its own candidate
programs, a handful of statements per program, and 164 features per statement.

Five recipes (`CONFIGS`) are provided.  Every recipe can be shrunk with `scale`
(fewer programs) and `trees` (fewer trees) so that a slow CPU oracle can score the
whole case; the distributions and the structure stay the same.

Conventions fixed here (and relied on by both implementations' callers):

* A model is a concatenation of trees.  Tree `t` owns nodes
  `[tree_off[t], tree_off[t+1])`; node ids inside the arrays are LOCAL to the tree
  and the root is local node 0.
* `split_feature[n] < 0` marks a leaf whose output is `value[n]`.  Otherwise the
  node is internal and a row goes LEFT iff `x[split_feature[n]] < threshold[n]`
  (strict), else RIGHT.
* "depth d" counts split levels: a full tree of depth d has 2^d - 1 internal nodes
  and 2^d leaves, numbered in heap order (children of n are 2n+1, 2n+2).  Irregular
  trees are numbered in breadth-first order; children ids exceed the parent's.
* Features are row-major float32, one row per statement; program `p` owns rows
  `[prog_off[p], prog_off[p+1])`.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

N_FEATURES = 164


@dataclass
class Model:
    """One family's tree ensemble as flat host arrays (see module docstring)."""
    n_features: int
    tree_off: np.ndarray       # int32 [T+1]
    split_feature: np.ndarray  # int32 [N]  (<0 => leaf)
    threshold: np.ndarray      # float32 [N]
    left: np.ndarray           # int32 [N]  local child id, -1 at leaves
    right: np.ndarray          # int32 [N]
    value: np.ndarray          # float32 [N] leaf output (0 at internal nodes)
    bias: float = 0.0

    @property
    def n_trees(self) -> int:
        return int(self.tree_off.shape[0] - 1)

    @property
    def n_nodes(self) -> int:
        return int(self.split_feature.shape[0])


@dataclass
class Family:
    model: Model
    features: np.ndarray   # float32 [R, D] row-major
    prog_off: np.ndarray   # int32 [P+1]
    k: int

    @property
    def n_rows(self) -> int:
        return int(self.features.shape[0])

    @property
    def n_programs(self) -> int:
        return int(self.prog_off.shape[0] - 1)


@dataclass
class Case:
    name: str
    seed: int
    families: List[Family] = field(default_factory=list)
    notes: str = ""

    @property
    def n_rows(self) -> int:
        return sum(f.n_rows for f in self.families)

    @property
    def n_programs(self) -> int:
        return sum(f.n_programs for f in self.families)

    @property
    def feature_bytes(self) -> int:
        return sum(f.features.nbytes for f in self.families)


# --------------------------------------------------------------------------------------
# features
# --------------------------------------------------------------------------------------

def draw_features(rng: np.random.Generator, n_rows: int, zero_frac: float,
                  n_features: int = N_FEATURES,
                  col_scale: Optional[np.ndarray] = None) -> np.ndarray:
    """Rows of `n_features` float32: each entry is exactly 0 with probability
    `zero_frac`, else uniform on [0,1).  With `col_scale` (float64 per column) every
    column is multiplied in float64 and rounded to float32 once."""
    out = np.empty((n_rows, n_features), dtype=np.float32)
    step = max(1, (1 << 22) // n_features)          # ~16 MB blocks keep temporaries small
    for lo in range(0, n_rows, step):
        hi = min(n_rows, lo + step)
        u = rng.random((hi - lo, n_features), dtype=np.float32)
        z = rng.random((hi - lo, n_features), dtype=np.float32) < np.float32(zero_frac)
        u[z] = 0.0
        if col_scale is not None:
            u = (u.astype(np.float64) * col_scale[None, :]).astype(np.float32)
        out[lo:hi] = u
    return out


def draw_col_scale(rng: np.random.Generator, n_features: int = N_FEATURES) -> np.ndarray:
    """Per-column scale 10^U(-3,3), float64."""
    return np.power(10.0, rng.uniform(-3.0, 3.0, size=n_features))


# --------------------------------------------------------------------------------------
# trees
# --------------------------------------------------------------------------------------

def _tree_shape_full(depth: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(is_leaf, left, right) of a full tree of `depth` split levels, heap order."""
    n_int = (1 << depth) - 1
    n = (1 << (depth + 1)) - 1
    ids = np.arange(n, dtype=np.int32)
    is_leaf = ids >= n_int
    left = np.where(is_leaf, -1, 2 * ids + 1).astype(np.int32)
    right = np.where(is_leaf, -1, 2 * ids + 2).astype(np.int32)
    return is_leaf, left, right


def _tree_shape_irregular(rng: np.random.Generator, max_depth: int,
                          q: float) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Breadth-first numbered tree.  The root is always internal; every other node
    above `max_depth` independently becomes a leaf with probability `q`; nodes at
    `max_depth` are leaves."""
    is_leaf_parts, left_parts, right_parts = [], [], []
    level_leaf = np.zeros(1, dtype=bool)            # root internal
    if max_depth == 0:
        level_leaf[:] = True
    next_id = 1
    depth = 0
    while True:
        n_int = int((~level_leaf).sum())
        l = np.full(level_leaf.shape[0], -1, dtype=np.int32)
        r = np.full(level_leaf.shape[0], -1, dtype=np.int32)
        child0 = next_id + 2 * np.arange(n_int, dtype=np.int32)
        l[~level_leaf] = child0
        r[~level_leaf] = child0 + 1
        is_leaf_parts.append(level_leaf)
        left_parts.append(l)
        right_parts.append(r)
        if n_int == 0:
            break
        next_id += 2 * n_int
        depth += 1
        if depth >= max_depth:
            level_leaf = np.ones(2 * n_int, dtype=bool)
        else:
            level_leaf = rng.random(2 * n_int) < q
    return (np.concatenate(is_leaf_parts), np.concatenate(left_parts),
            np.concatenate(right_parts))


def draw_model(rng: np.random.Generator, features: np.ndarray, n_trees: int, depth: int,
               early_leaf_q: float = 0.0, leaf_sigma: float = 0.1,
               bias: float = 0.0) -> Model:
    """An ensemble over the columns of `features`.

    Split features are uniform over the columns.  A node that splits on column j takes
    as threshold the value X[r', j] of a row r' drawn uniformly from `features`, so the
    threshold distribution follows the column's own (zeros and scale included).  Leaf
    outputs are N(0, leaf_sigma) float32.  `early_leaf_q == 0` gives full trees of
    `depth`; otherwise irregular trees of at most `depth`."""
    n_rows, n_features = features.shape
    shapes = []
    if early_leaf_q <= 0.0:
        shape = _tree_shape_full(depth)
        shapes = [shape] * n_trees
    else:
        shapes = [_tree_shape_irregular(rng, depth, early_leaf_q) for _ in range(n_trees)]
    sizes = np.array([s[0].shape[0] for s in shapes], dtype=np.int64)
    tree_off = np.zeros(n_trees + 1, dtype=np.int32)
    np.cumsum(sizes, out=tree_off[1:])
    is_leaf = np.concatenate([s[0] for s in shapes]) if n_trees else np.zeros(0, bool)
    left = np.concatenate([s[1] for s in shapes]) if n_trees else np.zeros(0, np.int32)
    right = np.concatenate([s[2] for s in shapes]) if n_trees else np.zeros(0, np.int32)
    n = is_leaf.shape[0]
    feat = rng.integers(0, n_features, size=n, dtype=np.int32)
    if n_rows > 0:
        src_row = rng.integers(0, n_rows, size=n, dtype=np.int64)
        thr = features[src_row, feat].astype(np.float32)
    else:
        thr = rng.random(n, dtype=np.float32)
    val = (rng.standard_normal(n) * leaf_sigma).astype(np.float32)
    split_feature = np.where(is_leaf, -1, feat).astype(np.int32)
    threshold = np.where(is_leaf, np.float32(0), thr).astype(np.float32)
    value = np.where(is_leaf, val, np.float32(0)).astype(np.float32)
    return Model(n_features=n_features, tree_off=tree_off, split_feature=split_feature,
                 threshold=threshold, left=left.astype(np.int32),
                 right=right.astype(np.int32), value=value, bias=float(bias))


# --------------------------------------------------------------------------------------
# program structure
# --------------------------------------------------------------------------------------

def fixed_prog_off(n_programs: int, stmts: int) -> np.ndarray:
    return (np.arange(n_programs + 1, dtype=np.int64) * stmts).astype(np.int32)


def uniform_prog_off(rng: np.random.Generator, n_programs: int, lo: int, hi: int) -> np.ndarray:
    s = rng.integers(lo, hi + 1, size=n_programs, dtype=np.int64)
    off = np.zeros(n_programs + 1, dtype=np.int64)
    np.cumsum(s, out=off[1:])
    return off.astype(np.int32)


def zipf_program_counts(n_families: int, largest: int, smallest: int, exponent: float) -> List[int]:
    """Rank-size rule P_i = clamp(round(largest * i^-exponent), smallest, largest)."""
    out = []
    for i in range(1, n_families + 1):
        p = int(round(largest * (i ** (-exponent))))
        out.append(max(smallest, min(largest, p)))
    return out


# --------------------------------------------------------------------------------------
# the five recipes
# --------------------------------------------------------------------------------------

@dataclass(frozen=True)
class Recipe:
    name: str
    families: int
    trees: int
    depth: int
    early_leaf_q: float
    zero_frac: float
    k: int
    description: str


CONFIGS: Sequence[Recipe] = (
    Recipe("cfg0_single_small", 1, 100, 6, 0.0, 0.30, 64,
           "1 family, 100 full trees depth 6, 4096 programs x 8 statements"),
    Recipe("cfg1_eight_families", 8, 300, 8, 0.0, 0.30, 128,
           "8 families, 300 full trees depth 8 each, 10000 programs x 16 statements each"),
    Recipe("cfg2_large_population", 1, 500, 10, 0.0, 0.30, 1024,
           "1 family, 500 full trees depth 10, 262144 programs x 8 statements"),
    Recipe("cfg3_powerlaw_families", 30, 200, 8, 0.2, 0.50, 64,
           "30 families, Zipf(1.2) program counts 65536..256, 1..64 statements, "
           "200 irregular trees of depth <= 8 (early leaf 0.2)"),
    Recipe("cfg4_deep_irregular", 64, 400, 12, 0.3, 0.30, 256,
           "64 families, 400 irregular trees of depth <= 12 (early leaf 0.3), 2M rows, "
           "1..32 statements, log-uniform column scales"),
)


def _scaled(n: int, scale: float, floor: int = 1) -> int:
    return max(floor, int(round(n * scale)))


def make_case(cfg: int, seed: int = 0, scale: float = 1.0, trees: Optional[int] = None,
              k: Optional[int] = None) -> Case:
    """Build workload `cfg` (0..4).

    `scale` multiplies program counts (cfg 4: the total row count), `trees` overrides
    the number of trees per family, `k` overrides the cut.  scale=1 and no overrides
    give the full-size workload.  The generator stream is `default_rng([seed, cfg])`.
    """
    rc = CONFIGS[cfg]
    rng = np.random.default_rng([seed, cfg])
    n_trees = rc.trees if trees is None else int(trees)
    kk = rc.k if k is None else int(k)
    case = Case(name=rc.name, seed=seed,
                notes=f"{rc.description}; scale={scale}, trees={n_trees}, k={kk}")

    if cfg in (0, 1, 2):
        per_family = {0: (4096, 8), 1: (10000, 16), 2: (262144, 8)}[cfg]
        n_prog = _scaled(per_family[0], scale)
        for _ in range(rc.families):
            off = fixed_prog_off(n_prog, per_family[1])
            X = draw_features(rng, int(off[-1]), rc.zero_frac)
            m = draw_model(rng, X, n_trees, rc.depth)
            case.families.append(Family(m, X, off, kk))
        return case

    if cfg == 3:
        counts = zipf_program_counts(rc.families, 65536, 256, 1.2)
        counts = [_scaled(c, scale, floor=4) for c in counts]
        order = rng.permutation(rc.families)
        for i in order:
            off = uniform_prog_off(rng, counts[int(i)], 1, 64)
            X = draw_features(rng, int(off[-1]), rc.zero_frac)
            m = draw_model(rng, X, n_trees, rc.depth, early_leaf_q=rc.early_leaf_q)
            case.families.append(Family(m, X, off, kk))
        return case

    if cfg == 4:
        total_rows = _scaled(2_000_000, scale, floor=rc.families * 8)
        # programs of 1..32 statements until the row budget is met (last one truncated)
        est = int(total_rows / 16.5 * 1.2) + 64
        s = rng.integers(1, 33, size=est, dtype=np.int64)
        while s.sum() < total_rows:
            s = np.concatenate([s, rng.integers(1, 33, size=est, dtype=np.int64)])
        c = np.cumsum(s)
        n_prog = int(np.searchsorted(c, total_rows, side="left")) + 1
        s = s[:n_prog].copy()
        s[-1] -= int(c[n_prog - 1] - total_rows)
        fam_of = rng.integers(0, rc.families, size=n_prog)
        for f in range(rc.families):
            sf = s[fam_of == f]
            off = np.zeros(sf.shape[0] + 1, dtype=np.int64)
            np.cumsum(sf, out=off[1:])
            scale_cols = draw_col_scale(rng)
            X = draw_features(rng, int(off[-1]), rc.zero_frac, col_scale=scale_cols)
            m = draw_model(rng, X, n_trees, rc.depth, early_leaf_q=rc.early_leaf_q)
            case.families.append(Family(m, X, off.astype(np.int32), kk))
        return case

    raise ValueError(f"unknown config {cfg}")


def make_foresee_case(seed: int = 0, scale: float = 1.0, families: int = 12,
                      trees: int = 200, depth: int = 8, early_leaf_q: float = 0.2,
                      k: int = 16) -> Case:
    """The family-scoped step of the paper's Algorithm 1 as one batch: every family's single
    model scores the candidate pools of its member subgraphs and g*p = 16 candidates per
    subgraph go on (Section 4.2, p = 0.25, g = 64).

    `families` families of 2..6 member subgraphs (Table 1 of the paper: 9-38 subgraphs per
    network); a pool holds 320..4288 programs (the pool sizes of the Section 3.2 example) of
    1..32 statements; models and features as in the power-law workload (irregular trees of
    depth <= 8, 50 % exact zeros).  The entries of `Case.families` are the pools; pools of one
    family share one `Model` object, which is drawn from the first pool's rows.
    """
    rng = np.random.default_rng([seed, 1001])
    case = Case(name="foresee_step", seed=seed,
                notes=f"foresee step: {families} families x 2..6 pools of 320..4288 programs, "
                      f"k={k}; scale={scale}, trees={trees}")
    for _ in range(families):
        members = int(rng.integers(2, 7))
        model = None
        for _ in range(members):
            n_prog = _scaled(int(rng.integers(320, 4289)), scale, floor=4)
            off = uniform_prog_off(rng, n_prog, 1, 32)
            X = draw_features(rng, int(off[-1]), 0.5)
            if model is None:
                model = draw_model(rng, X, trees, depth, early_leaf_q=early_leaf_q)
            case.families.append(Family(model, X, off, k))
    return case


def draw_cuts(X: np.ndarray, max_cuts: int = 255) -> Tuple[np.ndarray, np.ndarray]:
    """Candidate thresholds for histogram training: per column, at most `max_cuts` of its
    distinct values (never the smallest, which nothing lies below), evenly spaced in rank
    when there are more.  Returns (cut_off [D+1] int32, cuts float32), ascending per column."""
    off = [0]
    out = []
    for j in range(X.shape[1]):
        u = np.unique(X[:, j])
        u = u[~np.isnan(u)][1:]
        if u.shape[0] > max_cuts:
            pick = np.unique(np.round(np.linspace(0, u.shape[0] - 1, max_cuts)).astype(np.int64))
            u = u[pick]
        out.append(u.astype(np.float32))
        off.append(off[-1] + u.shape[0])
    cuts = np.concatenate(out) if out else np.zeros(0, np.float32)
    return np.asarray(off, np.int32), cuts.astype(np.float32)


@dataclass
class TrainSet:
    """Measured programs of one family: what train_cost_model of Algorithm 1 receives."""
    features: np.ndarray   # float32 [R, D] row-major
    prog_off: np.ndarray   # int32 [P+1]
    target: np.ndarray     # float32 [P]
    cut_off: np.ndarray    # int32 [D+1]
    cuts: np.ndarray       # float32

    @property
    def n_rows(self) -> int:
        return int(self.features.shape[0])

    @property
    def n_programs(self) -> int:
        return int(self.prog_off.shape[0] - 1)


@dataclass
class Response:
    """A hidden per-statement response used to draw synthetic measurement targets: a few step
    terms a*[x[f] >= c] plus a few smooth terms w*x[f]*x[g].  It only makes targets that have
    something to learn in them; it is not a model of the scoring method."""
    step_feature: np.ndarray   # int64 [S]
    step_cut: np.ndarray       # float32 [S]
    step_amp: np.ndarray       # float64 [S]
    pair_a: np.ndarray         # int64 [Q]
    pair_b: np.ndarray         # int64 [Q]
    pair_w: np.ndarray         # float64 [Q]

    def rows(self, X: np.ndarray) -> np.ndarray:
        """float64 response of every row of X."""
        out = np.zeros(X.shape[0], np.float64)
        for f, c, a in zip(self.step_feature, self.step_cut, self.step_amp):
            out += a * (X[:, f] >= c)
        for fa, fb, w in zip(self.pair_a, self.pair_b, self.pair_w):
            out += w * (X[:, fa].astype(np.float64) * X[:, fb].astype(np.float64))
        return out


def draw_response(rng: np.random.Generator, probe: np.ndarray, steps: int = 60, pairs: int = 12,
                  sigma: float = 0.1) -> Response:
    """`steps` step terms whose cuts are values the probe rows themselves hold in that column
    (so exact zeros are frequent cuts, as they are frequent values) and `pairs` product terms."""
    n_rows, n_features = probe.shape
    sf = rng.integers(0, n_features, size=steps)
    sc = probe[rng.integers(0, max(1, n_rows), size=steps), sf].astype(np.float32)
    sa = rng.standard_normal(steps) * sigma
    pa = rng.integers(0, n_features, size=pairs)
    pb = rng.integers(0, n_features, size=pairs)
    pw = rng.standard_normal(pairs) * sigma
    return Response(sf, sc, sa, pa, pb, pw)


def _program_totals(rows: np.ndarray, off: np.ndarray) -> np.ndarray:
    """Per-program totals of a per-row quantity (empty programs total 0)."""
    n = off.shape[0] - 1
    if n <= 0:
        return np.zeros(0, np.float64)
    c = np.concatenate([[0.0], np.cumsum(rows, dtype=np.float64)])
    o = off.astype(np.int64)
    return c[o[1:]] - c[o[:-1]]


def make_train_set(seed: int, n_programs: int, stmts: Tuple[int, int] = (1, 16),
                   n_features: int = N_FEATURES, zero_frac: float = 0.3, max_cuts: int = 255,
                   steps: int = 60, pairs: int = 12, noise: float = 0.02) -> TrainSet:
    """Synthetic measured programs: features as in the scoring workloads, targets = a hidden
    step-plus-smooth response of the statements (`draw_response`), totalled per program, plus
    Gaussian noise (so there is something to learn), rounded to float32."""
    rng = np.random.default_rng([seed, 4242])
    lo, hi = stmts
    off = uniform_prog_off(rng, n_programs, lo, hi) if hi > lo else fixed_prog_off(n_programs, lo)
    X = draw_features(rng, int(off[-1]), zero_frac, n_features=n_features)
    hidden = draw_response(rng, X, steps, pairs)
    y = _program_totals(hidden.rows(X), off)
    y = y + rng.normal(0.0, noise, size=n_programs)
    cut_off, cuts = draw_cuts(X, max_cuts)
    return TrainSet(X, off, y.astype(np.float32), cut_off, cuts)


def make_train_case(seed: int = 0, scale: float = 1.0, families: int = 8,
                    max_cuts: int = 255) -> List[TrainSet]:
    """Training sets of one tuning job: `families` family models, each with the measured
    programs of its member subgraphs -- 2000..6000 programs of 1..16 statements, so that the
    job holds roughly 32 000 measured candidates (the paper's Section 5.2 quotes "more than
    30000 candidates as training data" for a 30-subgraph network)."""
    rng = np.random.default_rng([seed, 2002])
    out = []
    for i in range(families):
        n = _scaled(int(rng.integers(2000, 6001)), scale, floor=8)
        out.append(make_train_set(int(rng.integers(1 << 30)) + i, n, stmts=(1, 16),
                                  max_cuts=max_cuts))
    return out


@dataclass
class Subgraph:
    """One subgraph of a synthetic network: measured programs to train on and a validation
    pool with its (noise-free) true scores."""
    family: int
    train: TrainSet
    val_features: np.ndarray   # float32 [R, D]
    val_prog_off: np.ndarray   # int32 [P+1]
    val_target: np.ndarray     # float32 [P]


def make_network(seed: int = 0, n_subgraphs: int = 11, n_families: int = 4, samples: int = 256,
                 val: int = 256, stmts: Tuple[int, int] = (1, 8), n_features: int = 32,
                 max_cuts: int = 63, own_weight: float = 0.35, noise: float = 0.02) -> List[Subgraph]:
    """A network in the shape of the paper's Section 3.1 study (11 subgraphs, 256 measured
    candidates each).  Subgraphs of one family share a hidden response (`draw_response`); every
    subgraph adds a smaller one of its own (`own_weight`), so that pooling samples inside a family
    helps, pooling across families hurts, and training alone starves.  All subgraphs share one
    cut list (drawn from the union of the training features) so that any model can score any
    subgraph's candidates."""
    rng = np.random.default_rng([seed, 3003])
    fam_of = np.sort(rng.integers(0, n_families, size=n_subgraphs))
    fam_of[:n_families] = np.arange(n_families)              # every family has a member
    fam_of = np.sort(fam_of)
    probe = draw_features(rng, 2048, 0.3, n_features=n_features)
    fam_hidden = [draw_response(rng, probe, 48, 8) for _ in range(n_families)]
    parts = []
    for s in range(n_subgraphs):
        own = draw_response(rng, probe, 16, 4, sigma=0.1 * own_weight / 0.35)
        def pool(n_prog):
            off = uniform_prog_off(rng, n_prog, stmts[0], stmts[1])
            X = draw_features(rng, int(off[-1]), 0.3, n_features=n_features)
            y = _program_totals(fam_hidden[int(fam_of[s])].rows(X) + own.rows(X), off)
            return X, off, y
        Xt, offt, yt = pool(samples)
        Xv, offv, yv = pool(val)
        yt = yt + rng.normal(0.0, noise, size=samples)
        parts.append((int(fam_of[s]), Xt, offt, yt.astype(np.float32), Xv, offv, yv.astype(np.float32)))
    cut_off, cuts = draw_cuts(np.concatenate([p[1] for p in parts]), max_cuts)
    return [Subgraph(f, TrainSet(Xt, offt, yt, cut_off, cuts), Xv, offv, yv)
            for f, Xt, offt, yt, Xv, offv, yv in parts]


def pool_train_sets(sets: List[TrainSet]) -> TrainSet:
    """The measured programs of several subgraphs as one training set (same cut lists)."""
    X = np.concatenate([t.features for t in sets])
    lens = np.concatenate([np.diff(t.prog_off) for t in sets]).astype(np.int64)
    off = np.zeros(lens.shape[0] + 1, np.int64)
    np.cumsum(lens, out=off[1:])
    return TrainSet(X, off.astype(np.int32), np.concatenate([t.target for t in sets]),
                    sets[0].cut_off, sets[0].cuts)


def make_small_family(seed: int, n_programs: int, stmts: Tuple[int, int], n_trees: int,
                      depth: int, early_leaf_q: float = 0.0, zero_frac: float = 0.3,
                      n_features: int = N_FEATURES, k: int = 16, bias: float = 0.0,
                      dyadic_leaves: bool = False) -> Family:
    """A free-form family for tests.  With `dyadic_leaves` every leaf output is an
    integer multiple of 1/1024 with magnitude < 1, so any fp32 sum of fewer than 2^13
    of them is exact whatever the order of additions."""
    rng = np.random.default_rng([seed, 977])
    lo, hi = stmts
    off = uniform_prog_off(rng, n_programs, lo, hi) if hi > lo else fixed_prog_off(n_programs, lo)
    X = draw_features(rng, int(off[-1]), zero_frac, n_features=n_features)
    m = draw_model(rng, X, n_trees, depth, early_leaf_q=early_leaf_q, bias=bias)
    if dyadic_leaves:
        leaf = m.split_feature < 0
        q = rng.integers(-1023, 1024, size=m.n_nodes).astype(np.float32) / np.float32(1024)
        m.value = np.where(leaf, q, np.float32(0)).astype(np.float32)
    return Family(m, X, off, k)
