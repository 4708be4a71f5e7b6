"""ctypes front of the plain-C CPU oracle in `fs_oracle.c`.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's CPU-baseline
leg import this module; the scoring library itself never does.  The functions take the
flat model arrays described in `fs_oracle.c` (trees concatenated, node ids local to each
tree, `split_feature < 0` marks a leaf, strict `<` goes left) and row-major float32
features, and return what the paper's tuning round needs from its cost model: per-row
ensemble outputs, per-program sums over statements, and the k best programs
(Section 2 "Building the Cost Model", Section 3.2 top-k selection, Section 4.2 tune step).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fs_oracle.c")
_LIB = os.path.join(_HERE, "libfs_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with strict IEEE float semantics (no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
               "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        model = [ctypes.c_int32, ctypes.c_int32, i32p, i32p, f32p, i32p, i32p]
        lib.fso_leaf_indices.argtypes = model + [f32p, ctypes.c_int64, i32p]
        lib.fso_leaf_indices.restype = None
        lib.fso_row_scores.argtypes = model + [f32p, ctypes.c_float, f32p, ctypes.c_int64, f32p]
        lib.fso_row_scores.restype = None
        lib.fso_program_scores.argtypes = [f32p, i32p, ctypes.c_int32, f32p]
        lib.fso_program_scores.restype = None
        lib.fso_score_programs.argtypes = model + [f32p, ctypes.c_float, f32p, i32p,
                                                   ctypes.c_int32, ctypes.c_int32, f32p]
        lib.fso_score_programs.restype = None
        lib.fso_topk.argtypes = [f32p, ctypes.c_int32, ctypes.c_int32, i32p, f32p]
        lib.fso_topk.restype = ctypes.c_int
        _lib = lib
    return _lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _model_args(m):
    keep = []
    ptrs = []
    for arr, conv in ((m.tree_off, _i32), (m.split_feature, _i32), (m.threshold, _f32),
                      (m.left, _i32), (m.right, _i32)):
        a, p = conv(arr)
        keep.append(a)
        ptrs.append(p)
    return keep, [ctypes.c_int32(m.n_features), ctypes.c_int32(m.n_trees)] + ptrs


def leaf_indices(model, X: np.ndarray) -> np.ndarray:
    """int32 [R, T]: the leaf (node id local to its tree) each row reaches in each tree."""
    lib = _load()
    Xc, xp = _f32(X)
    assert Xc.ndim == 2 and Xc.shape[1] == model.n_features
    keep, margs = _model_args(model)
    out = np.empty((Xc.shape[0], model.n_trees), dtype=np.int32)
    lib.fso_leaf_indices(*margs, xp, ctypes.c_int64(Xc.shape[0]),
                         out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    return out


def row_scores(model, X: np.ndarray) -> np.ndarray:
    """float32 [R]: bias + sequential fp32 sum over trees of the reached leaf's value."""
    lib = _load()
    Xc, xp = _f32(X)
    assert Xc.ndim == 2 and Xc.shape[1] == model.n_features
    keep, margs = _model_args(model)
    val, vp = _f32(model.value)
    out = np.empty(Xc.shape[0], dtype=np.float32)
    lib.fso_row_scores(*margs, vp, ctypes.c_float(model.bias), xp, ctypes.c_int64(Xc.shape[0]),
                       out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    return out


def program_scores(row_score: np.ndarray, prog_off: np.ndarray) -> np.ndarray:
    """float32 [P]: sequential fp32 sum of each program's row scores, from +0."""
    lib = _load()
    rs, rp = _f32(row_score)
    off, op = _i32(prog_off)
    P = off.shape[0] - 1
    out = np.empty(P, dtype=np.float32)
    lib.fso_program_scores(rp, op, ctypes.c_int32(P),
                           out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    return out


def score_program_range(model, X: np.ndarray, prog_off: np.ndarray, p_begin: int,
                        p_end: int, out: np.ndarray | None = None) -> np.ndarray:
    """Scores of programs [p_begin, p_end) straight from the feature rows."""
    lib = _load()
    Xc, xp = _f32(X)
    off, op = _i32(prog_off)
    keep, margs = _model_args(model)
    val, vp = _f32(model.value)
    if out is None:
        out = np.empty(off.shape[0] - 1, dtype=np.float32)
    lib.fso_score_programs(*margs, vp, ctypes.c_float(model.bias), xp, op,
                           ctypes.c_int32(p_begin), ctypes.c_int32(p_end),
                           out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    return out


def score_programs(model, X: np.ndarray, prog_off: np.ndarray, threads: int = 1) -> np.ndarray:
    """All program scores.  `threads > 1` fans whole programs out over host threads; each
    program's additions keep their order, so the result is bit-identical to threads=1."""
    P = int(np.asarray(prog_off).shape[0] - 1)
    out = np.empty(P, dtype=np.float32)
    if threads <= 1 or P < 2 * threads:
        return score_program_range(model, X, prog_off, 0, P, out)
    _load()
    Xc = np.ascontiguousarray(X, dtype=np.float32)
    bounds = np.linspace(0, P, 8 * threads + 1).astype(np.int64)
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(lambda i: score_program_range(model, Xc, prog_off, int(bounds[i]),
                                                  int(bounds[i + 1]), out),
                    range(len(bounds) - 1)))
    return out


def score_program_sample(model, X: np.ndarray, prog_off: np.ndarray,
                         programs: np.ndarray) -> np.ndarray:
    """Scores of the listed programs only (each computed on its own)."""
    out = np.empty(int(np.asarray(prog_off).shape[0] - 1), dtype=np.float32)
    Xc = np.ascontiguousarray(X, dtype=np.float32)
    for p in np.asarray(programs, dtype=np.int64):
        score_program_range(model, Xc, prog_off, int(p), int(p) + 1, out)
    return out[np.asarray(programs, dtype=np.int64)]


def topk(score: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """(indices int32 [k], scores float32 [k]) by score descending, index ascending; if
    k exceeds the number of programs the tail is (-1, -inf)."""
    lib = _load()
    s, sp = _f32(score)
    idx = np.empty(k, dtype=np.int32)
    val = np.empty(k, dtype=np.float32)
    rc = lib.fso_topk(sp, ctypes.c_int32(s.shape[0]), ctypes.c_int32(k),
                      idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                      val.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc != 0:
        raise MemoryError("oracle top-k could not allocate")
    return idx, val


def gather_programs(sources, keep):
    """Survivors of a cut carried into a new family (the generation step of the evolutionary
    search of Section 2): `sources` is a list of (row-major features, prog_off, scores or None);
    `keep` indexes the concatenation of their programs, -1 meaning an empty program with score
    -inf.  Returns (features, prog_off, scores) in the order of `keep`.  Plain Python loops."""
    first = [0]
    for _, off, _ in sources:
        first.append(first[-1] + len(off) - 1)
    nf = sources[0][0].shape[1]
    rows, out_off, out_sc = [], [0], []
    for p in keep:
        p = int(p)
        if p < 0:
            out_off.append(out_off[-1])
            out_sc.append(-np.inf)
            continue
        s = max(i for i in range(len(sources)) if first[i] <= p)
        X, off, sc = sources[s]
        q = p - first[s]
        rows.append(X[off[q]:off[q + 1]])
        out_off.append(out_off[-1] + int(off[q + 1] - off[q]))
        out_sc.append(float(sc[q]) if sc is not None else -np.inf)
    feats = np.concatenate(rows) if rows else np.zeros((0, nf), np.float32)
    return feats.astype(np.float32), np.asarray(out_off, np.int32), np.asarray(out_sc, np.float32)
