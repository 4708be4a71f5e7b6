"""ctypes front of the plain-C training oracle in `fs_train_oracle.c`.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU-baseline leg import
this module; the library never does.  `train` runs boosting rounds of the family cost model
on measured programs (Algorithm 1 of the paper, train_cost_model; Section 4.3) exactly as the
C file's header defines them and returns the trees in the flat arrays the scoring path reads.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fs_train_oracle.c")
_LIB = os.path.join(_HERE, "libfs_train_oracle.so")
_lib = None


def build(force: bool = False) -> str:
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
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.fso_train.argtypes = [ctypes.c_int32, ctypes.c_int64, f32p, i32p, ctypes.c_int32, f32p,
                                  i32p, f32p, ctypes.c_float, ctypes.c_int32, ctypes.c_int32,
                                  ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                  ctypes.c_float, i32p, i32p, f32p, i32p, i32p, f32p,
                                  ctypes.c_int64, f32p, f32p, f64p]
        lib.fso_train.restype = ctypes.c_int
        lib.fso_bins.argtypes = [ctypes.c_int32, ctypes.c_int64, f32p, i32p, f32p, i32p]
        lib.fso_bins.restype = None
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


@dataclass
class Trained:
    tree_off: np.ndarray
    split_feature: np.ndarray
    threshold: np.ndarray
    left: np.ndarray
    right: np.ndarray
    value: np.ndarray
    row_pred: np.ndarray
    prog_pred: np.ndarray
    loss: np.ndarray          # before every round and after the last


def train(X, prog_off, target, cut_off, cuts, *, bias=0.0, n_rounds=1, max_depth=6, eta=0.3,
          lam=1.0, min_gain=0.0, min_child_weight=1.0, grad_scale=float(1 << 20)) -> Trained:
    lib = _load()
    X = np.ascontiguousarray(X, dtype=np.float32)
    n_rows, n_features = X.shape
    prog_off = np.ascontiguousarray(prog_off, dtype=np.int32)
    target = np.ascontiguousarray(target, dtype=np.float32)
    cut_off = np.ascontiguousarray(cut_off, dtype=np.int32)
    cuts = np.ascontiguousarray(cuts, dtype=np.float32)
    if cuts.size == 0:
        cuts = np.zeros(1, np.float32)
    n_programs = prog_off.shape[0] - 1
    cap = n_rounds * ((1 << (max_depth + 1)) - 1) + 1
    tree_off = np.zeros(n_rounds + 1, np.int32)
    sf = np.zeros(cap, np.int32)
    th = np.zeros(cap, np.float32)
    le = np.zeros(cap, np.int32)
    ri = np.zeros(cap, np.int32)
    va = np.zeros(cap, np.float32)
    row_pred = np.zeros(n_rows, np.float32)
    prog_pred = np.zeros(n_programs, np.float32)
    loss = np.zeros(n_rounds + 1, np.float64)
    rc = lib.fso_train(n_features, n_rows, _p(X, ctypes.c_float), _p(prog_off, ctypes.c_int32),
                       n_programs, _p(target, ctypes.c_float), _p(cut_off, ctypes.c_int32),
                       _p(cuts, ctypes.c_float), bias, n_rounds, max_depth, eta, lam, min_gain,
                       min_child_weight, grad_scale, _p(tree_off, ctypes.c_int32),
                       _p(sf, ctypes.c_int32), _p(th, ctypes.c_float), _p(le, ctypes.c_int32),
                       _p(ri, ctypes.c_int32), _p(va, ctypes.c_float), cap,
                       _p(row_pred, ctypes.c_float), _p(prog_pred, ctypes.c_float),
                       _p(loss, ctypes.c_double))
    if rc != 0:
        raise ValueError("fso_train rejected its arguments")
    n = int(tree_off[-1])
    return Trained(tree_off, sf[:n].copy(), th[:n].copy(), le[:n].copy(), ri[:n].copy(),
                   va[:n].copy(), row_pred, prog_pred, loss)


def bins(X, cut_off, cuts) -> np.ndarray:
    lib = _load()
    X = np.ascontiguousarray(X, dtype=np.float32)
    cut_off = np.ascontiguousarray(cut_off, dtype=np.int32)
    cuts = np.ascontiguousarray(cuts, dtype=np.float32)
    if cuts.size == 0:
        cuts = np.zeros(1, np.float32)
    out = np.zeros(X.shape, np.int32)
    lib.fso_bins(X.shape[1], X.shape[0], _p(X, ctypes.c_float), _p(cut_off, ctypes.c_int32),
                 _p(cuts, ctypes.c_float), _p(out, ctypes.c_int32))
    return out
