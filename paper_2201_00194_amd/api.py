"""Thin ctypes binding of `libfamilyseer.so` (see include/familyseer.h).

Only argument marshalling lives here: every step of scoring and of the top-k cut runs
in the library's HIP kernels.  PyTorch supplies device memory and the current stream.
The functions carry the names of the C entry points they call.  There is no CPU
fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfamilyseer.so")

FS_OK, FS_EINVAL, FS_ENOMEM, FS_EDEVICE, FS_EUNSUPPORTED = 0, -1, -2, -3, -4
FS_ROWMAJOR, FS_COLBLOCK64 = 0, 1
FS_MAX_TOPK = 16384
FS_MAX_FEATURES = 4096
FS_MAX_TREE_NODES = 65535

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -m paper_2201_00194_amd.build); "
        "there is no fallback path")

_lib = ctypes.CDLL(LIB_PATH)


class FsError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"familyseer error {code}: {message}")
        self.code = code


class _FsFamily(ctypes.Structure):
    _fields_ = [("model", ctypes.c_void_p), ("features", ctypes.c_void_p),
                ("layout", ctypes.c_int32), ("n_rows", ctypes.c_int64),
                ("prog_off", ctypes.c_void_p), ("n_programs", ctypes.c_int32),
                ("prog_score", ctypes.c_void_p), ("row_score", ctypes.c_void_p),
                ("leaf_idx", ctypes.c_void_p)]


class _FsTopkReq(ctypes.Structure):
    _fields_ = [("score", ctypes.c_void_p), ("n", ctypes.c_int32), ("k", ctypes.c_int32),
                ("out_idx", ctypes.c_void_p), ("out_score", ctypes.c_void_p)]


_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)
_lib.fs_last_error.restype = ctypes.c_char_p
_lib.fs_last_error.argtypes = []
_lib.fs_version.restype = ctypes.c_int
_lib.fs_version.argtypes = []
_lib.fs_model_create.restype = ctypes.c_int
_lib.fs_model_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32, ctypes.c_int32,
                                 _i32p, _i32p, _f32p, _i32p, _i32p, _f32p, ctypes.c_float]
_lib.fs_model_destroy.restype = None
_lib.fs_model_destroy.argtypes = [ctypes.c_void_p]
_lib.fs_score_families.restype = ctypes.c_int
_lib.fs_score_families.argtypes = [ctypes.c_int32, ctypes.POINTER(_FsFamily), ctypes.c_void_p]
_lib.fs_topk.restype = ctypes.c_int
_lib.fs_topk.argtypes = [ctypes.c_int32, ctypes.POINTER(_FsTopkReq), ctypes.c_void_p]
_lib.fs_topk_noalloc.restype = ctypes.c_int
_lib.fs_topk_noalloc.argtypes = [ctypes.c_int32, ctypes.POINTER(_FsTopkReq), ctypes.c_void_p]
_lib.fs_pack_colblock64.restype = ctypes.c_int
_lib.fs_pack_colblock64.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                    ctypes.c_void_p, ctypes.c_void_p]
_lib.fs_colblock64_floats.restype = ctypes.c_int64
_lib.fs_colblock64_floats.argtypes = [ctypes.c_int64, ctypes.c_int32]


_lib.fs_workspace_bytes.restype = ctypes.c_size_t
_lib.fs_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.POINTER(_FsFamily)]
_lib.fs_topk_workspace_bytes.restype = ctypes.c_size_t
_lib.fs_topk_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.POINTER(_FsTopkReq)]
_lib.fs_workspace_reserve.restype = ctypes.c_int
_lib.fs_workspace_reserve.argtypes = [ctypes.c_size_t, ctypes.c_size_t]
_lib.fs_tune_set.restype = ctypes.c_int
_lib.fs_tune_set.argtypes = [ctypes.c_int32, ctypes.c_int32]
_lib.fs_tune_get.restype = ctypes.c_int32
_lib.fs_tune_get.argtypes = [ctypes.c_int32]
(FS_TUNE_LDS_TILES, FS_TUNE_LDS_MODE, FS_TUNE_RANK, FS_TUNE_RANK_TILES, FS_TUNE_VERBOSE,
 FS_TUNE_TRAIN_SLAB_ROWS, FS_TUNE_TRAIN_SORT, FS_TUNE_TRAIN_PACKED, FS_TUNE_LDS_GROUPS) = range(9)
FS_TUNE_OPTIONS = 9

_lib.fs_profile_begin.restype = ctypes.c_int
_lib.fs_profile_begin.argtypes = [ctypes.c_int32]
_lib.fs_profile_end.restype = ctypes.c_int
_lib.fs_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), _i32p]
KERNEL_CLASSES = ("traverse", "segsum", "topk", "pack", "traverse_global", "rank_code",
                  "traverse_rank", "train_hist", "train_split", "train_other")


def _check(rc: int) -> None:
    if rc != FS_OK:
        raise FsError(rc, _lib.fs_last_error().decode("utf-8", "replace"))


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def fs_version() -> int:
    return int(_lib.fs_version())


def fs_last_error() -> str:
    return _lib.fs_last_error().decode("utf-8", "replace")


class fs_model:
    """Owner of one `fs_model*` (one family's ensemble, device resident)."""

    def __init__(self, n_features: int, tree_off, split_feature, threshold, left, right, value,
                 bias: float = 0.0):
        to = np.ascontiguousarray(tree_off, dtype=np.int32)
        sf = np.ascontiguousarray(split_feature, dtype=np.int32)
        th = np.ascontiguousarray(threshold, dtype=np.float32)
        le = np.ascontiguousarray(left, dtype=np.int32)
        ri = np.ascontiguousarray(right, dtype=np.int32)
        va = np.ascontiguousarray(value, dtype=np.float32)
        n_trees = int(to.shape[0]) - 1
        handle = ctypes.c_void_p()
        rc = _lib.fs_model_create(
            ctypes.byref(handle), int(n_features), n_trees,
            to.ctypes.data_as(_i32p), sf.ctypes.data_as(_i32p), th.ctypes.data_as(_f32p),
            le.ctypes.data_as(_i32p), ri.ctypes.data_as(_i32p), va.ctypes.data_as(_f32p),
            ctypes.c_float(bias))
        _check(rc)
        self._h = handle
        self.n_features = int(n_features)
        self.n_trees = n_trees

    @classmethod
    def from_arrays(cls, m) -> "fs_model":
        """From any object with the fields of `workloads.Model`."""
        return cls(m.n_features, m.tree_off, m.split_feature, m.threshold, m.left, m.right,
                   m.value, m.bias)

    def destroy(self) -> None:
        if getattr(self, "_h", None) is not None and self._h:
            _lib.fs_model_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Family:
    """Argument bundle for one `fs_family` entry; tensors live on the device."""

    def __init__(self, model: fs_model, features: torch.Tensor, layout: int, n_rows: int,
                 prog_off: torch.Tensor, prog_score: torch.Tensor,
                 row_score: Optional[torch.Tensor] = None,
                 leaf_idx: Optional[torch.Tensor] = None):
        self.model, self.features, self.layout, self.n_rows = model, features, layout, int(n_rows)
        self.prog_off, self.prog_score = prog_off, prog_score
        self.row_score, self.leaf_idx = row_score, leaf_idx
        self.n_programs = int(prog_off.shape[0]) - 1 if prog_off is not None else 0


def _family_array(fams: Sequence[Family]):
    arr = (_FsFamily * max(1, len(fams)))()
    for i, f in enumerate(fams):
        arr[i].model = f.model._h if f.model is not None else None
        arr[i].features = _ptr(f.features)
        arr[i].layout = f.layout
        arr[i].n_rows = f.n_rows
        arr[i].prog_off = _ptr(f.prog_off)
        arr[i].n_programs = f.n_programs
        arr[i].prog_score = _ptr(f.prog_score)
        arr[i].row_score = _ptr(f.row_score)
        arr[i].leaf_idx = _ptr(f.leaf_idx)
    return arr


class PreparedFamilies:
    """A family array marshalled once, for callers that submit the same set repeatedly."""

    def __init__(self, fams: Sequence[Family]):
        self.fams = list(fams)
        self.arr = _family_array(self.fams)
        self.n = len(self.fams)


def fs_score_families(fams, stream: Optional[torch.cuda.Stream] = None) -> None:
    if not isinstance(fams, PreparedFamilies):
        fams = PreparedFamilies(fams)
    _check(_lib.fs_score_families(fams.n, fams.arr, _stream_ptr(stream)))


class TopkRequest:
    def __init__(self, score: Optional[torch.Tensor], n: int, k: int, out_idx: torch.Tensor,
                 out_score: Optional[torch.Tensor] = None):
        self.score, self.n, self.k, self.out_idx, self.out_score = score, int(n), int(k), out_idx, out_score


class PreparedTopk:
    def __init__(self, reqs: Sequence[TopkRequest]):
        self.reqs = list(reqs)
        self.n = len(self.reqs)
        self.arr = (_FsTopkReq * max(1, self.n))()
        for i, r in enumerate(self.reqs):
            self.arr[i].score = _ptr(r.score)
            self.arr[i].n = r.n
            self.arr[i].k = r.k
            self.arr[i].out_idx = _ptr(r.out_idx)
            self.arr[i].out_score = _ptr(r.out_score)


def fs_topk(reqs, stream: Optional[torch.cuda.Stream] = None) -> None:
    if not isinstance(reqs, PreparedTopk):
        reqs = PreparedTopk(reqs)
    _check(_lib.fs_topk(reqs.n, reqs.arr, _stream_ptr(stream)))


def fs_topk_noalloc(reqs, stream: Optional[torch.cuda.Stream] = None) -> None:
    if not isinstance(reqs, PreparedTopk):
        reqs = PreparedTopk(reqs)
    _check(_lib.fs_topk_noalloc(reqs.n, reqs.arr, _stream_ptr(stream)))


def fs_workspace_bytes(fams) -> int:
    if not isinstance(fams, PreparedFamilies):
        fams = PreparedFamilies(fams)
    return int(_lib.fs_workspace_bytes(fams.n, fams.arr))


def fs_topk_workspace_bytes(reqs) -> int:
    if not isinstance(reqs, PreparedTopk):
        reqs = PreparedTopk(reqs)
    return int(_lib.fs_topk_workspace_bytes(reqs.n, reqs.arr))


def fs_workspace_reserve(score_bytes: int, topk_bytes: int) -> None:
    _check(_lib.fs_workspace_reserve(int(score_bytes), int(topk_bytes)))


def fs_tune_set(option: int, value: int) -> None:
    _check(_lib.fs_tune_set(int(option), int(value)))


def fs_tune_get(option: int) -> int:
    return int(_lib.fs_tune_get(int(option)))


def fs_colblock64_floats(n_rows: int, n_features: int) -> int:
    return int(_lib.fs_colblock64_floats(int(n_rows), int(n_features)))


def fs_pack_colblock64(rowmajor: torch.Tensor, n_rows: int, n_features: int,
                       out: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    if out is None:
        out = torch.empty(fs_colblock64_floats(n_rows, n_features), dtype=torch.float32,
                          device=rowmajor.device)
    _check(_lib.fs_pack_colblock64(_ptr(rowmajor), int(n_rows), int(n_features), _ptr(out),
                                   _stream_ptr(stream)))
    return out


def fs_profile_begin(max_records: int) -> None:
    _check(_lib.fs_profile_begin(int(max_records)))


def fs_profile_end() -> dict:
    """{kernel class: (total ms, timed launches)}"""
    ms = (ctypes.c_double * len(KERNEL_CLASSES))()
    cnt = (ctypes.c_int32 * len(KERNEL_CLASSES))()
    _check(_lib.fs_profile_end(ms, cnt))
    return {name: (float(ms[i]), int(cnt[i])) for i, name in enumerate(KERNEL_CLASSES)}


# ---- conveniences for tests and the benchmark (allocation + marshalling only) ---------------

def upload_case(case, layout: int = FS_COLBLOCK64, **kw):
    """One `DeviceFamily` per entry of `case.families`; entries that share a host `Model`
    object share one `fs_model`."""
    models, out = {}, []
    for f in case.families:
        key = id(f.model)
        if key not in models:
            models[key] = fs_model.from_arrays(f.model)
        out.append(DeviceFamily(f, layout=layout, model=models[key], **kw))
    return out


class DeviceFamily:
    """Uploads one `workloads.Family` and allocates its outputs."""

    def __init__(self, fam, layout: int = FS_COLBLOCK64, device: str = "cuda:0",
                 want_row_score: bool = False, want_leaf_idx: bool = False, model=None):
        """`model`: an existing `fs_model` to use (families that share a cost model) instead
        of building one from `fam.model`."""
        dev = torch.device(device)
        self.host = fam
        self.model = model if model is not None else fs_model.from_arrays(fam.model)
        self.n_rows, self.n_programs, self.k = fam.n_rows, fam.n_programs, fam.k
        x = torch.from_numpy(np.ascontiguousarray(fam.features)).to(dev)
        if x.numel() == 0:
            x = torch.zeros(4, dtype=torch.float32, device=dev)
        if layout == FS_COLBLOCK64 and fam.n_rows > 0:
            self.features = fs_pack_colblock64(x, fam.n_rows, fam.model.n_features)
            torch.cuda.synchronize()
            del x
        else:
            self.features = x
        self.layout = layout
        self.prog_off = torch.from_numpy(np.ascontiguousarray(fam.prog_off, dtype=np.int32)).to(dev)
        self.prog_score = torch.full((max(1, fam.n_programs),), float("nan"), dtype=torch.float32,
                                     device=dev)
        self.row_score = (torch.full((max(1, fam.n_rows),), float("nan"), dtype=torch.float32,
                                     device=dev) if want_row_score else None)
        self.leaf_idx = (torch.full((max(1, fam.n_rows * fam.model.n_trees),), -1,
                                    dtype=torch.int16, device=dev) if want_leaf_idx else None)
        self.topk_idx = torch.full((max(1, fam.k),), -7, dtype=torch.int32, device=dev)
        self.topk_score = torch.full((max(1, fam.k),), float("nan"), dtype=torch.float32, device=dev)

    def family(self) -> Family:
        return Family(self.model, self.features, self.layout, self.n_rows, self.prog_off,
                      self.prog_score, self.row_score, self.leaf_idx)

    def topk_request(self) -> TopkRequest:
        return TopkRequest(self.prog_score, self.n_programs, self.k, self.topk_idx, self.topk_score)


# ---- training (familyseer_train.h) -------------------------------------------------------------

FS_TRAIN_MAX_DEPTH = 10
FS_TRAIN_MAX_CUTS = 255


class _FsTrainParams(ctypes.Structure):
    _fields_ = [("max_depth", ctypes.c_int32), ("eta", ctypes.c_float), ("lam", ctypes.c_float),
                ("min_gain", ctypes.c_float), ("min_child_weight", ctypes.c_float),
                ("grad_scale", ctypes.c_float)]


_lib.fs_trainer_create.restype = ctypes.c_int
_lib.fs_trainer_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32, ctypes.c_void_p,
                                   ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int32,
                                   ctypes.c_void_p, _i32p, _f32p, ctypes.c_float, ctypes.c_int32,
                                   ctypes.c_int32, ctypes.c_void_p]
_lib.fs_trainer_destroy.restype = None
_lib.fs_trainer_destroy.argtypes = [ctypes.c_void_p]
_lib.fs_train_boost.restype = ctypes.c_int
_lib.fs_train_boost.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32,
                                ctypes.POINTER(_FsTrainParams), ctypes.c_void_p]
_lib.fs_trainer_size.restype = ctypes.c_int
_lib.fs_trainer_size.argtypes = [ctypes.c_void_p, _i32p, ctypes.POINTER(ctypes.c_int64), ctypes.c_void_p]
_lib.fs_trainer_export.restype = ctypes.c_int
_lib.fs_trainer_export.argtypes = [ctypes.c_void_p, _i32p, _i32p, _f32p, _i32p, _i32p, _f32p,
                                   ctypes.c_void_p]
_lib.fs_trainer_predictions.restype = ctypes.c_int
_lib.fs_trainer_predictions.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]


def train_params(max_depth: int = 6, eta: float = 0.3, lam: float = 1.0, min_gain: float = 0.0,
                 min_child_weight: float = 1.0, grad_scale: float = float(1 << 20)) -> _FsTrainParams:
    return _FsTrainParams(max_depth, eta, lam, min_gain, min_child_weight, grad_scale)


class fs_trainer:
    """Owner of one `fs_trainer*`: a family's measured programs, binned, and the model so far."""

    def __init__(self, n_features: int, features: torch.Tensor, layout: int, n_rows: int,
                 prog_off: torch.Tensor, n_programs: int, target: torch.Tensor, cut_off, cuts,
                 bias: float = 0.0, max_depth: int = 6, max_trees: int = 64,
                 stream: Optional[torch.cuda.Stream] = None):
        co = np.ascontiguousarray(cut_off, dtype=np.int32)
        cu = np.ascontiguousarray(cuts, dtype=np.float32)
        if cu.size == 0:
            cu = np.zeros(1, np.float32)
        self.handle = ctypes.c_void_p()
        self.n_features, self.n_rows, self.n_programs, self.bias = n_features, n_rows, n_programs, bias
        _check(_lib.fs_trainer_create(ctypes.byref(self.handle), n_features, _ptr(features), layout,
                                      n_rows, _ptr(prog_off), n_programs, _ptr(target),
                                      co.ctypes.data_as(_i32p), cu.ctypes.data_as(_f32p), bias,
                                      max_depth, max_trees, _stream_ptr(stream)))

    @classmethod
    def from_train_set(cls, ts, layout: int = FS_COLBLOCK64, device: str = "cuda:0", **kw):
        dev = torch.device(device)
        x = torch.from_numpy(np.ascontiguousarray(ts.features)).to(dev)
        if layout == FS_COLBLOCK64:
            x = fs_pack_colblock64(x, ts.n_rows, ts.features.shape[1])
        off = torch.from_numpy(np.ascontiguousarray(ts.prog_off, dtype=np.int32)).to(dev)
        y = torch.from_numpy(np.ascontiguousarray(ts.target, dtype=np.float32)).to(dev)
        t = cls(ts.features.shape[1], x, layout, ts.n_rows, off, ts.n_programs, y, ts.cut_off,
                ts.cuts, **kw)
        torch.cuda.synchronize()          # the inputs may be freed once they are binned
        return t

    def size(self, stream: Optional[torch.cuda.Stream] = None):
        nt, nn = ctypes.c_int32(), ctypes.c_int64()
        _check(_lib.fs_trainer_size(self.handle, ctypes.byref(nt), ctypes.byref(nn), _stream_ptr(stream)))
        return int(nt.value), int(nn.value)

    def export(self, stream: Optional[torch.cuda.Stream] = None):
        """(tree_off, split_feature, threshold, left, right, value) as numpy arrays."""
        nt, nn = self.size(stream)
        to = np.zeros(nt + 1, np.int32)
        sf, le, ri = (np.zeros(max(1, nn), np.int32) for _ in range(3))
        th, va = (np.zeros(max(1, nn), np.float32) for _ in range(2))
        _check(_lib.fs_trainer_export(self.handle, to.ctypes.data_as(_i32p), sf.ctypes.data_as(_i32p),
                                      th.ctypes.data_as(_f32p), le.ctypes.data_as(_i32p),
                                      ri.ctypes.data_as(_i32p), va.ctypes.data_as(_f32p),
                                      _stream_ptr(stream)))
        return to, sf[:nn], th[:nn], le[:nn], ri[:nn], va[:nn]

    def predictions(self, stream: Optional[torch.cuda.Stream] = None):
        rows = torch.empty(self.n_rows, dtype=torch.float32, device="cuda")
        progs = torch.empty(self.n_programs, dtype=torch.float32, device="cuda")
        _check(_lib.fs_trainer_predictions(self.handle, _ptr(rows), _ptr(progs), _stream_ptr(stream)))
        return rows, progs

    def destroy(self) -> None:
        if self.handle:
            _lib.fs_trainer_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def fs_train_boost(trainers, n_rounds: int, params: _FsTrainParams,
                   stream: Optional[torch.cuda.Stream] = None) -> None:
    arr = (ctypes.c_void_p * max(1, len(trainers)))(*[t.handle for t in trainers])
    _check(_lib.fs_train_boost(len(trainers), arr, n_rounds, ctypes.byref(params), _stream_ptr(stream)))


# ---- population compaction ----------------------------------------------------------------------

class _FsGatherSrc(ctypes.Structure):
    _fields_ = [("features", ctypes.c_void_p), ("prog_off", ctypes.c_void_p),
                ("score", ctypes.c_void_p), ("n_programs", ctypes.c_int32)]


_lib.fs_gather_programs.restype = ctypes.c_int
_lib.fs_gather_programs.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(_FsGatherSrc),
                                    ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]


def fs_gather_programs(n_features: int, sources, keep: torch.Tensor, n_keep: int,
                       out_features: torch.Tensor, out_row_capacity: int,
                       out_prog_off: torch.Tensor, out_score: Optional[torch.Tensor],
                       status: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """`sources`: sequence of (features, prog_off, score-or-None, n_programs) device tensors."""
    arr = (_FsGatherSrc * max(1, len(sources)))()
    for i, (x, off, sc, n) in enumerate(sources):
        arr[i] = _FsGatherSrc(_ptr(x), _ptr(off), _ptr(sc), n)
    _check(_lib.fs_gather_programs(n_features, len(sources), arr, _ptr(keep), n_keep,
                                   _ptr(out_features), out_row_capacity, _ptr(out_prog_off),
                                   _ptr(out_score), _ptr(status), _stream_ptr(stream)))


def unpack_colblock64(x: torch.Tensor, n_rows: int, n_features: int) -> np.ndarray:
    """Host copy of an FS_COLBLOCK64 buffer as a row-major [n_rows, n_features] array (tests)."""
    tiles = (n_rows + 63) // 64
    a = x[: tiles * n_features * 64].cpu().numpy().reshape(tiles, n_features, 64)
    return np.ascontiguousarray(a.transpose(0, 2, 1).reshape(tiles * 64, n_features)[:n_rows])
