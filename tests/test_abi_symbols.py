"""The C-ABI library loads without a GPU and exports every function the header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in ("familyseer.h", "familyseer_train.h")]
LIB = os.path.join(ROOT, "paper_2201_00194_amd", "libfamilyseer.so")


def declared_functions():
    names = []
    for header in HEADERS:
        src = open(header).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names += re.findall(r"\b(fs_[a-z0-9_]+)\s*\(", src)
    return sorted(set(names))


def test_header_declares_the_named_entry_points():
    names = declared_functions()
    for must in ("fs_score_families", "fs_topk", "fs_model_create", "fs_model_destroy",
                 "fs_pack_colblock64", "fs_last_error", "fs_version", "fs_trainer_create",
                 "fs_train_boost", "fs_trainer_export", "fs_trainer_predictions",
                 "fs_trainer_size", "fs_trainer_destroy"):
        assert must in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        from paper_2201_00194_amd import build
        build.build()
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in include/*.h but not exported"
    lib.fs_version.restype = ctypes.c_int
    assert lib.fs_version() >= 100
    lib.fs_last_error.restype = ctypes.c_char_p
    assert lib.fs_last_error() is not None


def test_tuning_options_of_header_binding_and_library_agree():
    """The FS_TUNE_* options are numbered once, in familyseer.h; the Python binding repeats the
    numbers and the library accepts exactly that many (no GPU needed: fs_tune_set only stores)."""
    src = re.sub(r"/\*.*?\*/", "", open(HEADERS[0]).read(), flags=re.S)
    enum = dict((k, int(v)) for k, v in re.findall(r"\b(FS_TUNE_[A-Z_]+)\s*=\s*(\d+)", src))
    n = enum.pop("FS_TUNE_OPTIONS")
    assert sorted(enum.values()) == list(range(n))
    api_src = open(os.path.join(ROOT, "paper_2201_00194_amd", "api.py")).read()
    m = re.search(r"\(((?:\s*FS_TUNE_[A-Z_]+,?)+)\)\s*=\s*range\((\d+)\)", api_src)
    assert m, "api.py no longer lists the options as one range"
    names = re.findall(r"FS_TUNE_[A-Z_]+", m.group(1))
    assert int(m.group(2)) == n and names == sorted(enum, key=enum.get)
    if not os.path.exists(LIB):
        from paper_2201_00194_amd import build
        build.build()
    lib = ctypes.CDLL(LIB)
    lib.fs_tune_set.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.fs_tune_get.argtypes = [ctypes.c_int32]
    lib.fs_tune_get.restype = ctypes.c_int32
    for opt in range(n):
        assert lib.fs_tune_get(opt) == -1                 # automatic choice
        assert lib.fs_tune_set(opt, 3) == 0 and lib.fs_tune_get(opt) == 3
        assert lib.fs_tune_set(opt, -1) == 0 and lib.fs_tune_get(opt) == -1
    assert lib.fs_tune_set(n, 1) != 0 and lib.fs_tune_set(-1, 1) != 0


def test_host_side_validation_needs_no_gpu():
    """Argument errors are found on the host before any device work."""
    if not os.path.exists(LIB):
        from paper_2201_00194_amd import build
        build.build()
    lib = ctypes.CDLL(LIB)
    lib.fs_last_error.restype = ctypes.c_char_p
    lib.fs_colblock64_floats.restype = ctypes.c_int64
    lib.fs_colblock64_floats.argtypes = [ctypes.c_int64, ctypes.c_int32]
    assert lib.fs_colblock64_floats(65, 164) == 2 * 64 * 164
    assert lib.fs_colblock64_floats(0, 164) == 0
    assert lib.fs_score_families(-1, None, None) == -1
    assert b"negative" in lib.fs_last_error()
    assert lib.fs_score_families(0, None, None) == 0
    assert lib.fs_topk(3, None, None) == -1
    assert lib.fs_topk(0, None, None) == 0
    h = ctypes.c_void_p()
    i32 = ctypes.c_int32
    off = (i32 * 2)(0, 1)
    sf = (i32 * 1)(-1)
    z = (ctypes.c_float * 1)(0.0)
    ch = (i32 * 1)(-1)
    lib.fs_model_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), i32, i32] + [ctypes.c_void_p] * 6 + [ctypes.c_float]
    assert lib.fs_model_create(ctypes.byref(h), 0, 1, off, sf, z, ch, ch, z, 0.0) == -1
    assert lib.fs_model_create(None, 4, 1, off, sf, z, ch, ch, z, 0.0) == -1
    bad_off = (i32 * 2)(1, 2)
    assert lib.fs_model_create(ctypes.byref(h), 4, 1, bad_off, sf, z, ch, ch, z, 0.0) == -1
    # internal node whose child id does not exceed its own: rejected (would allow cycles)
    off3 = (i32 * 2)(0, 3)
    sf3 = (i32 * 3)(0, -1, -1)
    l3 = (i32 * 3)(0, -1, -1)
    r3 = (i32 * 3)(2, -1, -1)
    z3 = (ctypes.c_float * 3)(0.0, 0.0, 0.0)
    assert lib.fs_model_create(ctypes.byref(h), 4, 1, off3, sf3, z3, l3, r3, z3, 0.0) == -1
    assert b"child" in lib.fs_last_error()
    sf3b = (i32 * 3)(9, -1, -1)
    l3b = (i32 * 3)(1, -1, -1)
    assert lib.fs_model_create(ctypes.byref(h), 4, 1, off3, sf3b, z3, l3b, r3, z3, 0.0) == -1
    assert b"feature" in lib.fs_last_error()


def test_trainer_argument_errors_need_no_gpu():
    """fs_trainer_create / fs_train_boost reject bad arguments before touching the device."""
    if not os.path.exists(LIB):
        from paper_2201_00194_amd import build
        build.build()
    lib = ctypes.CDLL(LIB)
    lib.fs_last_error.restype = ctypes.c_char_p
    i32p, f32p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)
    lib.fs_trainer_create.restype = ctypes.c_int
    lib.fs_trainer_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32, ctypes.c_void_p,
                                      ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int32,
                                      ctypes.c_void_p, i32p, f32p, ctypes.c_float, ctypes.c_int32,
                                      ctypes.c_int32, ctypes.c_void_p]
    out = ctypes.c_void_p()
    cut_off = (ctypes.c_int32 * 3)(0, 2, 3)
    cuts = (ctypes.c_float * 3)(0.5, 0.25, 1.0)               # feature 0: not ascending
    fake = ctypes.c_void_p(4096)                              # never dereferenced on these paths

    def create(nf=2, rows=10, progs=5, co=cut_off, cu=cuts, depth=3, trees=4, layout=1):
        return lib.fs_trainer_create(ctypes.byref(out), nf, fake, layout, rows, fake, progs, fake,
                                     co, cu, 0.0, depth, trees, None)

    assert create() == -1 and b"ascending" in lib.fs_last_error()
    good = (ctypes.c_float * 3)(0.25, 0.5, 1.0)
    assert create(cu=good, nf=0) == -1
    assert create(cu=good, rows=0) == -1
    assert create(cu=good, depth=11) == -4                    # FS_EUNSUPPORTED
    assert create(cu=good, trees=0) == -1
    assert create(cu=good, layout=7) == -1
    assert out.value is None
    lib.fs_train_boost.restype = ctypes.c_int
    lib.fs_train_boost.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p,
                                   ctypes.c_void_p]
    assert lib.fs_train_boost(-1, None, 1, None, None) == -1


def test_headers_compile_as_c99_and_link(tmp_path):
    """The installed headers are plain C: a C99 program that includes both, fills the structs
    and calls argument-checking paths builds with -pedantic -Werror and runs without a GPU."""
    import subprocess
    if not os.path.exists(LIB):
        from paper_2201_00194_amd import build
        build.build()
    src = tmp_path / "abi.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "familyseer.h"
#include "familyseer_train.h"
int main(void) {
    fs_family fam;
    fs_topk_req req;
    fs_gather_src gs;
    fs_train_params tp;
    memset(&fam, 0, sizeof fam); memset(&req, 0, sizeof req); memset(&gs, 0, sizeof gs);
    memset(&tp, 0, sizeof tp);
    if (fs_version() < 100) return 1;
    if (fs_score_families(-1, &fam, NULL) != FS_EINVAL) return 2;
    if (strlen(fs_last_error()) == 0) return 3;
    req.k = FS_MAX_TOPK + 1;
    if (fs_topk(1, &req, NULL) != FS_EUNSUPPORTED) return 4;
    if (fs_colblock64_floats(65, 3) != 2 * 3 * 64) return 5;
    if (fs_train_boost(-1, NULL, 1, &tp, NULL) != FS_EINVAL) return 6;
    if (fs_gather_programs(0, 1, &gs, NULL, 0, NULL, 0, NULL, NULL, NULL, NULL) != FS_EINVAL) return 7;
    printf("ok %d %d\n", FS_TRAIN_MAX_DEPTH, FS_KERNEL_CLASSES);
    return 0;
}
''')
    exe = tmp_path / "abi"
    libdir = os.path.dirname(LIB)
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                    "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-lfamilyseer", "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert out.startswith("ok 10 10")
