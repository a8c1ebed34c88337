"""The C-ABI library loads and exports every symbol include/rps.h declares (no compute calls:
this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1810_07766_amd", "librps.so")


def _ensure_built():
    if not os.path.exists(LIB):
        from paper_1810_07766_amd import build
        build.build()


def test_library_exports_every_declared_symbol():
    _ensure_built()
    header = open(os.path.join(ROOT, "include", "rps.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(rps_[a-z_]+)\s*\(", header))
    assert {"rps_create", "rps_local_step", "rps_lossy_average", "rps_round", "rps_destroy"} <= declared
    lib = ctypes.CDLL(LIB)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in rps.h but not exported"


def test_binding_mirrors_the_header():
    _ensure_built()
    from paper_1810_07766_amd import rps
    header = open(os.path.join(ROOT, "include", "rps.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(rps_[a-z_]+)\s*\(", header))
    assert declared == set(rps.EXPORTS)


def test_argument_validation_needs_no_gpu():
    _ensure_built()
    lib = ctypes.CDLL(LIB)
    lib.rps_strerror.restype = ctypes.c_char_p
    ctx = ctypes.c_void_p()
    args = lambda n, N, p: (ctypes.byref(ctx), n, ctypes.c_int64(N), None, ctypes.c_double(p), ctypes.c_float(0.1),
                            ctypes.c_uint64(0), 0, 0, None)
    assert lib.rps_create(*args(0, 100, 0.1)) == -1
    assert lib.rps_create(*args(4, 101, 0.1)) == -1          # equal blocks need N % n == 0
    assert lib.rps_create(*args(4, 100, -0.5)) == -1
    assert lib.rps_create(*args(4, 100, float("nan"))) == -1
    assert lib.rps_destroy(None) == 0
    assert lib.rps_strerror(-1) == b"invalid argument"
    assert ctx.value is None
