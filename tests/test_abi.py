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


def test_header_is_plain_c(tmp_path):
    """include/rps.h compiles as C99 and as C++ on its own (no HIP or torch types in the signatures),
    and a C translation unit that names every entry point links against the library."""
    import subprocess
    _ensure_built()
    inc = os.path.join(ROOT, "include")
    header = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, "rps.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(rps_[a-z_]+)\s*\(", header)))
    src = tmp_path / "use_rps.c"
    src.write_text('#include "rps.h"\n#include <stdio.h>\ntypedef void (*fn)(void);\nint main(void) {\n  fn f[] = {'
                   + ", ".join(f"(fn){n}" for n in names)
                   + "};\n  printf(\"%d %s\\n\", (int)(sizeof f / sizeof f[0]), rps_strerror(RPS_EINVAL));\n"
                     "  return rps_destroy(0);\n}\n")
    exe = tmp_path / "use_rps"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe),
                    "-L", os.path.dirname(LIB), "-l:librps.so", f"-Wl,-rpath,{os.path.dirname(LIB)}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(None, 1)
    assert int(out[0]) == len(names) and out[1].strip() == "invalid argument"
    subprocess.run(["g++", "-std=c++17", "-fsyntax-only", "-x", "c++", "-I", inc, os.path.join(inc, "rps.h")], check=True)


def test_tile_major_index_formula():
    """workloads.to_tiled / from_tiled (the re-arrangement the tests hand to the library) against the
    index formula of include/rps.h: element (i, c) lives at ((c / T) * n + i) * T + c % T."""
    import numpy as np
    import torch
    import workloads
    for n, N, dt in ((3, 100, torch.float32), (5, 64, torch.float32), (2, 130, torch.bfloat16)):
        X = torch.arange(n * N, dtype=torch.float32).reshape(n, N).to(dt)
        Xt = workloads.to_tiled(X)
        T = workloads.TILE_BYTES // X.element_size()
        assert tuple(Xt.shape) == ((N + T - 1) // T, n, T)
        flat = Xt.reshape(-1)
        for i, c in ((0, 0), (n - 1, N - 1), (1, T), (n - 1, T - 1), (0, N // 2)):
            assert flat[((c // T) * n + i) * T + c % T] == X[i, c]
        assert torch.equal(workloads.from_tiled(Xt, N), X)
        if N % T:
            assert float(Xt[-1, :, N % T:].abs().sum()) == 0.0      # zero padding
    assert workloads.TILE_BYTES == 128


def test_constants_agree_with_the_header():
    _ensure_built()
    import workloads
    from paper_1810_07766_amd import rps
    header = open(os.path.join(ROOT, "include", "rps.h")).read()
    assert int(re.search(r"#define RPS_TILE_BYTES (\d+)", header).group(1)) == rps.RPS_TILE_BYTES == workloads.TILE_BYTES
    enums = dict(re.findall(r"(RPS_[A-Z0-9_]+)\s*=\s*(-?\d+)u?", header))
    for name, value in enums.items():
        assert getattr(rps, name) == int(value), name
    lib = ctypes.CDLL(LIB)
    lib.rps_storage_elems.restype = ctypes.c_int64
    lib.rps_storage_elems.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32]
    assert lib.rps_storage_elems(4, 1000, 0, 0) == 4000
    assert lib.rps_storage_elems(4, 1000, 0, rps.RPS_FLAG_LAYOUT_TILED) == 32 * 4 * 32
    assert lib.rps_storage_elems(65, 1000, 0, 0) == -1


def test_noise_cells_of_the_library_equal_the_oracle():
    """The library computes the cell values of the synthetic gradient noise on the host in 80-bit
    arithmetic, the oracle evaluates the same real values in double: both must land on the same
    (correctly rounded) fp32 bits, or the device's noise could not match the oracle's."""
    _ensure_built()
    import numpy as np
    from oracle import rps_oracle as oracle
    from paper_1810_07766_amd import rps
    radius, cos_sin = rps.rps_noise_cells()
    r, c, s = oracle.noise_grid()
    assert (radius.view(np.uint32) == r.view(np.uint32)).all()
    assert (cos_sin[:, 0].view(np.uint32) == c.view(np.uint32)).all()
    assert (cos_sin[:, 1].view(np.uint32) == s.view(np.uint32)).all()


def test_host_copy_of_the_mask_generator_equals_the_oracle():
    """rps_masks_host (the library's own host implementation of the network-outcome generator: Sec. 3
    drops, Alg. 1 step 6 permutation) against the oracle, bit for bit, without a GPU: worker counts
    1..64, both server rules, external servers, the extreme drop rates and the largest steps."""
    import numpy as np
    _ensure_built()
    from oracle import rps_oracle as oracle
    from paper_1810_07766_amd import rps
    rng = np.random.default_rng(7)
    steps = [0, 1, 2, 2 ** 32 - 1, 2 ** 32, 2 ** 40 + 7, 2 ** 56 - 1]
    for n in list(range(1, 9)) + [15, 16, 17, 31, 32, 33, 63, 64]:
        for p in (0.0, 0.01, 0.3, 1.0):
            seed = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
            for step in steps + [int(rng.integers(0, 2 ** 56))]:
                for identity in (False, True):
                    s_h, u_h, d_h = rps.rps_masks_host(n, p, seed, step, flags=rps.RPS_FLAG_SERVER_IDENTITY if identity else 0)
                    s_o, u_o, d_o = oracle.masks(seed, step, n, p, identity)
                    assert (s_h == s_o).all() and (u_h == u_o).all() and (d_h == d_o).all(), (n, p, seed, step, identity)
            for servers in (1, 3, 64):
                s_h, u_h, d_h = rps.rps_masks_host(n, p, seed, 5, servers=servers)
                s_o, u_o, d_o = oracle.masks(seed, 5, n, p, external_servers=servers)
                assert (s_h == s_o).all() and (u_h == u_o).all() and (d_h == d_o).all(), (n, p, seed, servers)
    # argument errors
    for bad in (dict(n=0), dict(n=65), dict(p=-0.1), dict(p=float("nan")), dict(step=2 ** 56), dict(flags=8),
                dict(servers=65), dict(servers=3, flags=1)):
        kw = dict(n=4, p=0.1, seed=0, step=0, flags=0, servers=0)
        kw.update(bad)
        try:
            rps.rps_masks_host(**kw)
        except rps.RpsError as e:
            assert e.code == rps.RPS_EINVAL
        else:
            raise AssertionError(f"accepted {bad}")


def test_launch_shape_sweep_grid_is_within_the_tuning_interface():
    """The sweep utility imports without a GPU and only proposes shapes that rps_set_launch_tuning
    accepts (rows per chunk 2 or 4, 1..16 wavefronts per workgroup, cap >= 0, 0..64 steps)."""
    from paper_1810_07766_amd import sweep_launch_shapes as sweep
    for tiled in (True, False):
        for n in (1, 2, 8, 32, 33, 64):
            for what in ("round, in-register gradient", "averaging alone", "round, gradient buffer", "gradient averaging"):
                grid = sweep._grid(what, n, tiled)
                assert len(grid) >= 5 and len(set(grid)) == len(grid)
                for rows, wpb, cap, steps in grid:
                    assert rows in (2, 4) and 1 <= wpb <= 16 and 0 <= cap <= 64 and 0 <= steps <= 64
