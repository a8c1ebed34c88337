"""ctypes binding of the plain-C CPU oracle (oracle/rps_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg; never by the HIP library or its Python binding.
Every function only marshals numpy arrays; the arithmetic is all in the C file,
whose comments cite the passages of arXiv 1810.07766 it follows.

Arrays: X, V, G are numpy [n, m], C-contiguous, float32 (dtype code 0) or
uint16 holding bf16 bit patterns (dtype code 1).  Masks are uint8 [n, n]
indexed [worker, block]; server is int32 [n].
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = ctypes.CDLL(_build.build(force=False))

_u8p = ctypes.POINTER(ctypes.c_uint8)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)

_lib.rps_oracle_philox4x32.argtypes = [ctypes.c_uint32, _u32p, _u32p, _u32p]
_lib.rps_oracle_philox4x32.restype = None
_lib.rps_oracle_masks.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                  ctypes.c_int32, _i32p, _u8p, _u8p]
_lib.rps_oracle_masks.restype = None
_lib.rps_oracle_noise_patch.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32, ctypes.c_uint64,
                                        ctypes.c_float, _f32p]
_lib.rps_oracle_noise_patch.restype = None
_lib.rps_oracle_noise.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int64, ctypes.c_float]
_lib.rps_oracle_noise.restype = ctypes.c_float
_lib.rps_oracle_noise_radius.argtypes = [ctypes.c_uint32]
_lib.rps_oracle_noise_radius.restype = ctypes.c_float
_lib.rps_oracle_noise_direction.argtypes = [ctypes.c_uint32, _f32p, _f32p]
_lib.rps_oracle_noise_direction.restype = None
_lib.rps_oracle_local_step.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64,
                                       _i64p, ctypes.c_int32, ctypes.c_float, ctypes.c_float,
                                       ctypes.c_float, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32]
_lib.rps_oracle_local_step.restype = None
_lib.rps_oracle_lossy_average.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, _i64p, ctypes.c_int32,
                                          _i64p, _u8p, _u8p, ctypes.c_int32, ctypes.c_int32]
_lib.rps_oracle_lossy_average.restype = None
_lib.rps_oracle_build_W.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _u8p, _u8p, _f64p]
_lib.rps_oracle_build_W.restype = None
_lib.rps_oracle_max_threads.argtypes = []
_lib.rps_oracle_max_threads.restype = ctypes.c_int32


def max_threads() -> int:
    return int(_lib.rps_oracle_max_threads())


def philox4x32(ctr, key, rounds: int = 10) -> np.ndarray:
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    _lib.rps_oracle_philox4x32(rounds, c.ctypes.data_as(_u32p), k.ctypes.data_as(_u32p),
                               out.ctypes.data_as(_u32p))
    return out


def masks(seed: int, step: int, n: int, p: float, identity_server: bool = False, external_servers: int = 0):
    """(server[nb] int32, U[n,nb] uint8, D[n,nb] uint8) of one round.  nb = n blocks served by the
    workers themselves, or `external_servers` blocks served by parameter servers that are not
    workers (server = -1, no reliable self link)."""
    assert 1 <= n <= 64 and 0.0 <= p <= 1.0 and 0 <= step < (1 << 56) and 0 <= external_servers <= 64
    nb = external_servers if external_servers else n
    mode = 2 if external_servers else (1 if identity_server else 0)
    server = np.empty(nb, dtype=np.int32)
    U = np.empty((n, nb), dtype=np.uint8)
    D = np.empty((n, nb), dtype=np.uint8)
    _lib.rps_oracle_masks(seed, step, n, nb, p, mode, server.ctypes.data_as(_i32p),
                          U.ctypes.data_as(_u8p), D.ctypes.data_as(_u8p))
    return server, U, D


def noise_patch(seed: int, step: int, pair: int, quad: int, sigma: float = 1.0) -> np.ndarray:
    """[2, 4] float32: sigma*z for workers (2*pair, 2*pair+1) x columns 4*quad..4*quad+3."""
    out = np.empty(8, dtype=np.float32)
    _lib.rps_oracle_noise_patch(seed, step, pair, quad, sigma, out.ctypes.data_as(_f32p))
    return out.reshape(2, 4)


def noise_grid():
    """(radius[4096], cos[4096], sin[4096]) float32: the cell values of the noise specification."""
    r = np.array([_lib.rps_oracle_noise_radius(k) for k in range(4096)], dtype=np.float32)
    c = np.empty(4096, dtype=np.float32)
    s = np.empty(4096, dtype=np.float32)
    cc, ss = ctypes.c_float(), ctypes.c_float()
    for a in range(4096):
        _lib.rps_oracle_noise_direction(a, ctypes.byref(cc), ctypes.byref(ss))
        c[a], s[a] = cc.value, ss.value
    return r, c, s


def noise(seed: int, step: int, worker: int, column: int, sigma: float = 1.0) -> float:
    return float(_lib.rps_oracle_noise(seed, step, worker, column, sigma))


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError("oracle arrays are float32 or uint16 (bf16 bits)")


def _cols_ptr(cols, m):
    if cols is None:
        return None, None
    c = np.ascontiguousarray(cols, dtype=np.int64)
    assert c.shape == (m,)
    return c, c.ctypes.data_as(_i64p)


def local_step(X: np.ndarray, G, gamma: float, *, sigma: float = 0.0, weight_decay: float = 0.0,
               seed: int = 0, step: int = 0, cols=None, threads: int = 1) -> None:
    """In place X <- X - gamma*G, or with G=None the synthetic gradient
    weight_decay*x + sigma*z (z from the counter-based noise of (seed, step))."""
    assert X.ndim == 2 and X.flags.c_contiguous
    n, m = X.shape
    code = _dtype_code(X)
    gp = None
    if G is not None:
        assert G.shape == X.shape and G.dtype == X.dtype and G.flags.c_contiguous
        gp = G.ctypes.data
    keep, cp = _cols_ptr(cols, m)
    _lib.rps_oracle_local_step(X.ctypes.data, gp, n, m, cp, code, gamma, sigma, weight_decay,
                               seed, step, threads)


def lossy_average(V: np.ndarray, offsets, U: np.ndarray, D: np.ndarray, *, cols=None,
                  threads: int = 1) -> None:
    """In place RS + AG round on V with the given delivery masks ([n, nb]; nb = len(offsets) - 1)."""
    assert V.ndim == 2 and V.flags.c_contiguous
    n, m = V.shape
    off = np.ascontiguousarray(offsets, dtype=np.int64)
    nb = off.shape[0] - 1
    U = np.ascontiguousarray(U, dtype=np.uint8)
    D = np.ascontiguousarray(D, dtype=np.uint8)
    assert U.shape == (n, nb) and D.shape == (n, nb)
    keep, cp = _cols_ptr(cols, m)
    _lib.rps_oracle_lossy_average(V.ctypes.data, n, m, cp, nb, off.ctypes.data_as(_i64p),
                                  U.ctypes.data_as(_u8p), D.ctypes.data_as(_u8p), _dtype_code(V), threads)


def build_W(j: int, U: np.ndarray, D: np.ndarray) -> np.ndarray:
    """Mixing matrix W of block j: X_next^(j) = V^(j) W, W[m, k] = weight of worker m in worker k."""
    U = np.ascontiguousarray(U, dtype=np.uint8)
    D = np.ascontiguousarray(D, dtype=np.uint8)
    n, nb = U.shape
    W = np.empty((n, n), dtype=np.float64)
    _lib.rps_oracle_build_W(n, nb, j, U.ctypes.data_as(_u8p), D.ctypes.data_as(_u8p), W.ctypes.data_as(_f64p))
    return W


def equal_offsets(n: int, N: int) -> np.ndarray:
    """The paper's equally-sized blocks: N must divide by n."""
    assert N % n == 0
    return np.arange(n + 1, dtype=np.int64) * (N // n)


def round_(X: np.ndarray, G, offsets, *, p: float, gamma: float, seed: int, step: int,
           sigma: float = 0.0, weight_decay: float = 0.0, identity_server: bool = False,
           external_servers: int = 0, mask_override=None, cols=None, threads: int = 1):
    """One full RPS round in the order of Alg. 1: local step, then RS, then AG.
    Returns the masks used."""
    n = X.shape[0]
    local_step(X, G, gamma, sigma=sigma, weight_decay=weight_decay, seed=seed, step=step,
               cols=cols, threads=threads)
    if mask_override is not None:
        server, U, D = mask_override
    else:
        server, U, D = masks(seed, step, n, p, identity_server, external_servers)
    lossy_average(X, offsets, U, D, cols=cols, threads=threads)
    return server, U, D


def consensus(X: np.ndarray):
    """(sum_i ||x_i - xbar||^2, ||xbar||^2) by the plain definition in float64: the disagreement
    ||X (I - A_n)||_F^2 of the supplement's Lemma 1 (rows of X are the workers)."""
    Xd = (X.astype(np.uint32) << 16).view(np.float32).astype(np.float64) if X.dtype == np.uint16 else X.astype(np.float64)
    xbar = Xd.mean(axis=0)
    return float(((Xd - xbar[None, :]) ** 2).sum()), float((xbar ** 2).sum())


def round_gradient_averaging(X: np.ndarray, G: np.ndarray, offsets, *, p: float, gamma: float, seed: int,
                             step: int, identity_server: bool = False, mask_override=None, cols=None,
                             threads: int = 1):
    """The paper's gradient-averaging comparison (Sec. 6): the lossy Reduce-Scatter / All-Gather
    is applied to the gradients, then each worker takes its local step with what it holds.
    Literally the composition of the two oracle steps: lossy_average on a copy of G, then
    local_step with that.  Returns the masks used."""
    n = X.shape[0]
    if mask_override is not None:
        server, U, D = mask_override
    else:
        server, U, D = masks(seed, step, n, p, identity_server)
    Gh = G.copy()
    lossy_average(Gh, offsets, U, D, cols=cols, threads=threads)
    local_step(X, Gh, gamma, threads=threads)
    return server, U, D


def estimate_mixing(seed: int, first_step: int, rounds: int, n: int, p: float, *, identity_server: bool = False,
                    external_servers: int = 0):
    """Monte-Carlo (alpha1, alpha2) by the definitions of Sec. 4.2: average W W^T and W A_n W^T over
    every block's mixing matrix of the outcomes generated for `rounds` steps, then read the constants
    off the diagonal of  a I + (1 - a) A_n  (mean diagonal entry = a + (1 - a)/n)."""
    A = np.full((n, n), 1.0 / n)
    WW = np.zeros((n, n)); WAW = np.zeros((n, n)); samples = 0
    for t in range(first_step, first_step + rounds):
        _, U, D = masks(seed, t, n, p, identity_server, external_servers)
        for j in range(U.shape[1]):
            W = build_W(j, U, D)
            WW += W @ W.T; WAW += W @ A @ W.T; samples += 1
    a1 = (n * np.trace(WW / samples) / n - 1.0) / (n - 1.0)
    a2 = (n * np.trace(WAW / samples) / n - 1.0) / (n - 1.0)
    return float(a1), float(a2)
