"""The allocation-free entry point rps_consensus_static (for callers that cannot call hipMalloc:
code under HIP graph capture, tight serving loops) against rps_consensus, through the C ABI.

Both run the same kernels in the same fixed reduction order, so the two results must be the same
bits; rps_consensus itself is checked against the oracle's float64 definition here as well.  Two
calls in a row share the GPU's static scratch, the second on a smaller input: stale partial sums
of the first call must not leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

import workloads
from oracle import rps_oracle as oracle
from gpu_common import device_tensor, to_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rps():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1810_07766_amd import rps as mod
    return mod


def _static(rps, X, n, N, dtype, flags, out):
    rps.rps_consensus_static(X, n, N, out, dtype=rps.RPS_DTYPE_BF16 if dtype == "bf16" else rps.RPS_DTYPE_F32, flags=flags)


@pytest.mark.parametrize("dtype,tiled", [("f32", False), ("f32", True), ("bf16", False), ("bf16", True)])
def test_static_consensus_matches_the_context_entry_point(rps, dtype, tiled):
    flags = rps.RPS_FLAG_LAYOUT_TILED if tiled else 0
    dt = rps.RPS_DTYPE_BF16 if dtype == "bf16" else rps.RPS_DTYPE_F32
    out = torch.full((2,), -1.0, device="cuda", dtype=torch.float64)
    # the first input spans more workgroups than the static scratch holds partials for (grid-stride),
    # the second is much smaller and ragged: fewer partials are written and read
    for n, N in ((24, 24 * 110_000), (7, 7001)):
        X0 = workloads.gaussian_model(n, N, seed=n + N)
        X0 = (0.5 + X0[0:1]) + 1e-3 * X0                     # workers nearly agree: the pivoted sums must not cancel
        Xr = device_tensor(X0, dtype)
        X = workloads.to_tiled(Xr) if tiled else Xr
        ctx = rps.RpsContext(n, N, 0.1, 0.1, 0, dt, block_offsets=workloads.block_offsets(n, N) if N % n == 0 else
                             np.linspace(0, N, n + 1).astype(np.int64), flags=flags)
        d_ctx, m_ctx = ctx.consensus(X)
        before = X.clone()
        _static(rps, X, n, N, dtype, flags, out)
        torch.cuda.synchronize()
        d, m = out.tolist()
        assert (d, m) == (d_ctx, m_ctx), f"n={n} N={N}: static {d, m} != context {d_ctx, m_ctx}"
        assert torch.equal(X, before)                         # read only
        d_ref, m_ref = oracle.consensus(to_oracle(Xr))
        assert abs(m - m_ref) <= 1e-11 * m_ref
        assert abs(d - d_ref) <= 1e-9 * d_ref + 1e-18 * m_ref * n
        ctx.destroy()


def test_static_consensus_needs_no_context_and_orders_on_the_stream(rps):
    """Called before any context exists on a side stream, twice back to back into two outputs."""
    n, N = 5, 5 * 3000
    s = torch.cuda.Stream()
    Xa = device_tensor(workloads.gaussian_model(n, N, seed=1), "f32")
    Xb = device_tensor(workloads.gaussian_model(3, 999, seed=2), "f32")
    outs = torch.zeros(2, 2, device="cuda", dtype=torch.float64)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        rps.rps_consensus_static(Xa, n, N, outs[0])
        rps.rps_consensus_static(Xb, 3, 999, outs[1])
    s.synchronize()
    for X, o in ((Xa, outs[0]), (Xb, outs[1])):
        d_ref, m_ref = oracle.consensus(to_oracle(X))
        d, m = o.tolist()
        assert abs(m - m_ref) <= 1e-11 * m_ref and abs(d - d_ref) <= 1e-9 * d_ref


def test_static_consensus_rejects_what_it_cannot_serve(rps):
    X = torch.zeros(4, 64, device="cuda")
    out = torch.zeros(2, device="cuda", dtype=torch.float64)
    lib = ctypes.CDLL(rps.LIB_PATH)
    lib.rps_consensus_static.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32,
                                         ctypes.c_void_p, ctypes.c_void_p]
    call = lambda x, n, N, dtype, flags, o: lib.rps_consensus_static(x, n, N, dtype, flags, o, None)
    xp, op = X.data_ptr(), out.data_ptr()
    assert call(xp, 65, 64, 0, 0, op) == rps.RPS_ETOOBIG                 # more workers than the scratch is laid out for
    assert call(xp, 4, (1 << 34) + 1, 0, 0, op) == rps.RPS_ETOOBIG       # wider than the interface's maximum
    assert call(xp, 0, 64, 0, 0, op) == rps.RPS_EINVAL
    assert call(xp, 4, 64, 7, 0, op) == rps.RPS_EINVAL
    assert call(xp, 4, 64, 0, 1, op) == rps.RPS_EINVAL                   # not a layout flag
    assert call(None, 4, 64, 0, 0, op) == rps.RPS_EINVAL
    assert call(xp, 4, 64, 0, 0, None) == rps.RPS_EINVAL
    host = np.zeros((4, 64), dtype=np.float32)
    assert call(host.ctypes.data, 4, 64, 0, 0, op) == rps.RPS_EINVAL     # X must be device memory
    torch.cuda.synchronize()
    assert out.tolist() == [0.0, 0.0]                                    # nothing was enqueued by the rejected calls
    assert "maximum" in rps.rps_strerror(rps.RPS_ETOOBIG)
