"""Helpers for the GPU parity tests: run the HIP library and the CPU oracle on the same
seeded inputs and compare element by element.

Tolerance (fp32 parameters): |gpu - oracle| <= rtol * (|oracle| + rms(oracle block)), rtol = 1e-6
for fp32 storage and 1e-2 for bf16 storage.  A pure element-wise relative error is unusable
(entries pass through zero); the block rms is the natural scale of a block's values.  Masks,
server permutation and every comparison labelled "bitwise" are exact.
"""
import numpy as np
import torch

import workloads
from oracle import rps_oracle as oracle
from paper_1810_07766_amd import rps

RTOL = {"f32": 1e-6, "bf16": 1e-2}


def device_tensor(a: np.ndarray, dtype: str) -> torch.Tensor:
    """numpy float32 [n, N] -> cuda tensor in the storage dtype."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t.contiguous()


def to_oracle(t: torch.Tensor) -> np.ndarray:
    """cuda/cpu tensor -> the oracle's array type (float32, or uint16 bf16 bits)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


def as_float(a: np.ndarray) -> np.ndarray:
    return workloads.from_bf16_bits(a).astype(np.float64) if a.dtype == np.uint16 else a.astype(np.float64)


def assert_close(gpu: np.ndarray, ref: np.ndarray, offsets, dtype: str, cols=None, what=""):
    """Element-wise comparison with the block-rms-scaled tolerance."""
    g, r = as_float(gpu), as_float(ref)
    assert g.shape == r.shape
    colidx = np.arange(r.shape[1]) if cols is None else np.asarray(cols)
    blk = np.searchsorted(np.asarray(offsets)[1:], colidx, side="right")
    worst = 0.0
    for j in np.unique(blk):
        sel = blk == j
        rms = np.sqrt(np.mean(r[:, sel] ** 2))
        tol = RTOL[dtype] * (np.abs(r[:, sel]) + rms)
        err = np.abs(g[:, sel] - r[:, sel])
        bad = err > tol
        if bad.any():
            k = np.argmax(err / np.maximum(tol, 1e-300))
            raise AssertionError(f"{what}: block {j}: {bad.sum()} of {bad.size} outside tolerance; worst "
                                 f"err/tol = {(err / np.maximum(tol, 1e-300)).flat[k]:.3g} "
                                 f"(gpu {g[:, sel].flat[k]!r}, oracle {r[:, sel].flat[k]!r})")
        worst = max(worst, float((err / np.maximum(tol, 1e-300)).max()))
    return worst


def masks_equal(ctx, seed, step, n, p, identity=False):
    s_g, u_g, d_g = ctx.get_masks(step)
    s_o, u_o, d_o = oracle.masks(seed, step, n, p, identity)
    # the library's host copy of the generator must tell the same story as its device table
    s_h, u_h, d_h = rps.rps_masks_host(n, p, seed, step, flags=rps.RPS_FLAG_SERVER_IDENTITY if identity else 0)
    assert (s_g == s_h).all() and (u_g == u_h).all() and (d_g == d_h).all(), f"device and host generator differ at step {step}"
    assert (s_g == s_o).all(), f"server permutation differs at step {step}"
    assert (u_g == u_o).all(), f"uplink mask differs at step {step}"
    assert (d_g == d_o).all(), f"downlink mask differs at step {step}"
