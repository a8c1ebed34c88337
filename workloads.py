"""Seeded synthetic inputs and the benchmark configurations.

This module serves both the HIP path's tests/benchmark and the CPU oracle's
tests.  It holds NO arithmetic of the method (no averaging, no masks, no SGD
step, no counter-based hash): only shapes, seeds and input generators.

The paper (arXiv 1810.07766, Sec. 6) trains ResNet-20/110 on CIFAR-10 and an
LSTM on ATIS; neither the data nor the models are needed to exercise the
averaging round, whose cost depends only on (n, N, dtype, block structure).
The configurations below stand in for those workloads with flat parameter
vectors sized like common DNNs and the paper's network model (n workers =
n servers, i.i.d. message loss p within the paper's tested 1-20 % range).
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    n: int                    # workers (= blocks = servers)
    N: int                    # parameters per worker
    dtype: str                # "f32" | "bf16"  (storage; math is fp32, sums fp64)
    p: float                  # message drop probability
    gamma: float              # step size
    rounds: int
    seed: int = 0
    sigma: float = 0.0        # std of the synthetic gradient noise (0: caller's gradient)
    weight_decay: float = 0.0
    unequal_blocks: bool = False
    block_seed: int = 1
    gradient: str = "synthetic"   # "synthetic" | "least_squares" | "mlp"
    extra: dict = field(default_factory=dict)


# BASELINE.json configs, in order.  "N(0,1e-2)" is read as a variance: sigma = 0.1.
CONFIGS = {
    "lsq_n4": Config("lsq_n4", n=4, N=10_000, dtype="f32", p=0.1, gamma=0.01, rounds=100,
                     gradient="least_squares", extra={"rows": 256}),
    "resnet18_n16": Config("resnet18_n16", n=16, N=11_200_000, dtype="f32", p=0.1, gamma=0.1,
                           rounds=50, sigma=0.1, weight_decay=1e-4),
    "resnet50_n32": Config("resnet50_n32", n=32, N=25_600_000, dtype="f32", p=0.05, gamma=0.1,
                           rounds=50, sigma=0.1),
    "mlp_n8": Config("mlp_n8", n=8, N=1024 * 2048 + 2048 * 1024, dtype="f32", p=0.2, gamma=0.5,
                     rounds=200, gradient="mlp", extra={"d_in": 1024, "d_hidden": 2048,
                                                        "d_out": 1024, "batch": 256}),
    "bert_n64_bf16": Config("bert_n64_bf16", n=64, N=110_000_000, dtype="bf16", p=0.1, gamma=0.1,
                            rounds=20, sigma=float(np.sqrt(1e-3)), unequal_blocks=True),
}
HEADLINE = "resnet50_n32"


def block_offsets(n: int, N: int, unequal: bool = False, block_seed: int = 1,
                  multiple: int = 8) -> np.ndarray:
    """Partition [0, N) into n blocks; returns n+1 int64 offsets.

    Equal blocks (the paper's "equally-sized blocks") need N % n == 0.  Unequal
    blocks: sizes drawn uniform in [0.5, 1.5] x N/n, rounded down to a multiple
    of `multiple` elements, the last block taking the remainder.
    """
    if not unequal:
        if N % n:
            raise ValueError("equal blocks need N % n == 0")
        return np.arange(n + 1, dtype=np.int64) * (N // n)
    rng = np.random.default_rng(block_seed)
    u = rng.uniform(0.5, 1.5, size=n)
    sizes = np.floor(N * u / u.sum() / multiple).astype(np.int64) * multiple
    sizes = np.maximum(sizes, multiple)
    sizes[-1] = N - sizes[:-1].sum()
    if sizes[-1] <= 0:
        raise ValueError("degenerate block sizes")
    off = np.zeros(n + 1, dtype=np.int64)
    off[1:] = np.cumsum(sizes)
    return off


def config_offsets(cfg: Config) -> np.ndarray:
    return block_offsets(cfg.n, cfg.N, cfg.unequal_blocks, cfg.block_seed)


def gaussian_model(n: int, N: int, seed: int, scale: float = 1.0, identical: bool = False) -> np.ndarray:
    """[n, N] float32 test state: i.i.d. N(0, scale^2), or one row repeated
    (Alg. 1 starts all workers from the same point)."""
    rng = np.random.default_rng(seed)
    if identical:
        row = (rng.standard_normal(N) * scale).astype(np.float32)
        return np.tile(row, (n, 1))
    return (rng.standard_normal((n, N)) * scale).astype(np.float32)


def least_squares_problem(n: int, N: int, rows: int, seed: int):
    """Per-worker least squares f_i(x) = 0.5 ||A_i x - b_i||^2 with
    A_i [rows, N] ~ N(0, 1/N), b_i ~ N(0, 1).  Returns (A [n, rows, N] f64, b [n, rows] f64)."""
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((n, rows, N)) / np.sqrt(N)
    b = rng.standard_normal((n, rows))
    return A, b


def sample_columns(offsets: np.ndarray, per_block: int, seed: int) -> np.ndarray:
    """Sorted sample of model coordinates: the first and last 9 columns of every
    block (block edges, ragged tails) plus `per_block` random ones."""
    rng = np.random.default_rng(seed)
    cols = []
    for j in range(len(offsets) - 1):
        lo, hi = int(offsets[j]), int(offsets[j + 1])
        if hi <= lo:
            continue
        edge = list(range(lo, min(lo + 9, hi))) + list(range(max(hi - 9, lo), hi))
        rnd = rng.integers(lo, hi, size=per_block).tolist() if per_block else []
        cols.extend(edge + rnd)
    return np.unique(np.asarray(cols, dtype=np.int64))


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even, via torch's
    own conversion (an input-format helper, independent of both implementations)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def mlp_problem(cfg: Config, seed: int):
    """Teacher W* [d_out, d_in] ~ N(0, 1/d_in) and the shared initial flat parameters
    (W1 [d_hidden, d_in] ~ N(0, 1/d_in), W2 [d_out, d_hidden] ~ N(0, 1/d_hidden); zero weights
    would give zero gradients).  torch CPU tensors from a seeded generator."""
    import torch
    e = cfg.extra
    g = torch.Generator().manual_seed(seed)
    teacher = torch.randn(e["d_out"], e["d_in"], generator=g) / e["d_in"] ** 0.5
    w1 = torch.randn(e["d_hidden"], e["d_in"], generator=g) / e["d_in"] ** 0.5
    w2 = torch.randn(e["d_out"], e["d_hidden"], generator=g) / e["d_hidden"] ** 0.5
    x0 = torch.cat([w1.reshape(-1), w2.reshape(-1)])
    return teacher, x0.repeat(cfg.n, 1).contiguous()


def mlp_batch(cfg: Config, teacher, step: int, seed: int):
    """Round `step`'s inputs x ~ N(0,1) [n, batch, d_in] and targets y = W* x (torch CPU)."""
    import torch
    e = cfg.extra
    g = torch.Generator().manual_seed(seed * 1_000_003 + step)
    xb = torch.randn(cfg.n, e["batch"], e["d_in"], generator=g)
    return xb, xb @ teacher.T


def mlp_loss_and_grad(cfg: Config, X, xb, yb):
    """Per-worker MSE loss of the 2-layer ReLU MLP held as flat rows of X, and its gradient
    [n, N] (PyTorch autograd on whatever device X lives on).  Input/model code, not part of
    the averaging method."""
    import torch
    e = cfg.extra
    k = e["d_hidden"] * e["d_in"]
    Xp = X.detach().clone().requires_grad_(True)
    W1 = Xp[:, :k].view(cfg.n, e["d_hidden"], e["d_in"])
    W2 = Xp[:, k:].view(cfg.n, e["d_out"], e["d_hidden"])
    h = torch.relu(torch.bmm(xb, W1.transpose(1, 2)))
    out = torch.bmm(h, W2.transpose(1, 2))
    loss = ((out - yb) ** 2).mean(dim=(1, 2))
    (G,) = torch.autograd.grad(loss.sum(), Xp)
    return loss.detach(), G.contiguous()


TILE_BYTES = 128   # the library's tile-major storage: segments of 128 bytes per (tile, worker)


def to_tiled(X):
    """[n, N] -> [ceil(N/T), n, T] (T = 128 bytes of elements; columns beyond N are zero padding).
    Pure re-arrangement of a torch tensor or numpy array; no arithmetic."""
    import torch
    t = torch.as_tensor(X)
    n, N = t.shape
    T = TILE_BYTES // t.element_size()
    tiles = (N + T - 1) // T
    if tiles * T != N:
        pad = torch.zeros(n, tiles * T - N, dtype=t.dtype, device=t.device)
        t = torch.cat([t, pad], dim=1)
    return t.reshape(n, tiles, T).permute(1, 0, 2).contiguous()


def from_tiled(Xt, N):
    """Inverse of to_tiled: [tiles, n, T] -> [n, N]."""
    tiles, n, T = Xt.shape
    return Xt.permute(1, 0, 2).reshape(n, tiles * T)[:, :N].contiguous()
