"""GPU parity at the benchmark configurations, in the launch configuration bench.py times.

Full-size states do not fit an element-by-element oracle run in seconds, so at full size the
oracle follows a SAMPLE of model coordinates (the first and last 9 columns of every block plus
random ones, all workers): every column of a round depends only on that column's n values, the
round's masks and the column's own noise, so the oracle can evolve the sample for the whole
trajectory from the seeded initial state without ever reading a value the HIP path produced.
One configuration (n=16, N=11.2M) is also compared in full for two rounds."""
import numpy as np
import pytest
import torch

import workloads
from oracle import rps_oracle as oracle
from gpu_common import as_float, assert_close, device_tensor, masks_equal, to_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rps():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1810_07766_amd import rps as mod
    return mod


def _seeded_state(cfg, scale, seed):
    """[n, N] device tensor of N(0, scale^2) from a seeded device generator (zeros if scale == 0)."""
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    if scale == 0.0:
        return torch.zeros(cfg.n, cfg.N, device="cuda", dtype=tdt)
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    X = torch.empty(cfg.n, cfg.N, device="cuda", dtype=tdt)
    for i in range(cfg.n):                                 # row by row: bounded temporaries
        X[i] = (torch.randn(cfg.N, device="cuda", generator=g) * scale).to(tdt)
    return X


def _sampled_trajectory(rps, cfg, p, rounds, init_scale, per_block=40, tiled=False):
    """The HIP path on the full state (row-major or tile-major), the oracle on sampled columns."""
    off = workloads.config_offsets(cfg)
    cols = workloads.sample_columns(off, per_block=per_block, seed=11)
    X = _seeded_state(cfg, init_scale, seed=5)
    idx = torch.from_numpy(cols).cuda()
    Xo = to_oracle(X.index_select(1, idx))
    if tiled:
        X = workloads.to_tiled(X)
        T = X.shape[2]

    def sample():
        return to_oracle(X[idx // T, :, idx % T].t().contiguous() if tiled else X.index_select(1, idx))

    ctx = rps.RpsContext(cfg.n, cfg.N, p, cfg.gamma, cfg.seed,
                         rps.RPS_DTYPE_BF16 if cfg.dtype == "bf16" else rps.RPS_DTYPE_F32, block_offsets=off,
                         flags=rps.RPS_FLAG_LAYOUT_TILED if tiled else 0)
    ctx.set_synthetic_grad(cfg.sigma, cfg.weight_decay)
    worst = 0.0
    for t in range(rounds):
        ctx.round(X, None, t)
        oracle.round_(Xo, None, off, p=p, gamma=cfg.gamma, seed=cfg.seed, step=t, sigma=cfg.sigma,
                      weight_decay=cfg.weight_decay, cols=cols)
        if t < 3 or t == rounds - 1 or t % 10 == 0:
            masks_equal(ctx, cfg.seed, t, cfg.n, p)
            worst = max(worst, assert_close(sample(), Xo, off, cfg.dtype, cols=cols, what=f"{cfg.name} p={p} round {t}"))
    # properties that hold at any size, checked on the whole last state: per block, every worker
    # whose reply arrived holds the same bits
    server, U, D = oracle.masks(cfg.seed, rounds - 1, cfg.n, p)
    Xrm = workloads.from_tiled(X, cfg.N) if tiled else X
    for j in (0, cfg.n // 2, cfg.n - 1):
        recv = np.flatnonzero(D[:, j])
        blk = Xrm[:, int(off[j]):int(off[j + 1])]
        ref = blk[int(recv[0])]
        for i in recv[1:]:
            assert torch.equal(blk[int(i)], ref)
    ctx.destroy()
    return worst


def test_config_lsq_n4_trajectory(rps):
    """n=4, N=10,000, least squares, gamma=0.01, p=0.1, 100 rounds.  Each side computes its own
    full gradient A_i^T (A_i x_i - b_i) in float64 on the host from its own state."""
    cfg = workloads.CONFIGS["lsq_n4"]
    off = workloads.config_offsets(cfg)
    A, b = workloads.least_squares_problem(cfg.n, cfg.N, cfg.extra["rows"], seed=cfg.seed)

    def grad(X):
        return np.stack([A[i].T @ (A[i] @ X[i].astype(np.float64) - b[i]) for i in range(cfg.n)]).astype(np.float32)

    def loss(X):
        return float(np.mean([0.5 * np.sum((A[i] @ X.astype(np.float64).mean(axis=0) - b[i]) ** 2) for i in range(cfg.n)]))

    Xo = np.zeros((cfg.n, cfg.N), dtype=np.float32)
    Xg = torch.zeros(cfg.n, cfg.N, device="cuda")
    ctx = rps.RpsContext(cfg.n, cfg.N, cfg.p, cfg.gamma, cfg.seed)
    l0 = loss(Xo)
    for t in range(cfg.rounds):
        Gg = torch.from_numpy(grad(Xg.cpu().numpy())).cuda()
        ctx.round(Xg, Gg, t)
        oracle.round_(Xo, grad(Xo), off, p=cfg.p, gamma=cfg.gamma, seed=cfg.seed, step=t)
        if t % 10 == 9:
            torch.cuda.synchronize()
            assert_close(Xg.cpu().numpy(), Xo, off, "f32", what=f"round {t}")
    lg, lo = loss(Xg.cpu().numpy()), loss(Xo)
    assert lo < 0.8 * l0                                    # it optimises
    assert abs(lg - lo) <= 1e-6 * lo
    ctx.destroy()


def test_config_resnet18_n16_full_state_two_rounds(rps):
    """n=16, N=11.2M, all 179 M elements compared for two rounds (p = 0.1)."""
    cfg = workloads.CONFIGS["resnet18_n16"]
    off = workloads.config_offsets(cfg)
    X = _seeded_state(cfg, 0.01, seed=3)
    Xo = to_oracle(X)
    ctx = rps.RpsContext(cfg.n, cfg.N, cfg.p, cfg.gamma, cfg.seed)
    ctx.set_synthetic_grad(cfg.sigma, cfg.weight_decay)
    threads = min(16, oracle.max_threads())
    for t in range(2):
        ctx.round(X, None, t)
        oracle.round_(Xo, None, off, p=cfg.p, gamma=cfg.gamma, seed=cfg.seed, step=t, sigma=cfg.sigma,
                      weight_decay=cfg.weight_decay, threads=threads)
        torch.cuda.synchronize()
        got = X.cpu().numpy()
        # same tolerance as assert_close, vectorised per block for this size
        for j in range(cfg.n):
            blk = slice(int(off[j]), int(off[j + 1]))
            r = Xo[:, blk].astype(np.float64)
            tol = 1e-6 * (np.abs(r) + np.sqrt(np.mean(r ** 2)))
            assert (np.abs(got[:, blk] - r) <= tol).all(), f"round {t} block {j}"
    ctx.destroy()


@pytest.mark.parametrize("p", [0.0, 0.01, 0.1])
def test_config_resnet18_n16_sampled(rps, p):
    cfg = workloads.CONFIGS["resnet18_n16"]
    _sampled_trajectory(rps, cfg, p, cfg.rounds, init_scale=0.0)


def test_config_resnet50_n32_sampled(rps):
    """Headline configuration: n=32, N=25.6M, p=0.05, 50 rounds from the all-zero start."""
    cfg = workloads.CONFIGS["resnet50_n32"]
    _sampled_trajectory(rps, cfg, cfg.p, cfg.rounds, init_scale=0.0)


def test_config_resnet50_n32_sampled_random_start(rps):
    cfg = workloads.CONFIGS["resnet50_n32"]
    _sampled_trajectory(rps, cfg, cfg.p, 10, init_scale=0.02)


@pytest.mark.parametrize("name,rounds,init", [("resnet50_n32", 50, 0.0), ("resnet50_n32", 10, 0.02),
                                               ("resnet18_n16", 50, 0.0), ("bert_n64_bf16", 8, 0.0)])
def test_config_tiled_layout_sampled(rps, name, rounds, init):
    """The benchmark workloads in the tile-major layout (the launch configuration bench.py times for
    the fp32 workloads), the oracle on sampled columns; the bf16 workload's width is not a
    multiple of the tile, so its last tile is padded."""
    cfg = workloads.CONFIGS[name]
    _sampled_trajectory(rps, cfg, cfg.p, rounds, init_scale=init, per_block=24 if cfg.n == 64 else 40, tiled=True)


def test_config_bert_n64_bf16_sampled(rps):
    """n=64, N=110M, bf16 storage, 64 unequal blocks, 20 rounds (14 GB of state)."""
    cfg = workloads.CONFIGS["bert_n64_bf16"]
    _sampled_trajectory(rps, cfg, cfg.p, cfg.rounds, init_scale=0.0, per_block=24)


@pytest.mark.parametrize("tiled", [False, True])
def test_config_mlp_n8_loss_tracks_oracle(rps, tiled):
    """n=8 workers, 2-layer MLP 1024->2048->1024 (N = 4,194,304), teacher targets, batch 256 per
    worker, p = 0.2, 200 rounds.  Gradients come from PyTorch (GPU side: on the GPU from the GPU
    state; oracle side: on the CPU from the oracle's state), the round from the library / the
    oracle.  The two trajectories are independent, so GEMM rounding differences feed back; the
    loss curves and the mean model must still track each other closely."""
    cfg = workloads.CONFIGS["mlp_n8"]
    off = workloads.config_offsets(cfg)
    teacher, X0 = workloads.mlp_problem(cfg, seed=cfg.seed)
    Xo = X0.numpy().copy()
    ctx = rps.RpsContext(cfg.n, cfg.N, cfg.p, cfg.gamma, cfg.seed, flags=rps.RPS_FLAG_LAYOUT_TILED if tiled else 0)
    if tiled:
        Xg = X0.cuda()
    else:
        # row-major: every worker's parameters stay one contiguous row; N * 4 bytes = 2^24 would put the
        # same columns of all rows on one memory channel, so the rows are held a little further apart
        ctx.set_row_pitch(rps.rps_recommended_row_pitch(cfg.N))
        Xg = ctx.empty_state(); Xg.copy_(X0.cuda())
        Gp = ctx.empty_state()
    threads = min(16, oracle.max_threads())
    first = last = None

    def gpu_round(X, G, t):
        """The library's round on [n, N] tensors; in the tile-major run through re-arranged copies
        (the model's forward/backward wants each worker's parameters contiguous)."""
        if not tiled:
            Gp.copy_(G)                                  # autograd hands back a dense [n, N] gradient
            ctx.round(X, Gp, t)
            return
        Xt = workloads.to_tiled(X)
        ctx.round(Xt, workloads.to_tiled(G), t)
        X.copy_(workloads.from_tiled(Xt, cfg.N))

    for t in range(cfg.rounds):
        xb, yb = workloads.mlp_batch(cfg, teacher, t, seed=7)
        lg, Gg = workloads.mlp_loss_and_grad(cfg, Xg, xb.cuda(), yb.cuda())
        gpu_round(Xg, Gg, t)
        lo, Go = workloads.mlp_loss_and_grad(cfg, torch.from_numpy(Xo), xb, yb)
        oracle.round_(Xo, Go.numpy(), off, p=cfg.p, gamma=cfg.gamma, seed=cfg.seed, step=t, threads=threads)
        lgm, lom = float(lg.mean()), float(lo.mean())
        assert abs(lgm - lom) <= 1e-3 * lom, f"round {t}: loss {lgm} vs oracle {lom}"
        first = lom if first is None else first
        last = lom
        if t % 50 == 49:
            print(f"round {t}: loss gpu {lgm:.6f} oracle {lom:.6f}", flush=True)
    assert last < 0.9 * first                                   # it trains
    got = Xg.cpu().numpy().astype(np.float64)
    ref = Xo.astype(np.float64)
    # independent trajectories: compare at the scale of the parameters, not bitwise
    assert np.abs(got.mean(axis=0) - ref.mean(axis=0)).max() <= 1e-3 * np.sqrt(np.mean(ref ** 2))
    # the round itself, from the oracle's final state and gradient, still matches element-wise
    Xs = torch.from_numpy(Xo).cuda()
    if not tiled:
        Xs = ctx.empty_state().copy_(Xs)
    gpu_round(Xs, Go.cuda(), cfg.rounds)
    oracle.round_(Xo, Go.numpy(), off, p=cfg.p, gamma=cfg.gamma, seed=cfg.seed, step=cfg.rounds, threads=threads)
    torch.cuda.synchronize()
    assert_close(Xs.cpu().numpy(), Xo, off, "f32", what="single round from the oracle state")
    ctx.destroy()


def test_config_resnet50_n32_contraction_rate(rps):
    """A property that holds at any size: one averaging round without gradients shrinks the
    disagreement sum_i ||x_i - xbar||^2 by beta = alpha_1 - alpha_2 in expectation (supplement,
    proof of Lemma 1).  At n = 32, p = 0.05 the 32 blocks x 3 fresh states average the ratio well; the
    exact beta comes from the supplement's case analysis (Lemmas 7 and 8), recomputed here."""
    from math import comb
    cfg = workloads.CONFIGS["resnet50_n32"]
    n, p = cfg.n, cfg.p
    q = 1 - p
    w11 = sum(comb(n - 1, m) * q ** m * p ** (n - 1 - m) / (m + 1) ** 2 for m in range(n))
    w1n2 = sum(comb(n - 2, m) * q ** (m + 1) * p ** (n - 2 - m) / (m + 2) ** 2 for m in range(n - 1))
    w1n = sum(comb(n - 2, m) * q ** (m + 1) * p ** (n - 2 - m) / (m + 2) for m in range(n - 1))
    e1 = (w11 * (1 + (n - 1) * q) + (1 + w1n2 * (1 + (n - 2) * q)) * p * (n - 1) + w1n2 * (2 + (n - 2) * q) * q * (n - 1)) / n
    a1 = (n * e1 - 1) / (n - 1)
    e2 = (w11 * ((1 + (n - 1) * q) ** 2 + (n - 1) * p * q)
          + (1 + 2 * w1n * ((n - 2) * q + 1) + w1n2 * (1 + 2 * (n - 2) * q + (n - 2) ** 2 * q * q + (n - 2) * p * q)) * p * (n - 1)
          + w1n2 * (((n - 2) * q + 2) ** 2 + (n - 2) * p * q) * q * (n - 1)) / n
    a2 = (e2 - 1) / (n - 1)
    beta = a1 - a2
    ctx = rps.RpsContext(cfg.n, cfg.N, cfg.p, cfg.gamma, cfg.seed)
    ratios = []
    for t in range(3):                                   # fresh i.i.d. state each time: the identity is an
        X = _seeded_state(cfg, 1.0, seed=21 + t)         # expectation over the masks for a FIXED state, and
        d0, _ = ctx.consensus(X)                         # after a round the disagreement sits in a few outlier
        ctx.lossy_average(X, t)                          # rows, which makes later single draws heavy-tailed
        d1, _ = ctx.consensus(X)
        ratios.append(d1 / d0)
        del X
    # each of the 32 blocks is an independent draw of the masks: 96 draws, a 30 % band
    assert abs(np.mean(ratios) - beta) < 0.30 * beta, (ratios, beta)
    ctx.destroy()


def test_config_lsq_n4_gradient_averaging_drifts(rps):
    """The paper's Sec. 6 observation on the least-squares workload: with 10 % loss, averaging
    gradients lets the worker models drift apart, averaging models does not.  Both runs use the
    library end to end (rounds and rps_consensus)."""
    cfg = workloads.CONFIGS["lsq_n4"]
    A, b = workloads.least_squares_problem(cfg.n, cfg.N, cfg.extra["rows"], seed=cfg.seed)
    At = torch.from_numpy(A).cuda(); bt = torch.from_numpy(b).cuda()

    def grad(X):
        r = torch.bmm(At, X.double().unsqueeze(2)).squeeze(2) - bt
        return torch.bmm(At.transpose(1, 2), r.unsqueeze(2)).squeeze(2).float().contiguous()

    ctx = rps.RpsContext(cfg.n, cfg.N, cfg.p, cfg.gamma, cfg.seed)
    Xm = torch.zeros(cfg.n, cfg.N, device="cuda"); Xg = torch.zeros(cfg.n, cfg.N, device="cuda")
    for t in range(cfg.rounds):
        ctx.round(Xm, grad(Xm), t)
        ctx.round_gradient_averaging(Xg, grad(Xg), t)
    dm, _ = ctx.consensus(Xm)
    dg, _ = ctx.consensus(Xg)
    assert dg > 10 * dm, (dg, dm)
    ctx.destroy()


@pytest.mark.parametrize("n,N,dtype,split,tiled", [(2, 1 << 34, "bf16", (1 << 33) + 1288, False),
                                                   (1, (1 << 32) + 3, "f32", None, False),
                                                   (1, 1 << 34, "f32", None, False),
                                                   (2, 1 << 34, "bf16", (1 << 33) + 1288, True),
                                                   (3, (1 << 32) + 3, "f32", ((1 << 31) + 5, (1 << 31) + 1000008), True)])
def test_maximum_width(rps, n, N, dtype, split, tiled):
    """The interface's widest model (N = 2^34 columns; column indices, noise counters and byte
    offsets all pass 2^32) and an odd width just past 2^32 (element-wise path, one worker).
    Starts from X = 0 (Alg. 1's identical start); the oracle evolves sampled columns -- both ends,
    both sides of 2^32, of the block boundary and of the last tile -- by itself for three rounds."""
    free, _ = torch.cuda.mem_get_info()
    elem = 2 if dtype == "bf16" else 4
    if free < n * (N + 64) * elem + (8 << 30):
        pytest.skip("not enough free device memory for the maximum-width state")
    cuts = [] if split is None else (list(split) if isinstance(split, tuple) else [split])
    off = np.array([0] + cuts + [N], dtype=np.int64)
    marks = [0, 1 << 32, N - 600] + cuts + [N - 40]
    cols = np.unique(np.concatenate([np.arange(max(m - 20, 0), min(m + 20, N)) for m in marks] +
                                    [workloads.sample_columns(off, per_block=60, seed=3)]))
    idx = torch.from_numpy(cols).cuda()
    p, gamma, seed = 0.3, 0.5, 2024
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    T = workloads.TILE_BYTES // elem
    X = torch.zeros(((N + T - 1) // T, n, T) if tiled else (n, N), device="cuda", dtype=tdt)

    def sample():
        return to_oracle(X[idx // T, :, idx % T].t().contiguous() if tiled else X.index_select(1, idx))

    Xo = sample()
    ctx = rps.RpsContext(n, N, p, gamma, seed, rps.RPS_DTYPE_BF16 if dtype == "bf16" else rps.RPS_DTYPE_F32,
                         block_offsets=off, flags=rps.RPS_FLAG_LAYOUT_TILED if tiled else 0)
    ctx.set_synthetic_grad(1.0, 0.01)
    for t in range(3):
        if t == 1:                                               # unfused once: the tiled local step at this width
            ctx.local_step(X, None, t); ctx.lossy_average(X, t)
        else:
            ctx.round(X, None, t)
        oracle.round_(Xo, None, off, p=p, gamma=gamma, seed=seed, step=t, sigma=1.0, weight_decay=0.01, cols=cols)
        masks_equal(ctx, seed, t, n, p)
        got = sample()
        assert_close(got, Xo, off, dtype, cols=cols, what=f"N={N} round {t}")
    assert np.abs(as_float(Xo)).max() > 0.1                     # the noise really moved the state
    ctx.destroy()
    del X
    torch.cuda.empty_cache()
