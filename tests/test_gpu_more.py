"""GPU parity, part two (through the C ABI, against the CPU oracle): padded row pitch, a decayed
step-size schedule, a worker cut off from the network for several rounds, and the grid of mixing
constants that the paper's Fig. 2 and Fig. 3 plot."""
import os

import numpy as np
import pytest
import torch

import workloads
from oracle import rps_oracle as oracle
from gpu_common import assert_close, device_tensor, to_oracle

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="module")
def rps():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1810_07766_amd import rps as mod
    return mod


def _dt(rps, dtype):
    return rps.RPS_DTYPE_BF16 if dtype == "bf16" else rps.RPS_DTYPE_F32


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,N,pad,dtype", [(8, 8 * 2048, 1024, "f32"), (5, 5 * 1601, 3, "f32"), (32, 32 * 1544, 64, "f32"),
                                           (16, 16 * 1544, 2048, "bf16"), (7, 7 * 999, 9, "bf16"), (64, 64 * 520, 8, "bf16")])
def test_row_pitch_every_entry_point(rps, n, N, pad, dtype):
    """X and G as [n, N] views of arrays whose rows are N + pad elements apart (rps_set_row_pitch):
    every entry point against the oracle, the padding never written; pads that keep the rows
    16-byte aligned (128-bit path) and pads that do not (element-wise path)."""
    pitch = N + pad
    off = workloads.block_offsets(n, N) if N % n == 0 else np.linspace(0, N, n + 1).astype(np.int64)
    p, gamma, seed = 0.25, 0.3, 5
    ctx = rps.RpsContext(n, N, p, gamma, seed, _dt(rps, dtype), block_offsets=off)
    ctx.set_synthetic_grad(0.5, 0.01)
    with pytest.raises(rps.RpsError):
        ctx.set_row_pitch(N - 1)
    ctx.set_row_pitch(pitch)
    sentinel = 12288.0
    X = ctx.empty_state(fill=sentinel); G = ctx.empty_state(fill=sentinel)
    X.copy_(device_tensor(workloads.gaussian_model(n, N, seed=3), dtype))
    G.copy_(device_tensor(workloads.gaussian_model(n, N, seed=4), dtype))
    Xo, Go = to_oracle(X), to_oracle(G)
    with pytest.raises(rps.RpsError):
        ctx.round(X.contiguous(), None, 0)                                 # rows N apart: not this context's pitch
    calls = ["round", "roundG", "local_step", "lossy_average", "local_stepG", "gradavg", "round"]
    for t, what in enumerate(calls):
        if what == "round":
            ctx.round(X, None, t)
            oracle.round_(Xo, None, off, p=p, gamma=gamma, seed=seed, step=t, sigma=0.5, weight_decay=0.01)
        elif what == "roundG":
            ctx.round(X, G, t)
            oracle.round_(Xo, Go, off, p=p, gamma=gamma, seed=seed, step=t)
        elif what == "local_step":
            ctx.local_step(X, None, t)
            oracle.local_step(Xo, None, gamma, sigma=0.5, weight_decay=0.01, seed=seed, step=t)
        elif what == "local_stepG":
            ctx.local_step(X, G, t)
            oracle.local_step(Xo, Go, gamma)
        elif what == "lossy_average":
            ctx.lossy_average(X, t)
            _, U, D = oracle.masks(seed, t, n, p)
            oracle.lossy_average(Xo, off, U, D)
        else:
            ctx.round_gradient_averaging(X, G, t)
            oracle.round_gradient_averaging(Xo, Go, off, p=p, gamma=gamma, seed=seed, step=t)
        torch.cuda.synchronize()
        assert_close(to_oracle(X), Xo, off, dtype, what=f"call {t} ({what}), pitch {pitch}")
    d, m = ctx.consensus(X)
    d_ref, m_ref = oracle.consensus(to_oracle(X))
    assert abs(m - m_ref) <= 1e-11 * m_ref and abs(d - d_ref) <= 1e-9 * d_ref
    # layout conversion with the padded pitch on the row-major side
    Xt = ctx.to_tiled(X)
    assert torch.equal(Xt, workloads.to_tiled(X.contiguous()))
    back = ctx.from_tiled(Xt)
    assert back.stride(0) == pitch and torch.equal(back, X)
    for T in (X, G):                                                       # the padding was never written
        full = torch.as_strided(T, (n, pitch), (pitch, 1))
        assert bool((full[:, N:] == sentinel).all())
    ctx.destroy()


def test_recommended_row_pitch(rps):
    for N, dt, elem in ((1 << 22, rps.RPS_DTYPE_F32, 4), (25_600_000, rps.RPS_DTYPE_F32, 4), (110_000_000, rps.RPS_DTYPE_BF16, 2),
                        (1000, rps.RPS_DTYPE_F32, 4)):
        pitch = rps.rps_recommended_row_pitch(N, dt)
        assert pitch >= N and (pitch * elem) % 65536 == 4096 and (pitch - N) * elem < 65536 + 4096
    assert rps.rps_recommended_row_pitch(0, rps.RPS_DTYPE_F32) == -1
    ctx = rps.RpsContext(4, 1024, 0.1, 0.1, 0, flags=rps.RPS_FLAG_LAYOUT_TILED)
    with pytest.raises(rps.RpsError):
        ctx.set_row_pitch(2048)                                            # the tiled layout has no row pitch
    ctx.destroy()


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("tiled,dtype", [(False, "f32"), (True, "f32"), (True, "bf16")])
def test_decayed_step_size_schedule(rps, tiled, dtype):
    """Sec. 5 (remark after Corollary 1): with a step size that decays over the rounds the algorithm
    reaches a critical point.  20 rounds with gamma_t = gamma_0 / sqrt(t + 1) set through
    rps_set_gamma before every round, against the oracle run with the same schedule; the fused round
    equals local step + lossy average bit for bit under the schedule."""
    n, N, p, seed = 12, 12 * 1100, 0.15, 77
    off = workloads.block_offsets(n, N)
    ctx = rps.RpsContext(n, N, p, 1.0, seed, _dt(rps, dtype), flags=rps.RPS_FLAG_LAYOUT_TILED if tiled else 0)
    ctx.set_synthetic_grad(0.2, 0.05)
    Xr = device_tensor(workloads.gaussian_model(n, N, seed=9, scale=0.5), dtype)
    Xo = to_oracle(Xr)
    X = workloads.to_tiled(Xr) if tiled else Xr
    for t in range(20):
        gamma = float(np.float32(0.4 / np.sqrt(t + 1.0)))
        ctx.set_gamma(gamma)
        unfused = X.clone()
        ctx.round(X, None, t)
        ctx.local_step(unfused, None, t); ctx.lossy_average(unfused, t)
        assert torch.equal(unfused, X), f"round {t}: fused and unfused differ"
        oracle.round_(Xo, None, off, p=p, gamma=gamma, seed=seed, step=t, sigma=0.2, weight_decay=0.05)
        got = workloads.from_tiled(X, N) if tiled else X
        assert_close(to_oracle(got), Xo, off, dtype, what=f"round {t}, gamma {gamma}")
    with pytest.raises(rps.RpsError):
        ctx.set_gamma(float("nan"))
    ctx.destroy()


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("tiled", [False, True])
def test_isolated_worker_drifts_and_rejoins(rps, tiled):
    """Failure forcing (Sec. 3's network, through the mask override): worker 0 is cut off -- all its
    uplinks and downlinks lost -- for 12 rounds while the others talk without loss, then it rejoins.
    While it is isolated its model takes its own noisy steps and the disagreement
    sum_i ||x_i - xbar||^2 (the quantity the supplement's Lemma 1 bounds) grows round after round;
    one loss-free round after rejoining removes it.  Every state against the oracle."""
    n, N, gamma, seed = 8, 8 * 1500, 0.1, 3
    off = workloads.block_offsets(n, N)
    ctx = rps.RpsContext(n, N, 0.0, gamma, seed, flags=rps.RPS_FLAG_LAYOUT_TILED if tiled else 0)
    ctx.set_synthetic_grad(0.3, 0.0)
    server = np.roll(np.arange(n, dtype=np.int32), 1)                # block j served by worker j-1: worker 0 serves block 1
    U = np.ones((n, n), dtype=np.uint8); D = np.ones((n, n), dtype=np.uint8)
    U[0, :] = 0; D[0, :] = 0                                         # worker 0: nothing goes out, nothing comes in
    U[0, 1] = D[0, 1] = 1                                            # except the link to itself (block it serves)
    U[1:, 1] = 0; D[1:, 1] = 0                                       # ... and nobody reaches that server either
    x0 = workloads.gaussian_model(1, N, seed=4)
    Xr = device_tensor(np.repeat(x0, n, axis=0), "f32")              # Alg. 1: identical start
    Xo = to_oracle(Xr)
    X = workloads.to_tiled(Xr) if tiled else Xr
    ctx.set_mask_override(server, U, D)
    dist = []
    for t in range(12):
        ctx.round(X, None, t)
        oracle.round_(Xo, None, off, p=0.0, gamma=gamma, seed=seed, step=t, sigma=0.3, mask_override=(server, U, D))
        got = workloads.from_tiled(X, N) if tiled else X
        assert_close(to_oracle(got), Xo, off, "f32", what=f"isolated, round {t}")
        d, _ = ctx.consensus(X)
        d_ref, _ = oracle.consensus(Xo)
        assert abs(d - d_ref) <= 1e-5 * d_ref
        dist.append(d)
    # a random walk of the isolated worker against the others' averaged walk: the disagreement keeps growing
    assert all(b > a for a, b in zip(dist[:6], dist[1:7])) and dist[-1] > 5 * dist[0]
    ctx.set_mask_override()                                          # p = 0: everything arrives again
    ctx.lossy_average(X, 100)
    _, U1, D1 = oracle.masks(seed, 100, n, 0.0)
    oracle.lossy_average(Xo, off, U1, D1)
    got = workloads.from_tiled(X, N) if tiled else X
    assert_close(to_oracle(got), Xo, off, "f32", what="after rejoining")
    d, _ = ctx.consensus(X)
    assert d <= 1e-10 * dist[-1]                                     # exact averaging: consensus restored
    ctx.destroy()


# ---------------------------------------------------------------------------------------------
def _alpha_grid():
    rows = []
    with open(os.path.join(GOLDEN, "alpha_grid.txt")) as f:
        for line in f:
            if not line.startswith("#"):
                v = line.split()
                rows.append((int(v[0]), float(v[1]), float(v[2]), float(v[3]), float(v[4])))
    return rows


def test_mixing_constants_over_the_grid_of_fig2_and_fig3(rps):
    """rps_estimate_mixing on the (n, p) grid of the paper's Fig. 2 (alpha2) and Fig. 3 (beta) at the
    benchmark worker counts: every row of tests/golden/alpha_grid.txt (exact sums of the supplement's
    Lemmas 7 and 8, written by an oracle-side script) is reproduced within 5 standard errors, and the
    device's estimates show what the paper reads off the figures: alpha2 falls as n grows (Sec. 4.2:
    the influence of p diminishes with more workers), beta grows with p and stays close to p."""
    rows = _alpha_grid()
    assert len(rows) == 20
    est = {}
    for n, p, a1, a2, beta in rows:
        ctx = rps.RpsContext(n, 64 * n, p, 0.1, 4321, rps.RPS_DTYPE_F32)
        rounds = max(1 << 10, (1 << 17) // n)
        b = np.array([ctx.estimate_mixing(k * rounds, rounds) for k in range(16)])
        ctx.destroy()
        m = b.mean(axis=0); se = b.std(axis=0, ddof=1) / np.sqrt(16.0)
        bm = (b[:, 0] - b[:, 1]).mean(); bse = (b[:, 0] - b[:, 1]).std(ddof=1) / np.sqrt(16.0)
        assert abs(m[0] - a1) < 5 * se[0] and se[0] < 0.03 * a1, (n, p, m, se, a1)
        assert abs(m[1] - a2) < 5 * se[1] and se[1] < 0.03 * a2, (n, p, m, se, a2)
        assert abs(bm - beta) < 5 * bse, (n, p, bm, bse, beta)
        est[(n, p)] = (m[0], m[1], bm)
    ns = sorted({n for n, _ in est}); ps = sorted({p for _, p in est})
    for p in ps:
        a2s = [est[(n, p)][1] for n in ns]
        assert all(x > y for x, y in zip(a2s, a2s[1:])), (p, a2s)            # Fig. 2: alpha2 falls with n
        assert a2s[-1] * ns[-1] < 2.5 * p * (1 - p) + 0.01                     # ... like p(1-p)/n
    for n in ns:
        betas = [est[(n, p)][2] for p in ps]
        assert all(x < y for x, y in zip(betas, betas[1:])), (n, betas)      # Fig. 3: beta grows with p
        assert all(abs(b - p) < 0.45 * p for b, p in zip(betas, ps)), (n, betas)


# ---------------------------------------------------------------------------------------------
def test_occupancy_cap_reaches_the_launch(rps):
    """The round kernels limit how many wavefronts a compute unit holds through an LDS allocation
    they never touch.  rps_query_occupancy reports what the runtime's occupancy calculator makes of
    the kernel and launch shape a context would use: a requested cap must arrive exactly where it is
    a whole number of workgroups, the built-in defaults must be what the library documents, and no
    cap must mean the register-limited occupancy of the kernel."""
    for tiled in (False, True):
        flags = rps.RPS_FLAG_LAYOUT_TILED if tiled else 0
        ctx = rps.RpsContext(32, 32 * 4096, 0.05, 0.1, 0, rps.RPS_DTYPE_F32, flags=flags)
        ctx.set_synthetic_grad(0.1, 0.0)
        free = {}
        for src in (0, 1, 2):
            ctx.set_launch_tuning(4, 8 if src == 2 else 1, 0, 0)
            free[src] = ctx.query_occupancy(src)
            assert 4 <= free[src] <= 32, (tiled, src, free[src])
        for cap in (2, 3, 5, 6, 8, 10, 12, 16):
            for src in (0, 1):                       # one wavefront per workgroup: the cap is met exactly
                ctx.set_launch_tuning(4, 1, cap, 0)
                assert ctx.query_occupancy(src) == min(cap, free[src]), (tiled, src, cap)
        # in-register gradient: workgroups of 8 wavefronts that also hold the 32 KB of noise cells; the cap is
        # rounded down to whole workgroups, and a workgroup cannot hold more than 64 KB of LDS, so two
        # workgroups always fit
        for cap in (8, 12, 16, 20, 24):
            ctx.set_launch_tuning(4, 8, cap, 0)
            assert ctx.query_occupancy(2) == min(max(2, cap // 8) * 8, free[2]), (tiled, cap)
        ctx.destroy()
    # built-in defaults (no tuning call): averaging alone is capped, the in-register round is not
    ctx = rps.RpsContext(32, 32 * 4096, 0.05, 0.1, 0, rps.RPS_DTYPE_F32, flags=rps.RPS_FLAG_LAYOUT_TILED)
    assert ctx.query_occupancy(0) == 11              # single wavefronts under the cap (about 44 KB in flight: 11 steps of 4 KB)
    assert ctx.query_occupancy(1) == 14              # gradient buffer: one workgroup of 14 as well
    assert ctx.query_occupancy(2) == 14              # 81-88 registers per lane: one workgroup of 14 wavefronts (measured best)
    ctx.destroy()
    ctx = rps.RpsContext(32, 32 * 4096, 0.05, 0.1, 0, rps.RPS_DTYPE_F32)
    assert ctx.query_occupancy(0) == 5 and ctx.query_occupancy(1) == 5
    ctx.destroy()


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("k", range(24))
def test_results_do_not_depend_on_the_launch_shape(rps, k):
    """rps_set_launch_tuning changes how the work is laid over wavefronts (rows per load chunk,
    workgroup width, occupancy cap, steps per wavefront), never what is computed: every entry point
    gives the same bits under three random launch shapes as under the built-in one, on seeded random
    workloads (workers, width, partition, dtype, drop rate, layout, server rule)."""
    import test_gpu_parity as P
    n, N, layout, dtype, p, tiled, identity, step0 = P._random_case(200 + k)
    off = P._offsets(n, N, layout, seed=k)
    flags = (rps.RPS_FLAG_LAYOUT_TILED if tiled else 0) | (rps.RPS_FLAG_SERVER_IDENTITY if identity else 0)
    code = rps.RPS_DTYPE_BF16 if dtype == "bf16" else rps.RPS_DTYPE_F32
    X0 = device_tensor(workloads.gaussian_model(n, N, seed=k), dtype)
    G0 = device_tensor(workloads.gaussian_model(n, N, seed=k + 500), dtype)
    if tiled:
        X0 = workloads.to_tiled(X0); G0 = workloads.to_tiled(G0)
    rng = np.random.default_rng(k)
    outs = []
    for variant in range(4):
        ctx = rps.RpsContext(n, N, p, 0.2, 900 + k, code, block_offsets=off, flags=flags)
        ctx.set_synthetic_grad(0.3, 0.02)
        if variant:
            ctx.set_launch_tuning(int(rng.choice([2, 4])), int(rng.choice([1, 2, 4, 8, 16])),
                                  int(rng.choice([0, 3, 5, 8, 12, 16, 24])), int(rng.choice([0, 1, 2, 3, 5])))
        X = X0.clone()
        ctx.round(X, None, step0); ctx.round(X, G0, step0 + 1); ctx.local_step(X, None, step0 + 2)
        ctx.lossy_average(X, step0 + 2); ctx.local_step(X, G0, step0 + 3); ctx.round_gradient_averaging(X, G0, step0 + 4)
        torch.cuda.synchronize()
        outs.append(X.clone())
        ctx.destroy()
    as_bits = torch.int16 if dtype == "bf16" else torch.int32
    for o in outs[1:]:
        assert torch.equal(o.view(as_bits), outs[0].view(as_bits)), (k, n, N, layout, dtype, p, tiled)
