"""Pins of the oracle's round (local step, Reduce-Scatter with drops, All-Gather with
drops) against what arXiv 1810.07766 and plain mathematics fix.  None of these tests
touches the HIP path."""
import numpy as np
import pytest
import torch

import workloads
from oracle import rps_oracle as oracle


def _random_masks(rng, n, p):
    """Arbitrary network outcome generated in the test (not by the oracle): a random
    permutation of servers, i.i.d. losses, reliable self links."""
    server = rng.permutation(n).astype(np.int32)
    U = (rng.random((n, n)) >= p).astype(np.uint8)
    D = (rng.random((n, n)) >= p).astype(np.uint8)
    U[server, np.arange(n)] = 1
    D[server, np.arange(n)] = 1
    return server, U, D


def _mixing_matrix(U, D, j):
    """W of Sec. 4.2, built here independently of the oracle: column k (worker k's result)
    is U[:, j]/|N_j| if the reply reached k, else e_k."""
    n = U.shape[0]
    W = np.eye(n)
    avg = U[:, j].astype(np.float64) / U[:, j].sum()
    for k in range(n):
        if D[k, j]:
            W[:, k] = avg
    return W


# -- local step ---------------------------------------------------------------------------------
def test_local_step_is_x_minus_gamma_g():
    """Alg. 1 step 5 / supplement relation V = X - gamma G, one rounding (fused multiply-add)."""
    rng = np.random.default_rng(0)
    X = rng.standard_normal((5, 1003)).astype(np.float32)
    G = rng.standard_normal((5, 1003)).astype(np.float32)
    gamma = np.float32(0.37)
    V = X.copy()
    oracle.local_step(V, G, float(gamma))
    exact = X.astype(np.float64) - np.float64(gamma) * G.astype(np.float64)   # product exact in f64
    ulp = np.spacing(np.abs(exact).astype(np.float32)).astype(np.float64)
    assert (np.abs(V - exact) <= 0.5 * ulp * (1 + 1e-6)).all()                 # correctly rounded


def test_synthetic_gradient_is_decay_plus_noise():
    n, N, gamma, sigma, lam = 3, 100, 0.5, 0.1, 0.25
    X = workloads.gaussian_model(n, N, seed=1)
    V = X.copy()
    oracle.local_step(V, None, gamma, sigma=sigma, weight_decay=lam, seed=8, step=6)
    for i in range(n):
        z = np.array([oracle.noise(8, 6, i, c, sigma) for c in range(N)], dtype=np.float64)
        exact = X[i].astype(np.float64) - gamma * (lam * X[i].astype(np.float64) + z)
        assert np.abs(V[i] - exact).max() < 2e-7 * (1 + np.abs(exact).max())


def test_column_subset_equals_full_run():
    n, N = 6, 960
    off = workloads.block_offsets(n, N)
    X = workloads.gaussian_model(n, N, seed=2)
    full = X.copy()
    m = oracle.round_(full, None, off, p=0.3, gamma=0.1, seed=4, step=9, sigma=0.2, weight_decay=0.01)
    cols = workloads.sample_columns(off, per_block=7, seed=3)
    sub = np.ascontiguousarray(X[:, cols])
    oracle.round_(sub, None, off, p=0.3, gamma=0.1, seed=4, step=9, sigma=0.2, weight_decay=0.01, cols=cols)
    assert (sub == full[:, cols]).all()


# -- special cases of the network ---------------------------------------------------------------
def test_no_loss_is_exact_averaging():
    """p = 0: Reduce-Scatter/All-Gather is the ordinary all-reduce average (Sec. 1, steps 1.1-1.2;
    W = A_n), so every worker ends with the column mean."""
    n, N = 8, 4000
    off = workloads.block_offsets(n, N)
    V = workloads.gaussian_model(n, N, seed=3)
    X = V.copy()
    server, U, D = oracle.masks(0, 0, n, 0.0)
    oracle.lossy_average(X, off, U, D)
    mean = V.astype(np.float64).mean(axis=0)
    assert np.abs(X - mean[None, :]).max() <= 6e-8 * np.abs(mean).max() + 1e-12
    assert (X == X[0:1]).all()


def test_total_loss_keeps_the_local_step():
    """p = 1: no message but a server's own arrives, so W = I and X_{t+1} = V_t bit for bit."""
    n, N = 8, 4000
    off = workloads.block_offsets(n, N)
    V = workloads.gaussian_model(n, N, seed=4)
    X = V.copy()
    server, U, D = oracle.masks(0, 5, n, 1.0)
    oracle.lossy_average(X, off, U, D)
    assert (X == V).all()


def test_lonely_server_broadcasts_its_own_block():
    """All uplinks of a block lost (the m = 0 term of the supplement's E[W11^2 | A] sum): the
    server averages only itself (weight 1) and still broadcasts."""
    n, N = 4, 400
    off = workloads.block_offsets(n, N)
    V = workloads.gaussian_model(n, N, seed=5)
    server = np.array([2, 0, 3, 1], dtype=np.int32)
    U = np.zeros((n, n), dtype=np.uint8); U[server, np.arange(n)] = 1
    D = np.ones((n, n), dtype=np.uint8)
    X = V.copy()
    oracle.lossy_average(X, off, U, D)
    for j in range(n):
        blk = slice(off[j], off[j + 1])
        assert (X[:, blk] == V[server[j], blk][None, :]).all()


@pytest.mark.parametrize("n,N,p,unequal", [(4, 1000, 0.3, False), (7, 7 * 33, 0.5, False), (16, 4096, 0.1, True)])
def test_receivers_agree_and_others_keep_v(n, N, p, unequal):
    """Supplement, Lemma 7 case 1: every node that received the averaged block holds the same
    value; a node that did not keeps its own v (eq. (dividex)).  Also the result is a convex
    combination (W is column-stochastic, Sec. 4.2)."""
    rng = np.random.default_rng(6)
    off = workloads.block_offsets(n, N, unequal=unequal, block_seed=3)
    V = workloads.gaussian_model(n, N, seed=7)
    server, U, D = _random_masks(rng, n, p)
    X = V.copy()
    oracle.lossy_average(X, off, U, D)
    for j in range(n):
        blk = slice(off[j], off[j + 1])
        recv = np.flatnonzero(D[:, j]); keep = np.flatnonzero(D[:, j] == 0)
        assert (X[recv][:, blk] == X[recv[0]][blk][None, :]).all()
        assert (X[keep][:, blk] == V[keep][:, blk]).all()
        contributors = np.flatnonzero(U[:, j])
        lo = V[contributors][:, blk].min(axis=0); hi = V[contributors][:, blk].max(axis=0)
        got = X[recv[0]][blk]
        assert ((got >= lo - 1e-7 * np.abs(lo)) & (got <= hi + 1e-7 * np.abs(hi))).all()


@pytest.mark.parametrize("n,p", [(3, 0.4), (8, 0.2), (33, 0.1)])
def test_loop_equals_global_view(n, p):
    """Sec. 4.2 eq. (updatingrule): X^{(j)}_{t+1} = V^{(j)}_t W^{(j)}_t, W not doubly stochastic."""
    rng = np.random.default_rng(8)
    N = n * 40
    off = workloads.block_offsets(n, N)
    V = workloads.gaussian_model(n, N, seed=9)
    server, U, D = _random_masks(rng, n, p)
    X = V.copy()
    oracle.lossy_average(X, off, U, D)
    doubly = True
    for j in range(n):
        W = _mixing_matrix(U, D, j)
        assert np.allclose(W.sum(axis=0), 1.0)                       # column-stochastic
        doubly &= np.allclose(W.sum(axis=1), 1.0)
        assert (oracle.build_W(j, U, D) == W).all()
        blk = slice(off[j], off[j + 1])
        Vj = V[:, blk].astype(np.float64).T                          # [len, n], columns = workers
        ref = (Vj @ W).T
        assert np.abs(X[:, blk] - ref).max() < 1e-6
    assert not doubly


def test_identity_input_reads_out_W():
    """With V^{(j)} = I_n the round's output is W itself: ties the loop to the matrix view."""
    n = 6
    rng = np.random.default_rng(10)
    off = workloads.block_offsets(n, n * n)
    V = np.tile(np.eye(n, dtype=np.float32), (1, n))
    server, U, D = _random_masks(rng, n, 0.4)
    X = V.copy()
    oracle.lossy_average(X, off, U, D)
    for j in range(n):
        W = X[:, off[j]:off[j + 1]].astype(np.float64).T
        assert np.abs(W - _mixing_matrix(U, D, j)).max() < 1e-7


# -- storage formats ---------------------------------------------------------------------------
def test_bf16_storage_rounds_to_nearest_even():
    n, N = 4, 2048
    off = workloads.block_offsets(n, N)
    Vf = workloads.gaussian_model(n, N, seed=11)
    Vb = workloads.to_bf16_bits(Vf)                                   # torch's RNE conversion
    Gb = workloads.to_bf16_bits(workloads.gaussian_model(n, N, seed=12))
    X = Vb.copy()
    oracle.local_step(X, Gb, 0.5)
    exact = workloads.from_bf16_bits(Vb).astype(np.float64) - 0.5 * workloads.from_bf16_bits(Gb).astype(np.float64)
    ref = torch.from_numpy(exact.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    # float32 rounding of `exact` before bf16 rounding can differ from a single rounding only at ties
    assert (X != ref).mean() < 1e-3
    assert np.abs(workloads.from_bf16_bits(X) - exact).max() <= 2.0 ** -8 * np.abs(exact).max()
    V = X.copy()
    server, U, D = oracle.masks(0, 0, n, 0.0)
    oracle.lossy_average(X, off, U, D)
    mean = workloads.from_bf16_bits(V).astype(np.float64).mean(axis=0)
    refm = torch.from_numpy(mean.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (X == refm[None, :]).all()


# -- quadratic objective -----------------------------------------------------------------------
def test_least_squares_matches_closed_form_gradient_descent():
    """Config-1-shaped problem (smaller): f_i(x) = 0.5 ||A_i x - b_i||^2.  With p = 0 and an
    identical start every worker follows x <- x - gamma (1/n) sum_i A_i^T (A_i x - b_i)
    (Sec. 4.1 local step + exact averaging); iterate that in double and compare."""
    n, N, rows, gamma, T = 4, 1000, 64, 0.05, 30
    off = workloads.block_offsets(n, N)
    A, b = workloads.least_squares_problem(n, N, rows, seed=13)
    X = np.zeros((n, N), dtype=np.float32)
    x = np.zeros(N)
    for t in range(T):
        G = np.stack([A[i].T @ (A[i] @ X[i].astype(np.float64) - b[i]) for i in range(n)]).astype(np.float32)
        oracle.round_(X, G, off, p=0.0, gamma=gamma, seed=0, step=t)
        x = x - gamma * np.mean([A[i].T @ (A[i] @ x - b[i]) for i in range(n)], axis=0)
        assert (X == X[0:1]).all()
    assert np.abs(X[0] - x).max() < 1e-5 * np.abs(x).max()
    # with loss, every worker's intermediate model is still its own closed-form gradient step
    X = workloads.gaussian_model(n, N, seed=14, scale=0.1)
    G = np.stack([A[i].T @ (A[i] @ X[i].astype(np.float64) - b[i]) for i in range(n)]).astype(np.float32)
    V = X.copy()
    oracle.local_step(V, G, gamma)
    assert np.abs(V - (X.astype(np.float64) - gamma * G.astype(np.float64))).max() < 1e-7


def test_rounds_are_stateless_so_resume_is_exact():
    n, N = 5, 500
    off = workloads.block_offsets(n, N)
    X0 = workloads.gaussian_model(n, N, seed=15)
    kw = dict(p=0.2, gamma=0.1, seed=77, sigma=0.1, weight_decay=1e-3)
    A = X0.copy()
    for t in range(10):
        oracle.round_(A, None, off, step=t, **kw)
    B = X0.copy()
    for t in range(5):
        oracle.round_(B, None, off, step=t, **kw)
    B = B.copy()                                                     # "reload"
    for t in range(5, 10):
        oracle.round_(B, None, off, step=t, **kw)
    assert (A == B).all()


def test_averaging_contracts_disagreement():
    """The consensus distance sum_i ||x_i - xbar||^2 (supplement, Lemma 1) shrinks under a round
    without gradients, by about beta = alpha_1 - alpha_2 in expectation."""
    n, N = 16, 16 * 500
    off = workloads.block_offsets(n, N)
    X = workloads.gaussian_model(n, N, seed=16)
    def dist(Y):
        Y = Y.astype(np.float64); return ((Y - Y.mean(axis=0)) ** 2).sum()
    d0 = dist(X)
    server, U, D = oracle.masks(1, 0, n, 0.1)
    oracle.lossy_average(X, off, U, D)
    assert dist(X) < 0.25 * d0                                       # beta ~ p for small p


def test_gradient_averaging_variant_special_cases_and_drift():
    """Sec. 6's comparison: averaging GRADIENTS under loss.  p = 0: every worker applies the mean
    gradient (identical workers stay identical); p = 1: plain local steps.  With loss, workers
    that start identical drift apart and nothing contracts the disagreement again, while model
    averaging (RPS) keeps it bounded: the mechanism behind the paper's 'worse convergence'."""
    n, N, rows, gamma = 4, 400, 32, 0.05
    off = workloads.block_offsets(n, N)
    A, b = workloads.least_squares_problem(n, N, rows, seed=31)
    grad = lambda X: np.stack([A[i].T @ (A[i] @ X[i].astype(np.float64) - b[i]) for i in range(n)]).astype(np.float32)
    X = workloads.gaussian_model(n, N, seed=32, identical=True)
    G = grad(X)
    Y = X.copy()
    oracle.round_gradient_averaging(Y, G, off, p=0.0, gamma=gamma, seed=0, step=0)
    ref = X[0].astype(np.float64) - gamma * G.astype(np.float64).mean(axis=0)
    assert (Y == Y[0:1]).all() and np.abs(Y[0] - ref).max() < 1e-6
    Y = X.copy(); Z = X.copy()
    oracle.round_gradient_averaging(Y, G, off, p=1.0, gamma=gamma, seed=0, step=0)
    oracle.local_step(Z, G, gamma)
    assert (Y == Z).all()
    Xg = X.copy(); Xm = X.copy()
    dg, dm = [], []
    for t in range(300):
        oracle.round_gradient_averaging(Xg, grad(Xg), off, p=0.2, gamma=gamma, seed=5, step=t)
        oracle.round_(Xm, grad(Xm), off, p=0.2, gamma=gamma, seed=5, step=t)
        dg.append(oracle.consensus(Xg)[0]); dm.append(oracle.consensus(Xm)[0])
    assert dg[-1] > 20 * dm[-1]                     # gradient averaging: disagreement accumulates
    assert max(dm[100:]) < 10 * np.mean(dm[50:100]) # model averaging: bounded steady state


def test_gradient_averaging_is_x_minus_gamma_g_times_w():
    """Sec. 6's gradient averaging in the global view of Sec. 4.2: the network acts on the gradients
    exactly as it acts on models, G~ = G W per block, and then X' = X - gamma G~.  W is rebuilt here
    (not by the oracle); checked for random outcomes and, by enumerating every (server, uplink,
    downlink) outcome of a block for n = 3, in expectation: E[W] = a0 I + (1 - a0) A_n preserves the
    mean, so E[mean_i x'_i] = xbar - gamma gbar, the same unbiasedness as model averaging
    (supplement, Lemma 3's first identity) -- what differs is that nothing contracts the spread."""
    import itertools
    rng = np.random.default_rng(7)
    n, N, gamma = 6, 6 * 40, 0.3
    off = workloads.block_offsets(n, N)
    X = rng.standard_normal((n, N)).astype(np.float32)
    G = rng.standard_normal((n, N)).astype(np.float32)
    for trial in range(5):
        server, U, D = _random_masks(rng, n, 0.35)
        Y = X.copy()
        oracle.round_gradient_averaging(Y, G, off, p=0.0, gamma=gamma, seed=0, step=0, mask_override=(server, U, D))
        for j in range(n):
            blk = slice(off[j], off[j + 1])
            W = _mixing_matrix(U, D, j)
            # the averaged gradient travels in fp32: one rounding of the column means, then one fused step
            Gt = (G[:, blk].astype(np.float64).T @ W).T.astype(np.float32)
            ref = X[:, blk].astype(np.float64) - gamma * Gt.astype(np.float64)
            assert np.abs(Y[:, blk] - ref).max() < 2e-6
    # expectation over every outcome of one block, n = 3, p = 0.25
    n, p, q = 3, 0.25, 0.75
    X = rng.standard_normal((n, 8)).astype(np.float32)
    G = rng.standard_normal((n, 8)).astype(np.float32)
    acc = np.zeros(8); total = 0.0
    for s in range(n):
        others = [i for i in range(n) if i != s]
        for ubits in itertools.product((0, 1), repeat=n - 1):
            for dbits in itertools.product((0, 1), repeat=n - 1):
                U = np.zeros((n, 1), dtype=np.uint8); D = np.zeros((n, 1), dtype=np.uint8)
                U[s, 0] = D[s, 0] = 1
                for i, u, d in zip(others, ubits, dbits):
                    U[i, 0], D[i, 0] = u, d
                prob = (1.0 / n) * np.prod([q if b else p for b in ubits + dbits])
                W = _mixing_matrix(U, D, 0)
                Xp = X.astype(np.float64) - gamma * (G.astype(np.float64).T @ W).T
                acc += prob * Xp.mean(axis=0); total += prob
    assert abs(total - 1.0) < 1e-12
    want = X.astype(np.float64).mean(axis=0) - gamma * G.astype(np.float64).mean(axis=0)
    assert np.abs(acc - want).max() < 1e-12
