"""Brute-force pins: enumerate EVERY network outcome of one block on tiny n through the
oracle's own round and compare with the formulas printed in arXiv 1810.07766:

  - E[W] A_n = A_n,  E[W W^T] = a1 I + (1-a1) A_n,  E[W A_n W^T] = a2 I + (1-a2) A_n,
    0 < a2 < a1 < 1                                   (Sec. 4.2, eqs. (def_alpha1), (def_alpha2))
  - a1 = (n E[sum_i W_1i^2] - 1)/(n-1),  a2 = (E[(sum_i W_1i)^2] - 1)/(n-1)
                                                      (supplement, Lemmas 7 and 8)
  - the exact conditional binomial sums for E[W11^2 | A], E[W1n^2 | not A, C],
    E[W1n | not A, C] and the probabilities P(A) = 1/n, P(not A, C) = p(n-1)/n   (same proofs)
  - the printed upper bounds on a1 and a2 (n >= 3: the proofs' sums assume it)
  - E_P[dxbar] = -gamma gbar and the second-moment identity     (supplement, Lemma 3)

The outcome space of one block: the server s (uniform over the n workers, Alg. 1 step 6),
an uplink pattern and a downlink pattern over the other n-1 workers (independent losses
with probability p, Sec. 3); the server's own links are reliable.
"""
import itertools
from math import comb

import numpy as np
import pytest

import workloads
from oracle import rps_oracle as oracle


def enumerate_block(n, p):
    """Yields (probability, server, W) over all outcomes; W is read out of the oracle's round
    by feeding it V^{(j)} = I_n (then X_{t+1}^{(j)} = W)."""
    q = 1.0 - p
    off = np.array([0] + [n] * n, dtype=np.int64)        # block 0 holds all n columns
    eye = np.eye(n, dtype=np.float32)
    for s in range(n):
        others = [i for i in range(n) if i != s]
        for up in itertools.product((0, 1), repeat=n - 1):
            for dn in itertools.product((0, 1), repeat=n - 1):
                U = np.zeros((n, n), dtype=np.uint8); D = np.zeros((n, n), dtype=np.uint8)
                U[s, 0] = D[s, 0] = 1
                for o, u, d in zip(others, up, dn):
                    U[o, 0] = u; D[o, 0] = d
                prob = (1.0 / n) * np.prod([q if b else p for b in up + dn])
                X = eye.copy()
                oracle.lossy_average(X, off, U, D)
                yield prob, s, D[:, 0].copy(), X.astype(np.float64).T     # X[k, m] = W[m, k]


def moments(n, p):
    A = np.full((n, n), 1.0 / n)
    EW = np.zeros((n, n)); EWW = np.zeros((n, n)); EWAW = np.zeros((n, n)); tot = 0.0
    for prob, s, d, W in enumerate_block(n, p):
        tot += prob; EW += prob * W; EWW += prob * W @ W.T; EWAW += prob * W @ A @ W.T
    assert abs(tot - 1.0) < 1e-12
    return EW, EWW, EWAW


def alpha_of(M, n):
    """M = a I + (1-a) A_n  =>  a from the (1,1) entry; also checks the whole structure."""
    a = (n * M[0, 0] - 1.0) / (n - 1.0)
    assert np.abs(M - (a * np.eye(n) + (1 - a) * np.full((n, n), 1.0 / n))).max() < 1e-6
    return a


# exact (unrelaxed) expressions from the case analysis of Lemmas 7 and 8
def E_W11sq_given_A(n, p):
    q = 1 - p
    return sum(comb(n - 1, m) * q ** m * p ** (n - 1 - m) / (m + 1) ** 2 for m in range(n))


def E_W1nsq_given_notA_C(n, p):
    q = 1 - p
    return sum(comb(n - 2, m) * q ** (m + 1) * p ** (n - 2 - m) / (m + 2) ** 2 for m in range(n - 1))


def E_W1n_given_notA_C(n, p):
    q = 1 - p
    return sum(comb(n - 2, m) * q ** (m + 1) * p ** (n - 2 - m) / (m + 2) for m in range(n - 1))


def alpha1_exact(n, p):
    q = 1 - p
    c1 = E_W11sq_given_A(n, p) * (1 + (n - 1) * q)
    c2 = 1 + E_W1nsq_given_notA_C(n, p) * (1 + (n - 2) * q)
    c3 = E_W1nsq_given_notA_C(n, p) * (2 + (n - 2) * q)
    e = c1 / n + c2 * p * (n - 1) / n + c3 * q * (n - 1) / n
    return (n * e - 1) / (n - 1)


def alpha2_exact(n, p):
    q = 1 - p
    c1 = E_W11sq_given_A(n, p) * ((1 + (n - 1) * q) ** 2 + (n - 1) * p * q)
    c2 = (1 + 2 * E_W1n_given_notA_C(n, p) * ((n - 2) * q + 1)
          + E_W1nsq_given_notA_C(n, p) * (1 + 2 * (n - 2) * q + (n - 2) ** 2 * q ** 2 + (n - 2) * p * q))
    c3 = E_W1nsq_given_notA_C(n, p) * (((n - 2) * q + 2) ** 2 + (n - 2) * p * q)
    e = c1 / n + c2 * p * (n - 1) / n + c3 * q * (n - 1) / n
    return (e - 1) / (n - 1)


@pytest.mark.parametrize("n,p", [(2, 0.3), (3, 0.1), (3, 0.5), (4, 0.1), (5, 0.2)])
def test_moment_structure_and_alpha_formulas(n, p):
    EW, EWW, EWAW = moments(n, p)
    A = np.full((n, n), 1.0 / n)
    assert np.abs(EW @ A - A).max() < 1e-7                       # (E W) A_n = A_n
    a0 = alpha_of(EW, n); a1 = alpha_of(EWW, n); a2 = alpha_of(EWAW, n)
    assert 0 < a2 < a1 < 1
    assert abs(a1 - alpha1_exact(n, p)) < 1e-6
    assert abs(a2 - alpha2_exact(n, p)) < 1e-6
    # the lemmas' row formulas
    e_sq = e_sum_sq = 0.0
    for prob, s, d, W in enumerate_block(n, p):
        e_sq += prob * (W[0] ** 2).sum(); e_sum_sq += prob * W[0].sum() ** 2
    assert abs(a1 - (n * e_sq - 1) / (n - 1)) < 1e-6
    assert abs(a2 - (e_sum_sq - 1) / (n - 1)) < 1e-6
    assert a0 > 0


@pytest.mark.parametrize("n,p", [(3, 0.25), (4, 0.1), (5, 0.4)])
def test_conditional_sums_of_the_proofs(n, p):
    PA = PnAC = 0.0; w11 = w1n = w1n1 = 0.0
    for prob, s, d, W in enumerate_block(n, p):
        if s == 0:                                   # event A: node 1 serves the block
            PA += prob; w11 += prob * W[0, 0] ** 2
        elif s == n - 1 and d[0] == 0:               # server is node n, node 1 got no reply (C)
            PnAC += prob; w1n += prob * W[0, n - 1] ** 2; w1n1 += prob * W[0, n - 1]
    assert abs(PA - 1.0 / n) < 1e-12
    assert abs(PnAC - p / n) < 1e-12                 # one of the n-1 equally likely servers
    assert abs(w11 / PA - E_W11sq_given_A(n, p)) < 1e-7
    assert abs(w1n / PnAC - E_W1nsq_given_notA_C(n, p)) < 1e-7
    assert abs(w1n1 / PnAC - E_W1n_given_notA_C(n, p)) < 1e-7


def test_closed_forms_for_two_workers():
    """n = 2 by hand (q = 1-p).  Server = node 1 (prob 1/2): W11 = 1/2 if node 2's copy arrives
    (q) else 1; W12 = W11 if node 2 gets the reply (q) else 0.  Server = node 2: W12 = 1/2 if
    node 1's copy arrives else 0; W11 = W12 if node 1 gets the reply else 1.  Summing:
    E[W11] = (1 + a0)/2 with a0 = p(1+p)/2;  a1 = 2 E[sum W1i^2] - 1 = 1.5 p - 0.5 p^2;
    a2 = E[(sum W1i)^2] - 1 = 1.25 p (1-p)."""
    for p in (0.05, 0.3, 0.9):
        EW, EWW, EWAW = moments(2, p)
        assert abs(alpha_of(EW, 2) - 0.5 * p * (1 + p)) < 1e-7
        assert abs(alpha_of(EWW, 2) - (1.5 * p - 0.5 * p * p)) < 1e-7
        assert abs(alpha_of(EWAW, 2) - 1.25 * p * (1 - p)) < 1e-7


@pytest.mark.parametrize("n,p", [(3, 0.1), (4, 0.2), (5, 0.05), (16, 0.1), (32, 0.05), (64, 0.1)])
def test_printed_upper_bounds_hold(n, p):
    q = 1 - p
    T1 = 2 * (1 - p ** (n + 1) - (n + 1) * q * p ** n - (n + 1) * n * q * q * p ** (n - 1) / 2 - q ** (n + 1)) / (n * (n + 1) * q * q)
    T2 = (1 - p ** n - n * q * p ** (n - 1) - q ** n) / ((n - 1) * q)
    T3 = n / (n - 1) * (1 - p ** (n - 1) - q ** (n - 1)) + q ** (n - 1)
    a1, a2 = alpha1_exact(n, p), alpha2_exact(n, p)
    assert a1 <= (n * p + q ** n + n * T1 + n * T2 - 1) / (n - 1) + 1e-12
    assert a2 <= (p * (1 + 2 * T3) + q ** (n - 1)) / n + 2 * p * q ** n / n + p ** n * q / n ** 2 + T1 + T2 + 1e-12
    assert 0 < a2 < a1 < 1


def test_expected_update_formula():
    """Supplement, Lemma 3: over the drop randomness of round t,
    E[dxbar] = -gamma gbar  and  E||dxbar||^2 = (a2/n) sum_j Tr(V^(j) (I - A_n) V^(j)T) + gamma^2 ||gbar||^2,
    checked per block by enumerating every outcome of the oracle's round on random X, G."""
    n, width, p, gamma = 4, 3, 0.3, 0.2
    rng = np.random.default_rng(5)
    Xb = rng.standard_normal((n, width)).astype(np.float32)       # one block, [workers, width]
    Gb = rng.standard_normal((n, width)).astype(np.float32)
    V = Xb.copy()
    oracle.local_step(V, Gb, gamma)
    Vd = V.astype(np.float64)
    xbar = Xb.astype(np.float64).mean(axis=0); gbar = Gb.astype(np.float64).mean(axis=0)
    off = np.array([0] + [width] * n, dtype=np.int64)
    q = 1 - p
    e1 = np.zeros(width); e2 = 0.0
    for s in range(n):
        others = [i for i in range(n) if i != s]
        for up in itertools.product((0, 1), repeat=n - 1):
            for dn in itertools.product((0, 1), repeat=n - 1):
                U = np.zeros((n, n), dtype=np.uint8); D = np.zeros((n, n), dtype=np.uint8)
                U[s, 0] = D[s, 0] = 1
                for o, u, d in zip(others, up, dn):
                    U[o, 0] = u; D[o, 0] = d
                prob = (1.0 / n) * np.prod([q if b else p for b in up + dn])
                Y = V.copy()
                oracle.lossy_average(Y, off, U, D)
                dx = Y.astype(np.float64).mean(axis=0) - xbar
                e1 += prob * dx; e2 += prob * (dx ** 2).sum()
    assert np.abs(e1 + gamma * gbar).max() < 1e-6
    a2 = alpha2_exact(n, p)
    tr = ((Vd - Vd.mean(axis=0)) ** 2).sum()                       # Tr(V^T (I - A_n) V)
    assert abs(e2 - (a2 / n * tr + gamma ** 2 * (gbar ** 2).sum())) < 1e-6


def test_fixed_server_breaks_the_mean_preservation():
    """Why Alg. 1 draws the server afresh: with the server fixed the expected mixing matrix is
    not of the a I + (1-a) A_n form (the server's copy is over-weighted), so E[dxbar] != -gamma gbar
    per block.  Conditioning the enumeration on s = 0 shows it."""
    n, p = 3, 0.2
    EW = np.zeros((n, n)); tot = 0.0
    for prob, s, d, W in enumerate_block(n, p):
        if s == 0:
            EW += prob * W; tot += prob
    EW /= tot
    rows = EW.sum(axis=1)
    assert rows[0] > 1.01 and rows[1] < 0.99 and abs(rows.sum() - n) < 1e-6


@pytest.mark.parametrize("n,p", [(16, 0.1), (32, 0.05)])
def test_generated_masks_reproduce_alpha2(n, p):
    """Monte-Carlo over the oracle's own mask generator at benchmark sizes: the sample mean of
    (sum_i W_1i)^2 gives a2 (Lemma 8); a2 n / (p (1-p)) stays O(1) (Sec. 5: a2 = O(p(1-p)/n))."""
    vals = []
    for step in range(1500):
        server, U, D = oracle.masks(123, step, n, p)
        cnt = U.sum(axis=0).astype(np.float64)                     # |N_j|
        # row 1 of W^(j): W[0,k] = U[0,j]/cnt_j if D[k,j] else (k == 0)
        recv = D.sum(axis=0).astype(np.float64)
        row_sum = U[0] / cnt * recv + (1 - D[0])
        vals.append(row_sum ** 2)
    vals = np.concatenate(vals)
    est = (vals.mean() - 1) / (n - 1)
    se = vals.std() / np.sqrt(vals.size) / (n - 1)
    exact = alpha2_exact(n, p)
    assert abs(est - exact) < 5 * se
    assert 0.5 < exact * n / (p * (1 - p)) < 4.0


def test_consensus_distance_definition_and_contraction():
    """sum_i ||x_i - xbar||^2 = ||X (I - A_n)||_F^2 = Tr(X (I - A_n) X^T) (supplement, proof of Lemma 1),
    and over the drop randomness of one round E||X W (I - A_n)||_F^2 = (a1 - a2) ||X (I - A_n)||_F^2
    (same proof: E[W (I - A_n) W^T] = (a1 - a2)(I - A_n)), checked by enumerating every outcome."""
    n, width, p = 4, 5, 0.3
    rng = np.random.default_rng(9)
    V = rng.standard_normal((n, width)).astype(np.float32)
    Vd = V.astype(np.float64).T                                   # columns = workers
    A = np.full((n, n), 1.0 / n)
    d0, m0 = oracle.consensus(V)
    assert abs(d0 - np.trace(Vd @ (np.eye(n) - A) @ Vd.T)) < 1e-12 * d0
    assert abs((V.astype(np.float64) ** 2).sum() - (d0 + n * m0)) < 1e-12 * d0      # Pythagoras
    same = np.tile(V[0:1], (n, 1))
    assert oracle.consensus(same)[0] == 0.0
    off = np.array([0] + [width] * n, dtype=np.int64)
    q = 1 - p
    expect = 0.0
    for s in range(n):
        others = [i for i in range(n) if i != s]
        for up in itertools.product((0, 1), repeat=n - 1):
            for dn in itertools.product((0, 1), repeat=n - 1):
                U = np.zeros((n, n), dtype=np.uint8); D = np.zeros((n, n), dtype=np.uint8)
                U[s, 0] = D[s, 0] = 1
                for o, u, d in zip(others, up, dn):
                    U[o, 0] = u; D[o, 0] = d
                prob = (1.0 / n) * np.prod([q if b else p for b in up + dn])
                Y = V.copy()
                oracle.lossy_average(Y, off, U, D)
                expect += prob * oracle.consensus(Y)[0]
    beta = alpha1_exact(n, p) - alpha2_exact(n, p)
    assert abs(expect - beta * d0) < 1e-5 * d0


@pytest.mark.parametrize("n,p", [(2, 0.3), (3, 0.2), (4, 0.5)])
def test_external_servers_expected_mixing(n, p):
    """Parameter servers that are not workers (the paper's Fig. 1: three servers, four workers; its
    footnote: the analysis extends to any numbers).  No link is reliable.  Enumerating all 4^n
    outcomes of one block: W is column-stochastic, and by exchangeability E[W] = a I + (1-a) A_n.
    By hand (q = 1-p): worker k keeps its own block if its reply is lost (p) or the server got
    nothing (q p^n); otherwise its column is U/|N|, and E[U_k/|N| ; |N|>0] = (1 - p^n)/n by
    symmetry.  So E[W_kk] = p + q p^n + q (1 - p^n)/n and E[W_mk] = q (1 - p^n)/n for m != k."""
    q = 1 - p
    off = np.array([0, n], dtype=np.int64)                      # one block of n columns, one server
    eye = np.eye(n, dtype=np.float32)
    EW = np.zeros((n, n)); tot = 0.0
    for up in itertools.product((0, 1), repeat=n):
        for dn in itertools.product((0, 1), repeat=n):
            U = np.array(up, dtype=np.uint8).reshape(n, 1); D = np.array(dn, dtype=np.uint8).reshape(n, 1)
            prob = np.prod([q if b else p for b in up + dn])
            X = eye.copy()
            oracle.lossy_average(X, off, U, D)
            W = X.astype(np.float64).T
            assert np.allclose(W.sum(axis=0), 1.0, atol=1e-6)   # column-stochastic, also when empty
            assert np.abs(W - oracle.build_W(0, U, D)).max() < 1e-6
            if sum(up) == 0:
                assert (X == eye).all()                         # server got nothing: nobody changes
            EW += prob * W; tot += prob
    assert abs(tot - 1) < 1e-12
    off_diag = q * (1 - p ** n) / n
    diag = p + q * p ** n + off_diag
    assert np.abs(np.diag(EW) - diag).max() < 1e-6
    assert np.abs(EW - np.diag(np.diag(EW)) - off_diag * (1 - np.eye(n))).max() < 1e-6
    assert np.allclose(EW.sum(axis=1), 1.0, atol=1e-6)          # mean preserved in expectation


def _alpha_table():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "alpha_table.txt")
    rows = [ln.split() for ln in open(path) if not ln.startswith("#")]
    return {(int(r[0]), float(r[1])): (float(r[2]), float(r[3]), float(r[4])) for r in rows}


def test_alpha_table_against_the_lemmas_sums_and_the_papers_trends():
    """The stored table (full enumeration through the oracle, tests/golden/make_alpha_table.py) against
    the exact binomial sums of the supplement's Lemmas 7 and 8 typed out above, the ordering
    0 < a2 < a1 < 1 (Sec. 4.2), and what the paper reads off Fig. 2 / Fig. 3 (Sec. 5): a2 shrinks
    as the network grows at fixed p (a2 = O(p(1-p)/n)), beta = a1 - a2 grows with p (beta = O(p))."""
    tab = _alpha_table()
    ns = sorted({k[0] for k in tab}); ps = sorted({k[1] for k in tab})
    assert len(tab) == len(ns) * len(ps) >= 30
    for (n, p), (a1, a2, beta) in tab.items():
        assert abs(a1 - alpha1_exact(n, p)) < 1e-11 and abs(a2 - alpha2_exact(n, p)) < 1e-11
        assert 0 < a2 < a1 < 1 and abs(beta - (a1 - a2)) < 1e-12
        assert a2 * n / (p * (1 - p)) < 4.0 and beta / p < 1.0
    for p in ps:
        a2s = [tab[(n, p)][1] for n in ns]
        assert all(x > y for x, y in zip(a2s, a2s[1:]))
    for n in ns:
        betas = [tab[(n, p)][2] for p in ps]
        assert all(x < y for x, y in zip(betas, betas[1:]))


@pytest.mark.parametrize("n,p,identity", [(4, 0.1, False), (3, 0.2, False), (5, 0.05, True)])
def test_monte_carlo_estimator_converges_to_the_table(n, p, identity):
    """oracle.estimate_mixing (definition-level averages of W W^T and W A_n W^T over generated
    outcomes) against the enumerated constants, within 5 batch standard errors.  A fixed server
    map gives the same constants: the second moments of one block's W do not depend on which
    worker serves it once averaged over rows."""
    a1_ref, a2_ref, _ = _alpha_table()[(n, p)]
    batches = np.array([oracle.estimate_mixing(77, 400 * b, 400, n, p, identity_server=identity) for b in range(12)])
    est = batches.mean(axis=0); se = batches.std(axis=0, ddof=1) / np.sqrt(len(batches))
    assert abs(est[0] - a1_ref) < 5 * se[0] and se[0] < 0.05 * a1_ref
    assert abs(est[1] - a2_ref) < 5 * se[1] and se[1] < 0.05 * a2_ref


def test_alpha_grid_file():
    """tests/golden/alpha_grid.txt (the (n, p) grid of the paper's Fig. 2 / Fig. 3 at the benchmark
    worker counts, written by tests/golden/make_alpha_grid.py): its exact columns against this file's
    own typing of the Lemma 7 / Lemma 8 sums (pinned above to full enumeration for small n), its
    oracle Monte-Carlo columns within 5 standard errors of them, and the figures' trends."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "alpha_grid.txt")
    rows = [line.split() for line in open(path) if not line.startswith("#")]
    assert len(rows) == 20
    table = {}
    for v in rows:
        n, p = int(v[0]), float(v[1])
        a1, a2, beta, m1, s1, m2, s2 = (float(x) for x in v[2:9])
        assert abs(a1 - alpha1_exact(n, p)) < 1e-10 and abs(a2 - alpha2_exact(n, p)) < 1e-10
        assert abs(beta - (a1 - a2)) < 1e-12
        assert abs(m1 - a1) < 5 * s1 and abs(m2 - a2) < 5 * s2, (n, p)
        assert 0 < a2 < a1 < 1
        table[(n, p)] = (a1, a2, beta)
    for p in (0.01, 0.05, 0.1, 0.2):
        a2s = [table[(n, p)][1] for n in (4, 8, 16, 32, 64)]
        assert all(x > y for x, y in zip(a2s, a2s[1:]))
    for n in (4, 8, 16, 32, 64):
        betas = [table[(n, p)][2] for p in (0.01, 0.05, 0.1, 0.2)]
        assert all(x < y for x, y in zip(betas, betas[1:]))
    # the survey's reference values
    assert abs(table[(32, 0.05)][0] - 0.050053) < 1e-6 and abs(table[(64, 0.1)][1] - 0.002818) < 1e-6
