"""Writes tests/golden/alpha_grid.txt: the mixing constants alpha1, alpha2 and beta = alpha1 - alpha2
of arXiv 1810.07766 (Sec. 4.2, eqs. (def_alpha1), (def_alpha2)) on the grid of worker counts and
drop rates that the paper's Fig. 2 (alpha2 over n and p) and Fig. 3 (beta over n and p) cover, at
the sizes the benchmark workloads use.

Two independent columns per constant:
  exact   the closed sums of the supplement's case analysis (Lemma 7: E[sum_i W_1i^2], Lemma 8:
          E[(sum_i W_1i)^2]; cases: worker 1 is the server / is not and its uplink is lost / is not
          and its uplink arrives), written out here.  tests/test_oracle_moments.py pins the same sums
          to full enumeration of every network outcome for n <= 7.
  oracle  Monte-Carlo over the outcomes the CPU oracle generates (its masks -> its mixing matrices ->
          averages of W W^T and W A_n W^T), with its standard error over 16 batches.

Calls only oracle/ (never the HIP library).  Run from the repository root:
    python tests/golden/make_alpha_grid.py
"""
import os
import sys
from math import comb

import numpy as np

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", ".."))
from oracle import rps_oracle as oracle  # noqa: E402

GRID_N = (4, 8, 16, 32, 64)
GRID_P = (0.01, 0.05, 0.1, 0.2)
SEED = 20241128
BATCHES = 16


def exact_alphas(n, p):
    """alpha1 = (n e1 - 1)/(n - 1), alpha2 = (e2 - 1)/(n - 1) with e1 = E[sum_i W_1i^2] and
    e2 = E[(sum_i W_1i)^2] of one block, row 1 of W being the weights of worker 1's copy."""
    q = 1.0 - p
    # worker 1 is the server (probability 1/n): m of the other n-1 copies arrive, weight 1/(m+1)
    w11 = sum(comb(n - 1, m) * q ** m * p ** (n - 1 - m) / (m + 1) ** 2 for m in range(n))
    # worker 1 is not the server and its copy arrives: m of the other n-2 non-server copies arrive
    w1n_sq = sum(comb(n - 2, m) * q ** (m + 1) * p ** (n - 2 - m) / (m + 2) ** 2 for m in range(n - 1))
    w1n = sum(comb(n - 2, m) * q ** (m + 1) * p ** (n - 2 - m) / (m + 2) for m in range(n - 1))
    # number of receivers: the server plus Binomial(n-1, q) (server case) or the server, plus
    # Binomial(n-2, q), plus worker 1 itself if its reply arrives (non-server cases)
    e1 = (w11 * (1 + (n - 1) * q)
          + (1 + w1n_sq * (1 + (n - 2) * q)) * p * (n - 1)
          + w1n_sq * (2 + (n - 2) * q) * q * (n - 1)) / n
    e2 = (w11 * ((1 + (n - 1) * q) ** 2 + (n - 1) * p * q)
          + (1 + 2 * w1n * ((n - 2) * q + 1)
             + w1n_sq * (1 + 2 * (n - 2) * q + (n - 2) ** 2 * q * q + (n - 2) * p * q)) * p * (n - 1)
          + w1n_sq * (((n - 2) * q + 2) ** 2 + (n - 2) * p * q) * q * (n - 1)) / n
    return (n * e1 - 1) / (n - 1), (e2 - 1) / (n - 1)


def oracle_alphas(n, p, rounds_per_batch):
    est = np.array([oracle.estimate_mixing(SEED, b * rounds_per_batch, rounds_per_batch, n, p) for b in range(BATCHES)])
    return est.mean(axis=0), est.std(axis=0, ddof=1) / np.sqrt(BATCHES)


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "alpha_grid.txt")
    with open(out, "w") as f:
        f.write("# alpha1, alpha2, beta = alpha1 - alpha2 of the RPS mixing matrix (arXiv 1810.07766, Sec. 4.2,\n"
                "# eqs. (def_alpha1), (def_alpha2); the grid of Fig. 2 (alpha2) and Fig. 3 (beta)): exact sums of the\n"
                "# supplement's Lemmas 7 and 8, and a Monte-Carlo estimate from the CPU oracle's own outcomes\n"
                f"# (seed {SEED}, {BATCHES} batches) with its standard error.  Written by tests/golden/make_alpha_grid.py.\n"
                "# n p alpha1_exact alpha2_exact beta_exact alpha1_oracle se alpha2_oracle se samples\n")
        for n in GRID_N:
            rounds = max(6, 1536 // n)                    # per batch; every round has n blocks = n samples of W
            for p in GRID_P:
                a1, a2 = exact_alphas(n, p)
                (m1, m2), (s1, s2) = oracle_alphas(n, p, rounds)
                f.write(f"{n} {p} {a1:.12e} {a2:.12e} {a1 - a2:.12e} {m1:.6e} {s1:.2e} {m2:.6e} {s2:.2e} {BATCHES * rounds * n}\n")
                print(n, p, a1, a2, m1, s1, m2, s2, flush=True)
    print("wrote", out)


if __name__ == "__main__":
    main()
