"""Writes tests/golden/alpha_table.txt: the mixing constants alpha1, alpha2 and beta = alpha1 - alpha2
of arXiv 1810.07766 (Sec. 4.2, eqs. (def_alpha1), (def_alpha2); the quantities its Fig. 2 and Fig. 3
plot over n and p) for small networks, by EXACT enumeration of every network outcome of one block
through the CPU oracle's own round: server uniform over the n workers (Alg. 1 step 6), every other
uplink and downlink lost independently with probability p (Sec. 3), own links reliable.

Calls only oracle/ (never the HIP library).  Run from the repository root:
    python tests/golden/make_alpha_table.py
"""
import itertools
import os
import sys

import numpy as np

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", ".."))
from oracle import rps_oracle as oracle  # noqa: E402

GRID_N = (2, 3, 4, 5, 6, 7)
GRID_P = (0.01, 0.05, 0.1, 0.2, 0.5)


def exact_alphas(n, p):
    q = 1.0 - p
    A = np.full((n, n), 1.0 / n)
    WW = np.zeros((n, n)); WAW = np.zeros((n, n)); total = 0.0
    for s in range(n):
        others = [i for i in range(n) if i != s]
        for up in itertools.product((0, 1), repeat=n - 1):
            for dn in itertools.product((0, 1), repeat=n - 1):
                U = np.zeros((n, 1), dtype=np.uint8); D = np.zeros((n, 1), dtype=np.uint8)
                U[s, 0] = D[s, 0] = 1
                for o, u, d in zip(others, up, dn):
                    U[o, 0] = u; D[o, 0] = d
                prob = (1.0 / n) * float(np.prod([q if b else p for b in up + dn]))
                W = oracle.build_W(0, U, D)
                WW += prob * W @ W.T; WAW += prob * W @ A @ W.T; total += prob
    assert abs(total - 1.0) < 1e-12
    # M = a I + (1 - a) A_n  =>  a = (n M_11 - 1) / (n - 1)
    a1 = (n * WW[0, 0] - 1.0) / (n - 1.0)
    a2 = (n * WAW[0, 0] - 1.0) / (n - 1.0)
    return a1, a2


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "alpha_table.txt")
    with open(out, "w") as f:
        f.write("# alpha1, alpha2, beta = alpha1 - alpha2 of the RPS mixing matrix (arXiv 1810.07766, Sec. 4.2,\n"
                "# eqs. (def_alpha1), (def_alpha2); content of Fig. 2 and Fig. 3 at small n), exact enumeration\n"
                "# of all outcomes of one block by tests/golden/make_alpha_table.py (CPU oracle only).\n"
                "# n p alpha1 alpha2 beta\n")
        for n in GRID_N:
            for p in GRID_P:
                a1, a2 = exact_alphas(n, p)
                f.write(f"{n} {p} {a1:.12e} {a2:.12e} {a1 - a2:.12e}\n")
    print("wrote", out)


if __name__ == "__main__":
    main()
