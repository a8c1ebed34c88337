"""Pins of the oracle's random-number layer against things other than itself.

The paper (arXiv 1810.07766) fixes the distributions only: every message is lost
independently with probability p (Sec. 3, "Unreliable Network Connection") and
the server of a block is drawn uniformly without replacement (Alg. 1 step 6).
The bit-level specification is this project's; these tests pin it to
  - the published Philox4x32-10 known-answer vectors,
  - the documented counter layout (re-derived here from the raw hash),
  - the target distributions (drop frequency, independence, uniform servers),
  - the textbook Box-Muller transform evaluated in double precision.
"""
import os

import numpy as np
import pytest
from scipy import stats

from oracle import rps_oracle as oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = oracle.philox4x32(v[0:4], v[4:6], rounds=10)
        assert [int(x) for x in out] == v[6:10]


def test_philox_is_a_bijection_on_small_slices():
    # distinct counters -> distinct outputs (a counter-based generator is a keyed bijection)
    outs = {tuple(int(x) for x in oracle.philox4x32([i, 0, 0, 0], [7, 9])) for i in range(2000)}
    assert len(outs) == 2000
    # the key matters
    assert tuple(oracle.philox4x32([1, 2, 3, 4], [0, 0])) != tuple(oracle.philox4x32([1, 2, 3, 4], [1, 0]))


def _word0(seed, step, a, b, domain):
    ctr = [a, b, step & 0xFFFFFFFF, (domain << 24) | ((step >> 32) & 0xFFFFFF)]
    key = [seed & 0xFFFFFFFF, seed >> 32]
    return int(oracle.philox4x32(ctr, key, rounds=10)[0])


@pytest.mark.parametrize("seed,step,n,p", [(0, 0, 4, 0.5), (12345678901234567, (5 << 32) + 17, 7, 0.3),
                                           (3, 99, 64, 0.05)])
def test_masks_follow_the_documented_counter_layout(seed, step, n, p):
    """drop iff hash word 0 of (worker, block, step, domain) < floor(p 2^32); domain 0 = uplink,
    1 = downlink, 2 = server sort key; self links forced after the draw."""
    server, U, D = oracle.masks(seed, step, n, p)
    keys = [(_word0(seed, step, i, 0, 2), i) for i in range(n)]
    assert [i for _, i in sorted(keys)] == server.tolist()
    T = int(np.floor(p * 2.0 ** 32))
    for i in range(n):
        for j in range(n):
            if i == server[j]:
                assert U[i, j] == 1 and D[i, j] == 1
            else:
                assert U[i, j] == (0 if _word0(seed, step, i, j, 0) < T else 1)
                assert D[i, j] == (0 if _word0(seed, step, i, j, 1) < T else 1)


def test_p_zero_and_p_one_are_exact():
    for step in range(20):
        server, U, D = oracle.masks(1, step, 9, 0.0)
        assert U.all() and D.all()
        server, U, D = oracle.masks(1, step, 9, 1.0)
        expect = np.zeros((9, 9), dtype=np.uint8)
        expect[server, np.arange(9)] = 1          # only the server's link to itself survives
        assert (U == expect).all() and (D == expect).all()


def test_server_is_a_uniform_permutation():
    n, rounds = 8, 4000
    counts = np.zeros((n, n))
    for step in range(rounds):
        server, _, _ = oracle.masks(42, step, n, 0.1)
        assert sorted(server.tolist()) == list(range(n))     # without replacement
        counts[np.arange(n), server] += 1
    # every (block, worker) cell ~ Binomial(rounds, 1/n): P(A) = 1/n in the paper's Lemma 7
    chi2 = ((counts - rounds / n) ** 2 / (rounds / n)).sum()
    assert chi2 < stats.chi2.ppf(1 - 1e-6, df=(n - 1) * (n - 1))
    # identity flag = the exposition's "worker i averages block i"
    server, _, _ = oracle.masks(42, 3, n, 0.1, identity_server=True)
    assert server.tolist() == list(range(n))


@pytest.mark.parametrize("p", [0.01, 0.1, 0.2])
def test_drop_frequency_and_independence(p):
    n, rounds = 16, 600
    drops_u = drops_d = both = total = 0
    for step in range(rounds):
        server, U, D = oracle.masks(7, step, n, p)
        off = np.ones((n, n), dtype=bool)
        off[server, np.arange(n)] = False
        u = U[off] == 0
        d = D[off] == 0
        drops_u += u.sum(); drops_d += d.sum(); both += (u & d).sum(); total += off.sum()
    sd = np.sqrt(p * (1 - p) / total)
    assert abs(drops_u / total - p) < 5 * sd
    assert abs(drops_d / total - p) < 5 * sd
    # uplink and downlink losses are independent: P(both) = p^2
    sd2 = np.sqrt(p * p * (1 - p * p) / total)
    assert abs(both / total - p * p) < 5 * sd2


def test_masks_change_with_seed_and_step():
    a = oracle.masks(0, 0, 16, 0.3)
    b = oracle.masks(0, 1, 16, 0.3)
    c = oracle.masks(1, 0, 16, 0.3)
    assert not (a[1] == b[1]).all() and not (a[1] == c[1]).all()
    d = oracle.masks(0, 0, 16, 0.3)
    assert all((x == y).all() for x, y in zip(a, d))      # stateless: same (seed, step) -> same bits
    e = oracle.masks(0, 1 << 32, 16, 0.3)                 # the high half of the step is hashed too
    assert not (a[1] == e[1]).all()


def test_external_server_masks():
    """n workers, nb != n external servers: same hash layout, nothing forced, server = -1."""
    n, nb, p, seed = 4, 3, 0.3, 11
    T = int(np.floor(p * 2.0 ** 32))
    drops = total = 0
    for step in range(400):
        server, U, D = oracle.masks(seed, step, n, p, external_servers=nb)
        assert U.shape == (n, nb) and D.shape == (n, nb) and (server == -1).all()
        if step < 5:
            for i in range(n):
                for j in range(nb):
                    assert U[i, j] == (0 if _word0(seed, step, i, j, 0) < T else 1)
                    assert D[i, j] == (0 if _word0(seed, step, i, j, 1) < T else 1)
        drops += (U == 0).sum() + (D == 0).sum(); total += 2 * n * nb
    assert abs(drops / total - p) < 5 * np.sqrt(p * (1 - p) / total)


# ---------------------------------------------------------------------------------------------
# Gaussian noise
# ---------------------------------------------------------------------------------------------
def _noise_reference(seed, step, pair, quad, sigma):
    """The textbook Box-Muller transform in double precision on the same hash words (counter
    (quad >> 7, (quad & 127) | pair << 7, step low, 3 << 24 | step high)): u1 = (kr + 1/2)/4096 from
    bits 2..13, angle 2 pi (ka + 1/2)/4096 with ka = bit 31 (the half turn) above bits 17..27.  Words 0,1 -> worker 2*pair,
    words 2,3 -> worker 2*pair+1, columns 4*quad..4*quad+3."""
    ctr = [(quad >> 7) & 0xFFFFFFFF, (quad & 127) | (pair << 7), step & 0xFFFFFFFF, (3 << 24) | ((step >> 32) & 0xFFFFFF)]
    key = [seed & 0xFFFFFFFF, seed >> 32]
    words = oracle.philox4x32(ctr, key, rounds=7)      # the noise stream uses 7 rounds
    out = []
    for w in words:
        w = int(w)
        u1 = (((w >> 2) & 0xFFF) + 0.5) / 4096.0
        phi = 2.0 * np.pi * (((w >> 17) & 0x7FF) + 0.5) / 4096.0 + (np.pi if w >> 31 else 0.0)
        r = np.sqrt(-2.0 * np.log(u1))
        out += [sigma * r * np.cos(phi), sigma * r * np.sin(phi)]
    return np.array(out).reshape(2, 4)


def test_noise_matches_textbook_box_muller():
    worst = 0.0
    for (seed, step, pair, quad) in [(0, 0, 0, 0), (5, 3, 15, 123456), (2 ** 40 + 1, 2 ** 33, 31, 2 ** 31 + 5)]:
        for sigma in (1.0, 0.1, float(np.float32(np.sqrt(1e-3)))):
            for q in range(quad, quad + 150):
                z = oracle.noise_patch(seed, step, pair, q, sigma).astype(np.float64)
                ref = _noise_reference(seed, step, pair, q, sigma)
                err = np.abs(z - ref).max() / sigma
                worst = max(worst, err)
                assert err < 1e-6                        # three fp32 roundings of values below 4.25
    assert worst > 0.0                                   # (fp32 roundings, not the double result)


def test_noise_cells_are_the_correctly_rounded_values():
    """Every cell value of the specification -- sqrt(-2 ln((k + 1/2)/4096)), cos and sin of
    2 pi (a + 1/2)/4096 -- is the fp32 number nearest to the exact real value (50-digit
    arithmetic), so any implementation that rounds correctly produces the same bits."""
    import mpmath
    mpmath.mp.dps = 50
    r, c, s = oracle.noise_grid()

    def nearest_f32(x):
        f = np.float32(float(x))                         # double rounding could miss a tie by one ulp:
        cands = [f, np.nextafter(f, np.float32(np.inf)), np.nextafter(f, np.float32(-np.inf))]
        return min(cands, key=lambda v: abs(mpmath.mpf(float(v)) - x))

    for k in range(4096):
        exact = mpmath.sqrt(-2 * mpmath.log((mpmath.mpf(k) + mpmath.mpf(1) / 2) / 4096))
        assert r[k] == nearest_f32(exact), k
        phi = 2 * mpmath.pi * (mpmath.mpf(k) + mpmath.mpf(1) / 2) / 4096
        assert c[k] == nearest_f32(mpmath.cos(phi)), k
        assert s[k] == nearest_f32(mpmath.sin(phi)), k
    assert (np.diff(r) < 0).all() and r[0] < 4.2453 and r[-1] > 0.0156
    assert (c == -c[::-1][np.r_[2048:4096, 0:2048]]).all()   # cos(phi + pi) = -cos(phi) on the half-shifted grid
    assert (s == -s[::-1]).all() and (c == c[::-1]).all()        # phi -> 2 pi - phi
    assert (c[2048:] == -c[:2048]).all() and (s[2048:] == -s[:2048]).all()   # the half turn only flips signs


def test_noise_law_over_all_cells():
    """The law of z is the uniform law over the 2^24 (radius, angle) cells: enumerate it exactly.
    Symmetric; variance, fourth moment and the sup-distance to the normal cdf as documented."""
    r, c, s = oracle.noise_grid()
    for trig in (c, s):
        z = np.outer(r.astype(np.float32), trig.astype(np.float32)).astype(np.float32).astype(np.float64).reshape(-1)
        assert abs(z.mean()) < 1e-9
        assert abs(z.var() - 0.999915) < 2e-6
        assert abs((z ** 4).mean() - 2.99733) < 2e-5
        assert abs(np.abs(z).max() - 4.2452) < 1e-3
        z.sort()
        F = (np.arange(z.size) + 0.5) / z.size
        assert np.abs(stats.norm.cdf(z) - F).max() < 1e-4


def test_noise_indexing_by_worker_and_column():
    """noise(worker, column) is entry [worker % 2, column % 4] of the patch (worker // 2, column // 4)."""
    for worker in (0, 1, 6, 7, 63):
        for column in (0, 1, 2, 3, 4, 1001, 2 ** 33 + 6):
            patch = oracle.noise_patch(3, 8, worker // 2, column // 4, 0.5)
            assert oracle.noise(3, 8, worker, column, 0.5) == patch[worker % 2, column % 4]


def test_noise_sigma_scaling_and_determinism():
    a = oracle.noise_patch(9, 4, 2, 77, 1.0)
    assert (oracle.noise_patch(9, 4, 2, 77, 1.0) == a).all()
    assert (oracle.noise_patch(9, 4, 2, 77, 0.25) == 0.25 * a).all()      # power of two: exact
    assert not (oracle.noise_patch(9, 4, 3, 77, 1.0) == a).any()          # worker pair enters the counter
    assert not (oracle.noise_patch(9, 5, 2, 77, 1.0) == a).any()          # step too
    assert not (oracle.noise_patch(9, 4, 2, 78, 1.0) == a).any()
    assert not (oracle.noise_patch(10, 4, 2, 77, 1.0) == a).any()         # and the seed


def test_noise_is_standard_normal():
    z = np.stack([oracle.noise_patch(11, 2, k, q, 1.0) for k in range(4) for q in range(50000)]).astype(np.float64)
    z = z.reshape(4, 50000, 2, 4)                     # [pair, quad, worker-in-pair, column-in-quad]
    flat = z.reshape(-1)
    n = flat.size                                     # 1.6 M samples
    assert abs(flat.mean()) < 5 / np.sqrt(n)
    assert abs(flat.var() - 1.0) < 5 * np.sqrt(2.0 / n) + 2e-4
    assert abs((flat ** 3).mean()) < 5 * np.sqrt(15.0 / n)
    assert abs((flat ** 4).mean() - 3.0) < 5 * np.sqrt(96.0 / n) + 2e-3
    assert stats.kstest(flat[:200000], "norm").pvalue > 1e-4
    # the two members of a Box-Muller pair, the two workers of a patch, neighbouring columns:
    # all uncorrelated (also in their squares)
    def corr(a, b):
        return abs(np.corrcoef(a.reshape(-1), b.reshape(-1))[0, 1])
    m = z[..., 0].size
    assert corr(z[..., 0], z[..., 1]) < 5 / np.sqrt(m)
    assert corr(z[:, :, 0, :], z[:, :, 1, :]) < 5 / np.sqrt(2 * m)
    assert corr(z[:, :-1, :, 3], z[:, 1:, :, 0]) < 5 / np.sqrt(m / 2)
    assert corr(z[..., 0] ** 2, z[..., 1] ** 2) < 5 / np.sqrt(m)
    assert corr(z[:, :, 0, :] ** 2, z[:, :, 1, :] ** 2) < 5 / np.sqrt(2 * m)
    # 12-bit radius index: |z| <= sqrt(2 ln 2^13)
    assert np.abs(flat).max() <= np.sqrt(2 * np.log(2.0 ** 13)) * (1 + 1e-6)
