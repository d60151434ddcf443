"""Pins for the oracle's generator: Philox4x32-10 words, the uniform map and Box-Muller.

The paper (Section 3, Algorithm 1) needs i.i.d. N(0, I_d) vectors from a generator
all machines share; its proofs use E zeta^2 = 1 and E zeta^4 = 3 (proof of Lemma 3.2).
"""
import os

import numpy as np
import pytest
from scipy import stats

import oracle

M0, M1 = 0xD2511F53, 0xCD9E8D57
MASK = 0xFFFFFFFF


def _read_kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_known_answers.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers(golden_dir):
    rows = _read_kat(golden_dir)
    assert len(rows) == 3
    for ctr, key, out in rows:
        got = oracle.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == out


def _inverse_round(c, k):
    """Invert one Philox round with modular inverses of the (odd) multipliers."""
    inv0 = pow(M0, -1, 1 << 32)
    inv1 = pow(M1, -1, 1 << 32)
    n0, lo_b, n2, lo_a = (int(x) for x in c)
    c0 = (lo_a * inv0) & MASK
    c2 = (lo_b * inv1) & MASK
    hi_a = (M0 * c0) >> 32
    hi_b = (M1 * c2) >> 32
    c1 = n0 ^ hi_b ^ k[0]
    c3 = n2 ^ hi_a ^ k[1]
    return [c0, c1, c2, c3]


def test_philox_round_is_a_bijection():
    rng = np.random.default_rng(11)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 1 << 32, 4, dtype=np.uint64)]
        key = [int(x) for x in rng.integers(0, 1 << 32, 2, dtype=np.uint64)]
        fwd = oracle.philox_round(ctr, key)
        assert _inverse_round(fwd, key) == ctr


def test_ten_rounds_unwind_to_the_counter():
    """Undo the ten rounds with the key schedule run backwards."""
    rng = np.random.default_rng(12)
    W0, W1 = 0x9E3779B9, 0xBB67AE85
    for _ in range(50):
        ctr = [int(x) for x in rng.integers(0, 1 << 32, 4, dtype=np.uint64)]
        key = [int(x) for x in rng.integers(0, 1 << 32, 2, dtype=np.uint64)]
        c = [int(x) for x in oracle.philox4x32_10(ctr, key)]
        for r in reversed(range(10)):
            k = [(key[0] + r * W0) & MASK, (key[1] + r * W1) & MASK]
            c = _inverse_round(c, k)
        assert c == ctr


def _read_xi_golden(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "xi_blocks.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            a, b, c = line.split("|")
            seed, rnd, j, q = (int(t) for t in a.split())
            w = [int(t, 16) for t in b.split()]
            z = [float(t) for t in c.split()]
            rows.append((seed, rnd, j, q, w, z))
    return rows


def test_counter_layout_and_normals_match_golden(golden_dir):
    rows = _read_xi_golden(golden_dir)
    assert len(rows) == 5
    for seed, rnd, j, q, w, z in rows:
        assert [int(x) for x in oracle.words(seed, rnd, j, q)] == w
        # the words are Philox of counter (q, j, round lo, round hi), key (seed lo, seed hi)
        assert [int(x) for x in oracle.philox4x32_10(
            [q, j, rnd & MASK, rnd >> 32], [seed & MASK, seed >> 32])] == w
        np.testing.assert_allclose(oracle.xi_block(seed, rnd, j, q), z, rtol=0, atol=1e-11)
        for k in range(4):
            assert abs(oracle.xi(seed, rnd, j, 4 * q + k) - z[k]) <= 1e-11


def test_seed_and_round_high_words_enter_the_stream():
    base = oracle.words(5, 9, 3, 7)
    assert not np.array_equal(base, oracle.words(5 + (1 << 32), 9, 3, 7))
    assert not np.array_equal(base, oracle.words(5, 9 + (1 << 32), 3, 7))
    assert [int(x) for x in oracle.words(5 + (3 << 32), 9 + (2 << 32), 3, 7)] == \
        [int(x) for x in oracle.philox4x32_10([7, 3, 9, 2], [5, 3])]


def test_box_muller_special_values():
    # u1 = 1 (all-ones top 24 bits) gives exactly zero radius
    z0, z1 = oracle.box_muller(0xFFFFFFFF, 0x12345678)
    assert z0 == 0.0 and z1 == 0.0
    # smallest u1 = 2^-24, angle 0: the largest value the map can produce
    z0, z1 = oracle.box_muller(0x000000FF, 0x000000FF)
    assert abs(z0 - np.sqrt(48.0 * np.log(2.0))) < 1e-12 and z1 == 0.0
    # quarter turn: u2 = 1/4 -> cosine branch ~ 0, sine branch = r
    xa = 0x7FFFFF00  # u1 = 0.5
    r = np.sqrt(2.0 * np.log(2.0))
    z0, z1 = oracle.box_muller(xa, 0x40000000)
    assert abs(z0) < 1e-15 and abs(z1 - r) < 1e-15
    # half turn: cosine branch = -r
    z0, z1 = oracle.box_muller(xa, 0x80000000)
    assert abs(z0 + r) < 1e-15 and abs(z1) < 1e-15
    # the low 8 bits of a word are unused
    assert oracle.box_muller(0x12345600, 0x9ABCDE00) == oracle.box_muller(0x123456FF, 0x9ABCDEFF)
    # radius/angle identities for an arbitrary pair
    z0, z1 = oracle.box_muller(0x13572468, 0xC0000000)  # three-quarter turn
    u1 = ((0x13572468 >> 8) + 1) / 2.0 ** 24
    assert abs(z0 * z0 + z1 * z1 - (-2.0 * np.log(u1))) < 1e-12
    assert abs(z0) < 1e-14 and z1 < 0


def test_normals_have_gaussian_moments_and_law():
    """E z = 0, E z^2 = 1, E z^4 = 3 (the two moments the proof of Lemma 3.2 uses), KS vs N(0,1)."""
    N = 10_000_000
    z = oracle.xi_range(3, 0, 5, 0, N)
    s = 1.0 / np.sqrt(N)
    assert abs(z.mean()) < 5 * s
    assert abs((z ** 2).mean() - 1.0) < 5 * np.sqrt(2.0) * s
    assert abs((z ** 3).mean()) < 5 * np.sqrt(15.0) * s
    assert abs((z ** 4).mean() - 3.0) < 5 * np.sqrt(96.0) * s
    assert np.abs(z).max() <= np.sqrt(48.0 * np.log(2.0)) + 1e-12
    ks = stats.kstest(z[:500_000], "norm")
    assert ks.pvalue > 1e-3
    # the four lanes of a block are mutually uncorrelated and each N(0,1)
    zz = z.reshape(-1, 4)
    C = np.corrcoef(zz.T)
    assert np.abs(C - np.eye(4)).max() < 5.0 / np.sqrt(N / 4)
    for k in range(4):
        assert stats.kstest(zz[:200_000, k], "norm").pvalue > 1e-3


def test_streams_are_independent_across_j_round_and_seed():
    N = 1_000_000
    a = oracle.xi_range(3, 0, 0, 0, N)
    others = [oracle.xi_range(3, 0, 1, 0, N), oracle.xi_range(3, 1, 0, 0, N),
              oracle.xi_range(4, 0, 0, 0, N), oracle.xi_range(3, 0, 0, N, N)]
    for b in others:
        assert abs(np.mean(a * b)) < 5.0 / np.sqrt(N)
        assert abs(np.mean(a * a * b * b) - 1.0) < 5.0 * np.sqrt(8.0 / N)


def test_xi_is_a_pure_function_of_its_indices():
    a = oracle.xi_range(9, 2, 7, 0, 64)
    b = oracle.xi_range(9, 2, 7, 0, 64)
    assert np.array_equal(a, b)
    # a range that starts inside a block agrees with the aligned one
    c = oracle.xi_range(9, 2, 7, 5, 20)
    assert np.array_equal(c, a[5:25])
