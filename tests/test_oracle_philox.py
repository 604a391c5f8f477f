"""Pins for the oracle's noise generator (counter-based, Philox4x32-10 layout;
requirement from Eq. 2 / App. B.1: xi_0, eta_b i.i.d. N(0, I), fresh per split)."""
import os

import numpy as np
from scipy import stats

from oracle import philox, sde

M0, M1 = 0xD2511F53, 0xCD9E8D57


def _inverse_round(out, k0, k1):
    """Inverse of one round, from the definition: the low products give c0, c2
    back through the modular inverses of the (odd) multipliers."""
    inv0, inv1 = pow(M0, -1, 1 << 32), pow(M1, -1, 1 << 32)
    o0, o1, o2, o3 = (int(x) for x in out)
    c2 = (o1 * inv1) & 0xFFFFFFFF
    c0 = (o3 * inv0) & 0xFFFFFFFF
    hi1, hi0 = (M1 * c2) >> 32, (M0 * c0) >> 32
    return c0, o0 ^ hi1 ^ k0, c2, o2 ^ hi0 ^ k1


def test_known_answer_vectors_of_the_published_generator():
    """The raw words against the generator's published known answers (tests/golden/): fixes the
    multipliers, the Weyl increments, the round count and the word order."""
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_known_answers.txt")
    rows = [[int(w, 16) for w in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        ctr, key, want = row[0:4], row[4:6], row[6:10]
        got = philox.philox4x32_10(np.array([ctr], dtype=np.uint64), key[0] | (key[1] << 32))[0]
        assert [int(x) for x in got] == want


def test_round_is_a_bijection_with_the_defined_inverse():
    rng = np.random.default_rng(0)
    for _ in range(50):
        c = rng.integers(0, 1 << 32, size=4, dtype=np.uint64)
        k0, k1 = (int(x) for x in rng.integers(0, 1 << 32, size=2, dtype=np.uint64))
        out = philox.philox_round(c[None], k0, k1)[0]
        assert _inverse_round(out, k0, k1) == tuple(int(x) for x in c)


def test_every_counter_word_and_the_seed_matter():
    base = philox.philox4x32_10(np.array([[5, 6, 7, 0]]), 99)[0]
    for pos in range(4):
        ctr = np.array([[5, 6, 7, 0]])
        ctr[0, pos] += 1
        other = philox.philox4x32_10(ctr, 99)[0]
        flipped = sum(bin(int(a) ^ int(b)).count("1") for a, b in zip(base, other))
        assert 32 < flipped < 96          # about half of 128 bits
    for seed in (98, 99 + (1 << 32)):     # low and high key word
        other = philox.philox4x32_10(np.array([[5, 6, 7, 0]]), seed)[0]
        flipped = sum(bin(int(a) ^ int(b)).count("1") for a, b in zip(base, other))
        assert 32 < flipped < 96


def test_words_are_uniform():
    w = philox.words(1223627, 17, 3, philox.TAG_ETA, 1 << 16).ravel()
    top = (w >> np.uint32(24)).astype(np.int64)
    chi2 = ((np.bincount(top, minlength=256) - w.size / 256) ** 2 / (w.size / 256)).sum()
    assert chi2 < stats.chi2.ppf(1 - 1e-6, 255)
    bits = np.unpackbits(w.view(np.uint8))
    assert abs(bits.mean() - 0.5) < 5 / np.sqrt(bits.size)
    u = philox.uniform(w)
    assert u.min() > 0.0 and u.max() < 1.0
    # u = (2k+1)/2^24 is exactly representable in fp32 (24 significant bits)
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)


def test_normals_are_standard_and_streams_independent():
    D = 1 << 18
    a = philox.normals(7, 3, 2, philox.TAG_ETA, D)
    assert stats.kstest(a, "norm").pvalue > 1e-4
    assert abs(a.mean()) < 5 / np.sqrt(D) and abs(a.var() - 1) < 5 * np.sqrt(2 / D)
    assert abs(stats.kurtosis(a)) < 0.05
    # neighbours inside a quad, across quads, and other streams are uncorrelated
    assert abs(np.corrcoef(a[0::2], a[1::2])[0, 1]) < 5 / np.sqrt(D / 2)
    assert abs(np.corrcoef(a[:-4], a[4:])[0, 1]) < 5 / np.sqrt(D)
    for other in (philox.normals(7, 4, 2, philox.TAG_ETA, D), philox.normals(7, 3, 3, philox.TAG_ETA, D),
                  philox.normals(7, 3, 2, philox.TAG_XI0, D), philox.normals(8, 3, 2, philox.TAG_ETA, D)):
        assert abs(np.corrcoef(a, other)[0, 1]) < 5 / np.sqrt(D)


def test_box_muller_layout_by_hand():
    # element 0 = r cos, element 1 = r sin of the pair (word0 -> radius, word1 -> angle)
    w = philox.words(11, 2, 5, philox.TAG_ETA, 1)[0]
    u = [((int(x) >> 9) + 0.5) / (1 << 23) for x in w]
    n = philox.normals(11, 2, 5, philox.TAG_ETA, 4)
    for a, b in ((0, 1), (2, 3)):
        r, th = np.sqrt(-2 * np.log(u[a])), 2 * np.pi * u[b]
        assert np.isclose(n[a], r * np.cos(th), rtol=1e-14)
        assert np.isclose(n[b], r * np.sin(th), rtol=1e-14)
        assert np.isclose(n[a] ** 2 + n[b] ** 2, -2 * np.log(u[a]), rtol=1e-12)


def test_branch_noise_moments():
    """App. B.1: each xi_b ~ N(0, I) and Cov(xi_b, xi_b') = I / (1 + s^2)."""
    D = 1 << 18
    xi0 = philox.normals(3, 10, 4, philox.TAG_XI0, D)
    for s in (1.0, 2.0, 4.0, 8.0):
        xb = [sde.branch_noise(xi0, philox.normals(3, child, 4, philox.TAG_ETA, D), s) for child in (21, 22, 23)]
        for x in xb:
            assert abs(x.var() - 1) < 5 * np.sqrt(2 / D) and abs(x.mean()) < 5 / np.sqrt(D)
            assert stats.kstest(x, "norm").pvalue > 1e-4
        for i in range(3):
            for j in range(i + 1, 3):
                cov = np.mean(xb[i] * xb[j])
                assert abs(cov - 1 / (1 + s * s)) < 6 / np.sqrt(D)
    # s = 0: all siblings identical
    assert np.array_equal(sde.branch_noise(xi0, xb[0], 0.0), xi0)
