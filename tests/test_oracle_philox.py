"""Pins for the oracle's Philox4x32-10: published known-answer vectors, the element ->
(counter, word) mapping, and uniformity of the derived [0,1) floats."""
import os

import numpy as np

from oracle import philox


def _kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([int(t, 16) for t in line.split()])
    return rows


def test_known_answer_vectors(golden_dir):
    rows = _kat(golden_dir)
    assert len(rows) >= 2
    for r in rows:
        out = philox.philox4x32_10([r[0]], [r[1]], [r[2]], [r[3]], r[4], r[5])
        assert [int(o[0]) for o in out] == r[6:10]


def test_vectorised_equals_scalar_calls():
    rng = np.random.default_rng(5)
    c = rng.integers(0, 2 ** 32, size=(4, 64), dtype=np.uint64)
    k0, k1 = 0x12345678, 0x9ABCDEF0
    vec = philox.philox4x32_10(c[0], c[1], c[2], c[3], k0, k1)
    for j in range(64):
        one = philox.philox4x32_10([c[0, j]], [c[1, j]], [c[2, j]], [c[3, j]], k0, k1)
        assert [int(v[j]) for v in vec] == [int(o[0]) for o in one]


def test_element_mapping():
    seed, layer, n = (7 << 32) | 0xDEADBEEF, 5, 37
    w = philox.element_words(seed, layer, n)
    for i in (0, 1, 2, 3, 4, 17, 36):
        out = philox.philox4x32_10([i >> 2], [0], [layer], [0], seed & 0xFFFFFFFF, seed >> 32)
        assert int(w[i]) == int(out[i & 3][0])
    # different layer or seed -> different stream
    assert not np.array_equal(w, philox.element_words(seed, layer + 1, n))
    assert not np.array_equal(w, philox.element_words(seed + 1, layer, n))


def test_uniform_range_and_moments():
    u = philox.element_uniform(123, 3, 400_000)
    assert u.dtype == np.float32
    assert u.min() >= 0.0 and u.max() < 1.0
    # multiples of 2^-24
    assert np.all((u.astype(np.float64) * 2 ** 24) % 1.0 == 0.0)
    assert abs(u.mean() - 0.5) < 4 * (1 / np.sqrt(12 * u.size))
    assert abs(u.var() - 1 / 12) < 1e-3
    hist, _ = np.histogram(u, bins=16, range=(0, 1))
    expected = u.size / 16
    chi2 = float(np.sum((hist - expected) ** 2 / expected))
    assert chi2 < 45.0            # 15 dof, p ~ 1e-4
