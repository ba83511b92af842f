"""Pins for the Top-K oracle: brute force with ties, conservation, limits, and the uniform
compression ratios the paper prints (size = value + index per kept entry)."""
import itertools
import os

import numpy as np

from oracle import lowrank, topk
from paper_2210_17357_amd import workloads as W

F32 = np.float32


def _brute_select(x, k):
    # pick k entries one at a time: largest |x|, lowest index among equals
    left = list(range(len(x)))
    kept = []
    for _ in range(k):
        best = left[0]
        for i in left[1:]:
            if abs(float(x[i])) > abs(float(x[best])):
                best = i
        kept.append(best)
        left.remove(best)
    return sorted(kept)


def test_brute_force_with_ties():
    rng = np.random.default_rng(0)
    for trial in range(60):
        n = int(rng.integers(1, 14))
        x = rng.integers(-3, 4, n).astype(F32) * F32(0.5)        # many tied magnitudes, +-0
        if trial % 5 == 0:
            x[rng.integers(0, n)] = F32(-0.0)
        for k in range(1, n + 1):
            assert list(topk.select(x, k)) == _brute_select(x, k)
            kept = set(_brute_select(x, k))
            expect = sum(float(x[i]) ** 2 for i in range(n) if i not in kept)
            assert abs(topk.error(x, k) - expect) < 1e-12


def test_k_rule():
    assert topk.k_of(64, 0.001) == 1            # every layer sends at least one entry
    assert topk.k_of(30, 0.1) == 3
    assert topk.k_of(25, 0.1) == 3              # 2.5 rounds half up
    assert topk.k_of(1000, 0.005) == 5
    assert topk.k_of(10, 1.0) == 10
    assert topk.k_of(10, 5.0) == 10


def test_density_one_is_exact_and_errors_monotone_and_conserved():
    rng = np.random.default_rng(1)
    x = rng.laplace(0, 1e-3, 5000).astype(F32)
    assert topk.error(x, topk.k_of(x.size, 1.0)) == 0.0
    ks = [topk.k_of(x.size, d) for d in W.TOPK_DENSITIES] + [x.size]
    errs = topk.errors_all(x, ks)
    assert all(errs[i] >= errs[i + 1] for i in range(len(errs) - 1))
    total = float(np.sum(x.astype(np.float64) ** 2))
    for k, e in zip(ks, errs):
        idx = topk.select(x, k)
        kept = float(np.sum(x[idx].astype(np.float64) ** 2))
        assert abs(kept + e - total) <= 1e-12 * total
        assert abs(e - topk.error(x, k)) <= 1e-12 * total
        # the smallest kept magnitude is >= the largest dropped one
        mask = np.ones(x.size, bool)
        mask[idx] = False
        if mask.any():
            assert np.abs(x[idx]).min() >= np.abs(x[mask]).max()


def test_all_zero_layer_and_compress_outputs():
    vals, idx, new_e = topk.compress(np.zeros(100, F32), None, 0.05)
    assert list(idx) == [0, 1, 2, 3, 4] and np.all(vals == 0) and np.all(new_e == 0)
    g = np.array([1, -5, 2, 5, -0.5, 0, 3], F32)
    e = np.array([0, 0, 0, 0, 0.5, 0, 0], F32)
    vals, idx, new_e = topk.compress(g, e, 3 / 7)
    assert list(idx) == [1, 3, 6] and list(vals) == [-5, 5, 3]
    assert list(new_e) == [1, 0, 2, 0, 0, 0, 0]
    p = topk.payload(vals, idx)
    assert p.size == topk.size_bytes(7, 3 / 7) == 24
    assert np.array_equal(p[:12].view(F32), vals) and np.array_equal(p[12:].view(np.uint32), idx)


def test_sizes_reproduce_paper_uniform_ratios(golden_dir):
    shapes = {("resnet50", 1000): W.resnet50_shapes(1000), ("resnet18", 100): W.resnet18_shapes(100)}
    with open(os.path.join(golden_dir, "paper_uniform_ratios.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for model, classes, family, param, printed in rows:
        sh = shapes[(model, int(classes))]
        total = 4 * sum(int(np.prod(s)) for s in sh)
        comp = 0
        for s in sh:
            n = int(np.prod(s))
            if len(s) == 1:
                comp += 4 * n
            elif family == "topk":
                comp += topk.size_bytes(n, float(param))
            else:
                comp += lowrank.size_bytes(s[0], n // s[0], int(param))
        assert abs(total / comp - float(printed)) < 0.01 * float(printed), (model, family)
