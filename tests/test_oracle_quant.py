"""Pins for the quantization oracle: closed-form bounds, exact special cases, stochastic
rounding statistics, payload format, and the single-rounding fma helper."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import quant
from paper_2210_17357_amd import workloads as W

F32 = np.float32
BITS = (2, 3, 4, 5, 6, 7, 8)


def _data(n, seed=0, scale=1e-3):
    rng = np.random.default_rng(seed)
    return (rng.standard_t(3, n) * scale).astype(F32)


def _bucket_range(x, bucket=128):
    r = np.zeros(x.size, np.float64)
    for s in range(0, x.size, bucket):
        xb = x[s:s + bucket]
        r[s:s + bucket] = float(F32(xb.max() - xb.min()))
    return r


@pytest.mark.parametrize("bits", BITS)
def test_deterministic_closed_form_bound(bits):
    # nearest grid point: |xhat - x| <= unit/2, i.e. err^2 <= range^2 / (4 (2^b-1)^2)
    x = _data(128 * 37 + 45, seed=bits)
    _, _, _, xhat = quant.quantize(x, bits)
    r = _bucket_range(x)
    err2 = (xhat.astype(np.float64) - x.astype(np.float64)) ** 2
    bound = r * r / (4.0 * (2 ** bits - 1) ** 2)
    assert np.all(err2 <= bound * (1 + 1e-5) + 1e-30)
    # and the bound is nearly attained somewhere (rules out a grid that is too fine)
    assert err2.max() > 0.5 * bound[np.argmax(err2)]


@pytest.mark.parametrize("bits", (2, 4, 8))
def test_stochastic_bound_unbiased_and_variance(bits):
    x = _data(128 * 4, seed=11)
    r = _bucket_range(x)
    unit = r / (2 ** bits - 1)
    reps = 600
    acc = np.zeros(x.size, np.float64)
    acc2 = np.zeros(x.size, np.float64)
    for s in range(reps):
        u = quant.layer_uniforms(1000 + s, 0, x.size)
        _, _, _, xhat = quant.quantize(x, bits, u=u)
        d = xhat.astype(np.float64) - x.astype(np.float64)
        assert np.all(np.abs(d) <= unit * (1 + 1e-5) + 1e-30)      # err^2 <= range^2/(2^b-1)^2
        acc += d
        acc2 += d * d
    mean = acc / reps
    # E[xhat] = x: mean error is small against its own standard error (unit/2 / sqrt(reps))
    assert np.all(np.abs(mean) <= 5.0 * 0.5 * unit / np.sqrt(reps) + 1e-12)
    # E[(xhat-x)^2] = unit^2 f (1-f), f = frac((x-m)/unit); summed over the layer
    m = np.repeat([x[s:s + 128].min() for s in range(0, x.size, 128)], 128).astype(np.float64)
    f = ((x.astype(np.float64) - m) / unit) % 1.0
    expect = np.sum(unit ** 2 * f * (1 - f))
    assert abs(np.sum(acc2 / reps) - expect) < 0.03 * expect


def test_constant_and_two_valued_buckets_have_zero_error():
    for bits in BITS:
        x = np.full(300, 0.37, F32)
        codes, mins, units, xhat = quant.quantize(x, bits)
        assert np.all(codes == 0) and np.array_equal(xhat, x) and np.all(units == 0)
        y = np.where(np.arange(256) % 3 == 0, F32(-0.125), F32(0.75)).astype(F32)
        codes, _, _, yhat = quant.quantize(y, bits)
        assert np.array_equal(yhat, y)
        assert set(np.unique(codes)) == {0, 2 ** bits - 1}
    assert quant.error(np.zeros(1000, F32), 4) == 0.0


def test_codes_are_nearest_grid_point_in_exact_arithmetic():
    # independent check of the decision itself with rationals (away from exact half-way points)
    x = _data(128, seed=3)
    for bits in (2, 5, 8):
        codes, mins, units, _ = quant.quantize(x, bits)
        m, M = Fraction(float(x.min())), Fraction(float(x.max()))
        lv = 2 ** bits - 1
        for xi, c in zip(x, codes):
            t = (Fraction(float(xi)) - m) * lv / (M - m)
            nearest = int(t + Fraction(1, 2))
            if abs((t % 1) - Fraction(1, 2)) > Fraction(1, 10 ** 4):
                assert int(c) == min(max(nearest, 0), lv)


def test_tiny_range_bucket_degenerates_to_zero_codes():
    # lv / r overflows fp32 -> inv := 0 -> all codes 0, xhat = min
    x = np.array([0.0, 1e-44, 2e-44, 0.0] * 32, F32)
    codes, mins, units, xhat = quant.quantize(x, 8)
    assert np.all(codes == 0) and np.all(xhat == mins[0])


def test_error_decreases_with_bits_on_workload_data():
    b = W.generate(W.workload("c0_tiny_quant"))
    for off, n in zip(b.offsets, b.numels):
        x = b.grads[off:off + n]
        errs = [quant.error(x, bits) for bits in BITS]
        assert all(errs[i] > errs[i + 1] for i in range(len(errs) - 1))
        # smooth data, fine grid: error ~ sum unit^2 / 12
        _, _, units, _ = quant.quantize(x, 8)
        cnt = np.minimum(128, n - 128 * np.arange(units.size))
        approx = float(np.sum(units.astype(np.float64) ** 2 * cnt) / 12.0)
        assert 0.7 * approx < errs[-1] < 1.3 * approx


def test_fast_path_equals_bucket_loop():
    x = _data(128 * 9 + 77, seed=8)
    u = quant.layer_uniforms(4, 2, x.size)
    for bits in BITS:
        for uu in (None, u):
            a = quant.quantize(x, bits, u=uu)
            b = quant.quantize_fast(x, bits, u=uu)
            for p, q in zip(a, b):
                assert np.array_equal(p, q)


def test_payload_layout_hand_example():
    # 3-bit codes 1,2,3,4,5,6,7,0 -> LSB-first stream: value 1 at bits 0..2, 2 at 3..5, ...
    codes = np.array([1, 2, 3, 4, 5, 6, 7, 0], np.uint8)
    bitstring = 0
    for i, c in enumerate(codes):
        bitstring |= int(c) << (3 * i)
    expect = np.frombuffer(bitstring.to_bytes(3, "little"), np.uint8)
    p = quant.pack(codes, np.array([1.5], F32), np.array([0.25], F32), 3, bucket=8)
    assert np.array_equal(p[:8].view(F32), np.array([1.5, 0.25], F32))
    assert np.array_equal(p[8:], expect)
    assert list(p[8:]) == [0xD1, 0x58, 0x1F]


@pytest.mark.parametrize("bits", BITS)
def test_payload_size_and_round_trip(bits):
    for n in (1, 7, 128, 129, 128 * 5 + 63):
        x = _data(n, seed=n)
        codes, mins, units, xhat = quant.quantize_fast(x, bits)
        p = quant.pack(codes, mins, units, bits)
        assert p.size == quant.size_bytes(n, bits)
        assert np.array_equal(quant.unpack(p, n, bits), xhat)
    assert quant.size_bytes(128, bits) == 16 * bits + 8


def test_compress_updates_error_feedback():
    g, e = _data(1000, 1), _data(1000, 2, 1e-4)
    payload, new_e, codes, xhat = quant.compress(g, e, 4)
    x = g + e
    assert np.array_equal(new_e, x - xhat)
    assert abs(float(np.sum(new_e.astype(np.float64) ** 2)) - quant.error(x, 4)) <= 1e-6 * quant.error(x, 4)


def test_fma32_single_rounding_against_rationals():
    rng = np.random.default_rng(0)
    q = rng.integers(0, 256, 4000).astype(F32)
    unit = (rng.standard_normal(4000) * 10.0 ** rng.uniform(-8, 2, 4000)).astype(F32)
    m = (rng.standard_normal(4000) * 10.0 ** rng.uniform(-8, 2, 4000)).astype(F32)
    # crafted double-rounding traps: q*unit + m = fp32 midpoint + a bit far below fp64 resolution
    q[:3] = [1, 3, 255]
    unit[:3] = [F32(2.0 ** -60), F32(2.0 ** -70), F32(-(2.0 ** -80))]
    m[:3] = [F32(1.0 + 2.0 ** -23) , F32(1.0), F32(1.0 + 2.0 ** -22)]
    got = quant.fma32(q, unit, m)
    for i in range(q.size):
        exact = Fraction(float(q[i])) * Fraction(float(unit[i])) + Fraction(float(m[i]))
        lo = np.nextafter(got[i], F32(-np.inf))
        hi = np.nextafter(got[i], F32(np.inf))
        dg = abs(exact - Fraction(float(got[i])))
        assert dg <= abs(exact - Fraction(float(lo))) and dg <= abs(exact - Fraction(float(hi)))
    # a genuine trap: the exact sum lies just above the midpoint between 1 and 1 + 2^-23
    q2 = np.array([3.0], F32)
    u2 = np.array([(2.0 ** -24 + 2.0 ** -47) / 1.0], F32)            # 24-bit significand
    m2 = np.array([1.0], F32)
    exact = Fraction(3) * Fraction(float(u2[0])) + 1
    r = quant.fma32(q2, u2, m2)[0]
    cands = [F32(1.0), np.nextafter(F32(1.0), F32(2)), np.nextafter(np.nextafter(F32(1.0), F32(2)), F32(2))]
    best = min(cands, key=lambda v: abs(exact - Fraction(float(v))))
    assert r == best
