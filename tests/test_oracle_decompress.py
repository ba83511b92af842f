"""Pins of the oracle's receiver side (payload -> dense image): it must undo what the sender did,
which ties it to definitions that are pinned elsewhere (codes = nearest grid point, kept set =
brute-force top-k, Phat Q^T = the projection) and to the profile: the squared distance between
x and the decoded image is the profiled error."""
import numpy as np

from oracle import lowrank, pipeline, quant, topk

QUANT, TOPK, LOWRANK = 0, 1, 2


def _x(n, seed, scale=1e-3):
    rng = np.random.default_rng(seed)
    return (rng.standard_t(3, n) * scale).astype(np.float32), (rng.standard_normal(n) * scale * 0.1).astype(np.float32)


def test_quant_image_is_x_minus_new_error_feedback_and_matches_profile():
    for n in (1, 7, 128, 129, 1000, 4099):
        g, e = _x(n, n)
        x = quant.form_x(g, e)
        for bits in (1, 2, 3, 5, 8):
            payload, new_e, extra = pipeline.compress_layer(g, e, 0, n, 0, 0, (QUANT, bits), 0)
            img = pipeline.decompress_layer(payload, n, 0, 0, (QUANT, bits))
            assert np.array_equal(img.view(np.uint32), extra["xhat"].view(np.uint32))
            # sender's residual and receiver's image add back to x up to the one rounding of x - xhat
            assert np.allclose(img.astype(np.float64) + new_e, x, rtol=0, atol=np.abs(x).max() * 2.0 ** -23)
            d = img.astype(np.float64) - x.astype(np.float64)
            assert abs(np.sum(d * d) - quant.error(x, bits)) <= 1e-12 * quant.error(x, bits)
            # every decoded value lies within half a grid step of x (closed form)
            nb = (n + 127) // 128
            unit = payload[:8 * nb].view(np.float32).reshape(nb, 2)[:, 1]
            step = np.repeat(unit, 128)[:n].astype(np.float64)
            assert (np.abs(d) <= 0.5 * step * (1 + 1e-6) + np.abs(x) * 2.0 ** -22).all()


def test_topk_image_keeps_exactly_the_selected_entries():
    for n in (1, 5, 1000, 4097):
        g, e = _x(n, 100 + n)
        x = quant.form_x(g, e)
        for d in (0.001, 0.05, 0.5, 1.0):
            payload, new_e, extra = pipeline.compress_layer(g, e, 0, n, 0, 0, (TOPK, d), 0)
            img = pipeline.decompress_layer(payload, n, 0, 0, (TOPK, d))
            k = topk.k_of(n, d)
            order = sorted(range(n), key=lambda i: (-abs(float(x[i])), i))[:k]       # brute force
            expect = np.zeros(n, np.float32)
            expect[order] = x[order]
            assert np.array_equal(img.view(np.uint32), expect.view(np.uint32))
            assert np.array_equal((img + new_e).view(np.uint32), (x + np.float32(0)).view(np.uint32))
            dd = img.astype(np.float64) - x
            assert abs(np.sum(dd * dd) - topk.error(x, k)) <= 1e-12 * topk.error(x, k)


def test_lowrank_image_is_the_projection():
    rng = np.random.default_rng(9)
    for (m, n, r) in ((8, 5, 2), (40, 33, 4), (64, 128, 16)):
        g = rng.standard_normal(m * n).astype(np.float32)
        q0 = rng.standard_normal((n, 64)).astype(np.float32)
        payload, new_e, extra = pipeline.compress_layer(g, None, 0, m * n, m, n, (LOWRANK, r), 0, q0_layer=q0)
        img = pipeline.decompress_layer(payload, m * n, m, n, (LOWRANK, r)).reshape(m, n).astype(np.float64)
        x = g.reshape(m, n).astype(np.float64)
        ph = extra["phat"].astype(np.float64)
        # image = Phat Phat^T X up to the fp32 rounding of the factors; it lies in span(Phat)
        assert np.allclose(img, ph @ (ph.T @ x), atol=1e-5 * np.abs(x).max())
        assert np.allclose(ph @ (ph.T @ img), img, atol=1e-5 * np.abs(x).max())
        assert np.allclose(img + new_e.reshape(m, n), x, atol=1e-5 * np.abs(x).max())
        err = np.sum((x - img) ** 2)
        assert abs(err - lowrank.error(x, q0, r)) <= 1e-5 * np.sum(x * x)


def test_accumulate_adds_in_fp32():
    g, e = _x(1000, 5)
    payload, _, _ = pipeline.compress_layer(g, e, 0, 1000, 0, 0, (QUANT, 4), 0)
    base = np.linspace(-1, 1, 1000).astype(np.float32)
    img = pipeline.decompress_layer(payload, 1000, 0, 0, (QUANT, 4))
    acc = pipeline.decompress_layer(payload, 1000, 0, 0, (QUANT, 4), out=base)
    assert np.array_equal(acc, base + img) and acc.dtype == np.float32
