"""Pins for the low-rank oracle: SVD lower bound and convergence, exact recovery of
low-rank inputs, full rank, projection identity, orthonormality, the zero-column guard."""
import numpy as np

from oracle import lowrank


def _tail(m, r):
    s = np.linalg.svd(m, compute_uv=False)
    return float(np.sum(s[r:] ** 2))


def _mat(m, n, rho, noise, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((m, rho)) @ rng.standard_normal((rho, n))) / np.sqrt(rho) \
        + noise * rng.standard_normal((m, n))


def test_never_below_svd_tail_and_converges_to_it():
    m = _mat(60, 45, 6, 0.3, 0)
    q0 = np.random.default_rng(1).standard_normal((45, 16))
    for r in (1, 2, 4, 8, 16):
        best = _tail(m, r)
        e1 = lowrank.error(m, q0, r, 1)
        e5 = lowrank.error(m, q0, r, 5)
        e60 = lowrank.error(m, q0, r, 60)
        assert e1 >= e5 * (1 - 1e-12) >= e60 * (1 - 1e-12) >= best * (1 - 1e-10)
        if r >= 6:                                   # spectral gap -> fast convergence
            assert e60 <= best * (1 + 1e-3)


def test_exact_rank_input_recovered_in_one_step():
    m = _mat(40, 50, 5, 0.0, 2)
    q0 = np.random.default_rng(3).standard_normal((50, 8))
    total = float(np.sum(m * m))
    assert lowrank.error(m, q0, 5, 1) < 1e-20 * total
    assert lowrank.error(m, q0, 8, 1) < 1e-20 * total      # guard zeroes the surplus columns
    assert lowrank.error(m, q0, 4, 1) > 1e-3 * total


def test_full_rank_is_exact():
    m = np.random.default_rng(4).standard_normal((12, 30))
    q0 = np.random.default_rng(5).standard_normal((30, 12))
    assert lowrank.error(m, q0, 12, 1) < 1e-20 * float(np.sum(m * m))


def test_orthonormal_projection_identity_nested_and_monotone():
    m = _mat(64, 48, 10, 0.2, 6)
    q0 = np.random.default_rng(7).standard_normal((48, 16))
    phat, q = lowrank.power_step(m, q0, 1)
    assert np.allclose(phat.T @ phat, np.eye(16), atol=1e-12)
    assert np.allclose(q, m.T @ phat)
    total = float(np.sum(m * m))
    prev = total
    for r in (1, 2, 4, 8, 16):
        e = lowrank.error(m, q0, r, 1)
        # Phat orthonormal, Q = M^T Phat  =>  ||M - Phat Q^T||^2 = ||M||^2 - ||Q||^2, and the
        # factors of rank r are the leading columns of the rank-16 run
        assert abs(e - (total - float(np.sum(q[:, :r] ** 2)))) < 1e-10 * total
        pr, qr = lowrank.power_step(m, q0[:, :r], 1)
        assert np.allclose(pr, phat[:, :r]) and np.allclose(qr, q[:, :r])
        assert e <= prev
        prev = e


def test_gram_schmidt_against_qr_and_zero_guard():
    rng = np.random.default_rng(8)
    p = rng.standard_normal((30, 6))
    g = lowrank.gram_schmidt(p)
    qq, rr = np.linalg.qr(p)
    qq = qq * np.sign(np.diag(rr))                 # QR with positive diagonal is unique
    assert np.allclose(g, qq, atol=1e-12)
    p[:, 3] = 2.0 * p[:, 1] - p[:, 0]              # dependent column -> zero column
    g = lowrank.gram_schmidt(p)
    assert np.all(g[:, 3] == 0.0)
    assert np.allclose(np.delete(g, 3, 1).T @ np.delete(g, 3, 1), np.eye(5), atol=1e-12)
    assert np.all(lowrank.gram_schmidt(np.zeros((5, 2))) == 0.0)


def test_compress_outputs_and_size():
    rng = np.random.default_rng(9)
    g = rng.standard_normal(20 * 30).astype(np.float32)
    e = (0.1 * rng.standard_normal(600)).astype(np.float32)
    q0 = rng.standard_normal((30, 8)).astype(np.float32)
    phat, q, new_e = lowrank.compress(g, e, 20, 30, q0, 4)
    assert phat.shape == (20, 4) and q.shape == (30, 4) and new_e.shape == (600,)
    x = (g + e).reshape(20, 30).astype(np.float64)
    assert np.allclose(new_e.reshape(20, 30), x - phat.astype(np.float64) @ q.T.astype(np.float64), atol=1e-5)
    assert lowrank.size_bytes(20, 30, 4) == 4 * 50 * 4 == phat.nbytes + q.nbytes
