"""Oracle: PowerSGD-style low-rank compression (family LOWRANK), rank r is the parameter.

The paper profiles the low-rank error of a rank by running power-iteration steps of
PowerSGD without the communication (appendix "Low-rank error computation", subsection
"Power Iteration Steps"), and gives the SVD tail sum as the optimum those steps approach
(subsection "Singular Value Decomposition").  One step, for a layer viewed as M [m x n]
(m = first dimension, n = product of the rest) and a warm-start Q0 [n x r]:

    P    = M Q0
    Phat = Gram-Schmidt(P)        columns left to right, modified Gram-Schmidt, each column
                                  divided by its norm; a column whose squared norm after
                                  projection is 0 or below 1e-10 x its squared norm before
                                  projection (a numerically dependent column: what is left
                                  is rounding noise in fp32 as well as in fp64) becomes the
                                  zero column
    Q    = M^T Phat
    Mhat = Phat Q^T;   error_r = ||M - Mhat||_F^2;   e' = M - Mhat
    size = 4 (m + n) r bytes;  payload = Phat [m x r] then Q [n x r], row-major fp32

More steps feed Q back in as the next warm start.  Rank r uses the first r columns of a
shared Q0 [n x r_max].  Everything here is fp64 and each rank is computed separately:
the plain definition, cost O(mn sum r).
"""
import numpy as np


def matrix_view(x: np.ndarray, rows: int, cols: int) -> np.ndarray:
    return np.asarray(x).reshape(rows, cols)


def gram_schmidt(p: np.ndarray) -> np.ndarray:
    p = np.array(p, np.float64, copy=True)
    r = p.shape[1]
    for j in range(r):
        before = float(np.dot(p[:, j], p[:, j]))
        for i in range(j):
            p[:, j] -= np.dot(p[:, i], p[:, j]) * p[:, i]
        after = float(np.dot(p[:, j], p[:, j]))
        if after == 0.0 or after < 1e-10 * before:
            p[:, j] = 0.0
        else:
            p[:, j] /= np.sqrt(after)
    return p


def power_step(m: np.ndarray, q0: np.ndarray, iters: int = 1):
    """(Phat [m x r], Q [n x r]) after `iters` power-iteration steps from warm start q0."""
    m = np.asarray(m, np.float64)
    q = np.asarray(q0, np.float64)
    for _ in range(iters):
        phat = gram_schmidt(m @ q)
        q = m.T @ phat
    return phat, q


def error(m: np.ndarray, q0: np.ndarray, r: int, iters: int = 1) -> float:
    m = np.asarray(m, np.float64)
    phat, q = power_step(m, np.asarray(q0)[:, :r], iters)
    res = m - phat @ q.T
    return float(np.sum(res * res))


def size_bytes(rows: int, cols: int, r: int) -> int:
    return 4 * (rows + cols) * r


def compress(g: np.ndarray, e, rows: int, cols: int, q0: np.ndarray, r: int, iters: int = 1):
    """One layer: (Phat f32 [m x r], Q f32 [n x r], new error feedback f32 [m*n])."""
    g = np.asarray(g, np.float32)
    x = g.copy() if e is None else g + np.asarray(e, np.float32)
    m = matrix_view(x, rows, cols).astype(np.float64)
    phat, q = power_step(m, np.asarray(q0)[:, :r], iters)
    new_e = (m - phat @ q.T).astype(np.float32).reshape(-1)
    return phat.astype(np.float32), q.astype(np.float32), new_e


def decompress(payload_bytes: np.ndarray, rows: int, cols: int, r: int) -> np.ndarray:
    """Receiver side: Phat Q^T from the payload (Phat [m x r] then Q [n x r], fp32), product
    formed in fp64 and rounded once to fp32, flattened row-major."""
    buf = np.asarray(payload_bytes, np.uint8)
    phat = buf[:4 * rows * r].view(np.float32).reshape(rows, r).astype(np.float64)
    q = buf[4 * rows * r:4 * (rows + cols) * r].view(np.float32).reshape(cols, r).astype(np.float64)
    return (phat @ q.T).astype(np.float32).reshape(-1)
