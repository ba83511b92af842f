"""Oracle: layer-wise Top-K sparsification (family TOPK), density d is the parameter.

The paper keeps, per layer, the fraction d of entries with the largest magnitude
(layer-wise, not global; Experimental Validation and "Global TopK" paragraphs) and relies on
error feedback for the rest.  Readings the paper leaves open:

  k       = min(n, max(1, floor(d*n + 0.5)))                    (fp64, every layer sends >= 1)
  order   = by |x| descending (compared as the fp32 bit pattern with the sign cleared),
            ties by index ascending;  kept = first k
  error   = sum over dropped entries of double(x)^2
  payload = kept values fp32[k] then kept indices uint32[k], both in ascending index order
  size    = 8k bytes  (the paper's uniform ratios ~ 1/(2d) pin value + index per entry)
  e'      = x on dropped entries, +0 on kept ones

The oracle is the plain definition: a stable sort.
"""
import math

import numpy as np

F32 = np.float32


def k_of(n: int, density: float) -> int:
    return min(n, max(1, int(math.floor(float(density) * float(n) + 0.5))))


def magnitude_keys(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, F32).view(np.uint32) & np.uint32(0x7FFFFFFF)


def select(x: np.ndarray, k: int) -> np.ndarray:
    """Indices (ascending) of the k kept entries."""
    keys = magnitude_keys(x).astype(np.int64)
    order = np.argsort(-keys, kind="stable")       # stable: equal magnitudes stay in index order
    return np.sort(order[:k]).astype(np.uint32)


def error(x: np.ndarray, k: int) -> float:
    kept = np.zeros(x.size, bool)
    kept[select(x, k)] = True
    d = np.asarray(x, F32)[~kept].astype(np.float64)
    return float(np.dot(d, d))


def errors_all(x: np.ndarray, ks) -> list:
    """Dropped energy for several k from one sort (same definition as error())."""
    x = np.asarray(x, F32)
    keys = magnitude_keys(x).astype(np.int64)
    order = np.argsort(-keys, kind="stable")
    sq = x[order].astype(np.float64) ** 2
    out = []
    for k in ks:
        out.append(float(np.sum(sq[k:])))
    return out


def size_bytes(n: int, density: float) -> int:
    return 8 * k_of(n, density)


def compress(g: np.ndarray, e, density: float):
    """One layer: (values f32[k], indices u32[k], new error feedback f32[n])."""
    g = np.asarray(g, F32)
    x = g.copy() if e is None else g + np.asarray(e, F32)
    k = k_of(x.size, density)
    idx = select(x, k)
    new_e = x.copy()
    new_e[idx] = F32(0.0)
    return x[idx].copy(), idx, new_e


def payload(values: np.ndarray, indices: np.ndarray) -> np.ndarray:
    return np.concatenate([values.astype(F32).view(np.uint8), indices.astype(np.uint32).view(np.uint8)])


def decompress(payload_bytes: np.ndarray, n: int, k: int) -> np.ndarray:
    """Receiver side: the dense image of a Top-K payload (values[k] then indices[k]):
    zero everywhere except the kept positions."""
    buf = np.asarray(payload_bytes, np.uint8)
    values = buf[:4 * k].view(F32)
    indices = buf[4 * k:8 * k].view(np.uint32)
    out = np.zeros(n, F32)
    out[indices] = values
    return out
