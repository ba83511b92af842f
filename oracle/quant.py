"""Oracle: bucketed min-max quantization with b bits per value (family QUANT).

The paper uses "QSGD" quantization through a communication library and treats the
bit-width as the per-layer compression parameter (Experimental Validation section); it
prints no quantizer formula.  The reading implemented here (stated op by op so that the
integer codes are reproducible in IEEE fp32):

  x      = fl32(g + e)
  bucket = 128 consecutive elements of one layer (the last bucket of a layer may be short)
  m, M   = min, max of the bucket;  r = fl32(M - m)
  lv     = 2^b - 1;  unit = fl32(r / lv);  inv = fl32(lv / r);  inv := 0 if lv / r is not finite
  q      = floor(fma32(fl32(x - m), inv, 0.5))     deterministic (one rounding inside the floor)
         = floor(fma32(fl32(x - m), inv, u))       stochastic, u in [0,1) from Philox(seed, layer, i)
  q      = min(max(q, 0), lv)
  xhat   = fma32(q, unit, m)               one rounding
  error  = sum (double(xhat) - double(x))^2
  size   = sum over buckets (ceil(cnt*b/8) + 8) bytes
  payload per layer = [min, unit] fp32 pairs of all buckets, then each bucket's codes as an
           LSB-first bit stream padded to a whole byte.

Every fp32 step is one numpy float32 ufunc (correctly rounded, never fused).
"""
import numpy as np

from . import philox

F32 = np.float32


def form_x(g: np.ndarray, e) -> np.ndarray:
    g = np.asarray(g, F32)
    return g.copy() if e is None else g + np.asarray(e, F32)


def fma32(a: np.ndarray, b: np.ndarray, c: np.ndarray) -> np.ndarray:
    """round_to_fp32(a*b + c) with a single rounding, for a*b exactly representable in fp64
    (true here: two fp32 factors have at most 48 significant bits in their product)."""
    p = a.astype(np.float64) * b.astype(np.float64)         # exact
    c = c.astype(np.float64)
    s = p + c                                               # rounded to fp64
    bb = s - p                                              # TwoSum: s + err == p + c exactly
    err = (p - (s - bb)) + (c - bb)
    r = s.astype(F32)
    d = s - r.astype(np.float64)                            # exact
    # Double rounding can only go wrong when s sits exactly on an fp32 midpoint and the
    # discarded part err pushes the true sum past it.
    up = np.nextafter(r, F32(np.inf))
    dn = np.nextafter(r, F32(-np.inf))
    half_up = (up.astype(np.float64) - r.astype(np.float64)) * 0.5
    half_dn = (r.astype(np.float64) - dn.astype(np.float64)) * 0.5
    with np.errstate(invalid="ignore"):
        fix_up = (d > 0) & (d == half_up) & (err > 0)
        fix_dn = (d < 0) & (-d == half_dn) & (err < 0)
    r = np.where(fix_up, up, r)
    r = np.where(fix_dn, dn, r)
    return r.astype(F32)


def bucket_bounds(n: int, bucket: int):
    starts = np.arange(0, n, bucket, dtype=np.int64)
    return starts, np.minimum(starts + bucket, n)


def quantize(x: np.ndarray, bits: int, bucket: int = 128, u=None):
    """Codes, per-bucket (min, unit) and dequantized values of one layer.

    x: float32[n]; u: float32[n] uniforms for stochastic rounding or None (deterministic).
    Returns (codes uint8[n], mins f32[nb], units f32[nb], xhat f32[n])."""
    x = np.asarray(x, F32)
    n = x.size
    starts, ends = bucket_bounds(n, bucket)
    nb = starts.size
    codes = np.zeros(n, np.uint8)
    xhat = np.zeros(n, F32)
    mins = np.zeros(nb, F32)
    units = np.zeros(nb, F32)
    lv = F32(2 ** bits - 1)
    for j in range(nb):
        xb = x[starts[j]:ends[j]]
        m = xb.min()
        r = F32(xb.max() - m)
        with np.errstate(divide="ignore", over="ignore", invalid="ignore"):
            unit = F32(r / lv)
            inv = F32(lv / r)
        if not np.isfinite(inv):
            inv = F32(0.0)
        xm = xb - m
        if u is None:
            q = np.floor(fma32(xm, np.full(xm.shape, inv, F32), np.full(xm.shape, 0.5, F32)))
        else:
            q = np.floor(fma32(xm, np.full(xm.shape, inv, F32), u[starts[j]:ends[j]]))
        q = np.minimum(np.maximum(q, F32(0.0)), lv)
        codes[starts[j]:ends[j]] = q.astype(np.uint8)
        xhat[starts[j]:ends[j]] = fma32(q, np.full(q.shape, unit, F32), np.full(q.shape, m, F32))
        mins[j] = m
        units[j] = unit
    return codes, mins, units, xhat


def quantize_fast(x: np.ndarray, bits: int, bucket: int = 128, u=None):
    """Same arithmetic as quantize(), all buckets at once (whole buckets vectorised, the short
    tail bucket handled by quantize()).  Used on the multi-million-element workloads."""
    x = np.asarray(x, F32)
    n = x.size
    nfull = n // bucket
    lv = F32(2 ** bits - 1)
    codes = np.zeros(n, np.uint8)
    xhat = np.zeros(n, F32)
    nb = (n + bucket - 1) // bucket
    mins = np.zeros(nb, F32)
    units = np.zeros(nb, F32)
    if nfull:
        xb = x[:nfull * bucket].reshape(nfull, bucket)
        m = xb.min(axis=1, keepdims=True)
        r = (xb.max(axis=1, keepdims=True) - m).astype(F32)
        with np.errstate(divide="ignore", over="ignore", invalid="ignore"):
            unit = (r / lv).astype(F32)
            inv = (lv / r).astype(F32)
        inv = np.where(np.isfinite(inv), inv, F32(0.0)).astype(F32)
        xm = xb - m
        if u is None:
            q = np.floor(fma32(xm, np.broadcast_to(inv, xm.shape), np.full(xm.shape, 0.5, F32)))
        else:
            q = np.floor(fma32(xm, np.broadcast_to(inv, xm.shape), u[:nfull * bucket].reshape(nfull, bucket)))
        q = np.minimum(np.maximum(q, F32(0.0)), lv)
        codes[:nfull * bucket] = q.astype(np.uint8).reshape(-1)
        xhat[:nfull * bucket] = fma32(q, np.broadcast_to(unit, q.shape),
                                      np.broadcast_to(m, q.shape)).reshape(-1)
        mins[:nfull] = m[:, 0]
        units[:nfull] = unit[:, 0]
    if nfull * bucket < n:
        s = nfull * bucket
        c2, m2, u2, h2 = quantize(x[s:], bits, bucket, None if u is None else u[s:])
        codes[s:], xhat[s:], mins[nfull:], units[nfull:] = c2, h2, m2, u2
    return codes, mins, units, xhat


def squared_error(x: np.ndarray, xhat: np.ndarray) -> float:
    d = xhat.astype(np.float64) - x.astype(np.float64)
    return float(np.dot(d, d))


def layer_uniforms(seed: int, layer: int, n: int) -> np.ndarray:
    return philox.element_uniform(seed, layer, n)


def error(x: np.ndarray, bits: int, bucket: int = 128, u=None) -> float:
    _, _, _, xhat = quantize_fast(x, bits, bucket, u)
    return squared_error(x, xhat)


def size_bytes(n: int, bits: int, bucket: int = 128) -> int:
    total = 0
    for s in range(0, n, bucket):
        cnt = min(bucket, n - s)
        total += (cnt * bits + 7) // 8 + 8
    return total


def _bitstream(codes: np.ndarray, bits: int) -> np.ndarray:
    """LSB-first bit stream of one bucket: element i occupies bits [i*b, (i+1)*b); bit p of the
    stream is bit (p & 7) of byte (p >> 3); the last byte is zero-padded."""
    b = ((codes.astype(np.uint32)[:, None] >> np.arange(bits, dtype=np.uint32)) & 1).astype(np.uint8)
    return np.packbits(b.reshape(-1), bitorder="little")


def pack(codes: np.ndarray, mins: np.ndarray, units: np.ndarray, bits: int,
         bucket: int = 128) -> np.ndarray:
    """Layer payload (uint8 array): meta pairs first, then per-bucket bit streams."""
    n = codes.size
    meta = np.stack([mins.astype(F32), units.astype(F32)], axis=1).reshape(-1).view(np.uint8)
    out = [meta]
    nfull = n // bucket
    if nfull and (bucket * bits) % 8 == 0:
        # whole buckets end on a byte boundary, so their streams simply concatenate
        out.append(_bitstream(codes[:nfull * bucket], bits))
        rest = range(nfull * bucket, n, bucket)
    else:
        rest = range(0, n, bucket)
    for s in rest:
        out.append(_bitstream(codes[s:s + bucket], bits))
    return np.concatenate(out)


def unpack(payload: np.ndarray, n: int, bits: int, bucket: int = 128) -> np.ndarray:
    """Decode a layer payload back to the dequantized fp32 values."""
    nb = (n + bucket - 1) // bucket
    meta = payload[:8 * nb].view(F32).reshape(nb, 2)
    pos = 8 * nb
    xhat = np.zeros(n, F32)
    for j, s in enumerate(range(0, n, bucket)):
        cnt = min(bucket, n - s)
        nbytes = (cnt * bits + 7) // 8
        buf = payload[pos:pos + nbytes]
        pos += nbytes
        bitsarr = np.unpackbits(buf, bitorder="little")[:cnt * bits].reshape(cnt, bits)
        q = (bitsarr.astype(np.uint32) << np.arange(bits, dtype=np.uint32)).sum(axis=1).astype(F32)
        xhat[s:s + cnt] = fma32(q, np.full(cnt, meta[j, 1], F32), np.full(cnt, meta[j, 0], F32))
    return xhat


def compress(g: np.ndarray, e, bits: int, bucket: int = 128, u=None):
    """One layer: payload bytes and the new error-feedback buffer e' = fl32(x - xhat)."""
    x = form_x(g, e)
    codes, mins, units, xhat = quantize_fast(x, bits, bucket, u)
    return pack(codes, mins, units, bits, bucket), (x - xhat).astype(F32), codes, xhat
