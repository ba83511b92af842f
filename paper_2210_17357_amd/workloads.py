"""Seeded synthetic gradient workloads (shapes, value distributions, candidate lists).

This module holds NO arithmetic of the method: it only lists tensor shapes, draws
random values and lays tensors out in one flat buffer.  Both the CPU oracle's tests
and the HIP path's tests / benchmark take their inputs from here.

The five workloads stand in for the paper's gradient workloads (CIFAR-100 /
ImageNet CNNs, WikiText-103 transformers; Experimental setup section), which need
datasets and trained models that are not available: only tensor shapes and value
distributions are imitated.

Recipe (every tensor t of a workload with seed s has its own stream):
    rng_t   = numpy Generator(PCG64(SeedSequence([s, t])))
    scale_t = 10 ** rng_t.uniform(lo, hi)          (drawn first)
    values  = distribution(rng_t) * scale_t        (drawn second, fp64 -> fp32)
    ef      = ef_distribution(rng_t)               (drawn third, if the workload has one)
Per-tensor streams let a test generate one layer of the 355 M-element workload
without drawing the others.  `variant` v > 0 stands for a later step of the same run: scale_t as
above, values and ef from Generator(PCG64(SeedSequence([s, t, v]))).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

QUANT, TOPK, LOWRANK = 0, 1, 2

QUANT_BITS = (2, 3, 4, 5, 6, 7, 8)
TOPK_DENSITIES = (0.001, 0.005, 0.01, 0.02, 0.05, 0.1)
LOWRANK_RANKS = (4, 8, 16, 32, 64)


# --------------------------------------------------------------------------- shapes
def tiny_shapes() -> List[Tuple[int, ...]]:
    return [(16, 3, 3, 3), (32, 16, 3, 3), (64, 32, 3, 3), (10, 256)]


def _bn(c: int) -> List[Tuple[int, ...]]:
    return [(c,), (c,)]


def resnet18_shapes(num_classes: int = 1000) -> List[Tuple[int, ...]]:
    s: List[Tuple[int, ...]] = [(64, 3, 7, 7)] + _bn(64)
    inp = 64
    for stage, planes in enumerate((64, 128, 256, 512)):
        for block in range(2):
            s += [(planes, inp, 3, 3)] + _bn(planes)
            s += [(planes, planes, 3, 3)] + _bn(planes)
            if block == 0 and stage > 0:
                s += [(planes, inp, 1, 1)] + _bn(planes)
            inp = planes
    s += [(num_classes, 512), (num_classes,)]
    return s


def resnet50_shapes(num_classes: int = 1000) -> List[Tuple[int, ...]]:
    s: List[Tuple[int, ...]] = [(64, 3, 7, 7)] + _bn(64)
    inp = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for block in range(blocks):
            s += [(planes, inp, 1, 1)] + _bn(planes)
            s += [(planes, planes, 3, 3)] + _bn(planes)
            s += [(4 * planes, planes, 1, 1)] + _bn(4 * planes)
            if block == 0:
                s += [(4 * planes, inp, 1, 1)] + _bn(4 * planes)
            inp = 4 * planes
    s += [(num_classes, 2048), (num_classes,)]
    return s


def transformer_lm_shapes(layers: int = 16, d: int = 512, d_ff: int = 2048,
                          vocab: int = 32768) -> List[Tuple[int, ...]]:
    s: List[Tuple[int, ...]] = [(vocab, d)]
    for _ in range(layers):
        s += [(d,), (d,)]                                   # layer norm 1
        for _proj in range(4):                              # q, k, v, o
            s += [(d, d), (d,)]
        s += [(d,), (d,)]                                   # layer norm 2
        s += [(d_ff, d), (d_ff,), (d, d_ff), (d,)]          # fc1, fc2
    s += [(d,), (d,)]                                       # final layer norm
    return s


def gpt2_medium_shapes(layers: int = 24, d: int = 1024, d_ff: int = 4096,
                       vocab: int = 50257, ctx: int = 1024) -> List[Tuple[int, ...]]:
    s: List[Tuple[int, ...]] = [(vocab, d), (ctx, d)]
    for _ in range(layers):
        s += [(d,), (d,)]                                   # ln_1
        s += [(d, 3 * d), (3 * d,)]                         # fused qkv
        s += [(d, d), (d,)]                                 # attention projection
        s += [(d,), (d,)]                                   # ln_2
        s += [(d, d_ff), (d_ff,), (d_ff, d), (d,)]          # mlp
    s += [(d,), (d,)]                                       # ln_f
    return s


# ------------------------------------------------------------------------ workloads
@dataclass(frozen=True)
class Workload:
    name: str
    shapes: Tuple[Tuple[int, ...], ...]
    candidates: Tuple[Tuple[int, float], ...]      # (family, parameter)
    default: int                                   # index of the uniform default candidate
    n_bins: int
    values: str                                    # "student_t3" | "laplace" | "lowrank64"
    ef: str                                        # "zeros" | "normal0.1" | "same" | "none"
    scale_exp: Tuple[float, float]                 # per-layer scale = 10**U(lo, hi)
    seed: int = 0
    stochastic: bool = False
    bucket: int = 128
    only_2d: bool = False                          # 1-D tensors are sent raw, not profiled
    q_seed: int = 1
    r_max: int = 64
    variant: int = 0                               # another draw of the same model: see draw_tensor


def _cands(family: int, params: Sequence[float]) -> Tuple[Tuple[int, float], ...]:
    return tuple((family, float(p)) for p in params)


def workload(name: str) -> Workload:
    if name == "c0_tiny_quant":
        return Workload(name, tuple(tiny_shapes()), _cands(QUANT, QUANT_BITS), 2, 50,
                        "student_t3", "zeros", (-4.0, -2.0))
    if name == "c1_resnet18_quant":
        return Workload(name, tuple(resnet18_shapes()), _cands(QUANT, QUANT_BITS), 2, 1000,
                        "student_t3", "normal0.1", (-5.0, -2.0), stochastic=True)
    if name == "c2_resnet50_topk":
        return Workload(name, tuple(resnet50_shapes()), _cands(TOPK, TOPK_DENSITIES), 2, 1000,
                        "laplace", "same", (-5.0, -2.0))
    if name == "c3_transformer_lm_lowrank":
        return Workload(name, tuple(transformer_lm_shapes()), _cands(LOWRANK, LOWRANK_RANKS), 2,
                        2000, "lowrank64", "none", (-4.0, -2.0), only_2d=True)
    if name == "c4_gpt2_medium_mixed":
        return Workload(name, tuple(gpt2_medium_shapes()),
                        _cands(QUANT, QUANT_BITS) + _cands(TOPK, TOPK_DENSITIES), 2, 4000,
                        "student_t3", "normal0.1", (-5.0, -2.0))
    raise KeyError(name)


WORKLOADS = ("c0_tiny_quant", "c1_resnet18_quant", "c2_resnet50_topk",
             "c3_transformer_lm_lowrank", "c4_gpt2_medium_mixed")


# ----------------------------------------------------------------------- generation
@dataclass
class Batch:
    """One flat gradient buffer with its layer table."""
    grads: np.ndarray                      # float32 [total]
    ef: Optional[np.ndarray]               # float32 [total] or None
    offsets: np.ndarray                    # int64 [L]  (elements, into grads)
    numels: np.ndarray                     # int64 [L]
    rows: np.ndarray                       # int32 [L]  (0 for 1-D tensors)
    cols: np.ndarray                       # int32 [L]
    tensor_index: np.ndarray               # int64 [L]  index into Workload.shapes
    raw_bytes: int = 0                     # bytes of tensors not in the layer table
    q0: Optional[np.ndarray] = None        # float32 flat, per layer [cols x r_max], LOWRANK only
    q_offsets: Optional[np.ndarray] = None  # int64 [L] element offsets into q0


def tensor_rng(seed: int, t: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(t)])))


def draw_tensor(w: Workload, t: int) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Values and error-feedback of tensor t of workload w, flattened (row-major) fp32."""
    shape = w.shapes[t]
    n = int(np.prod(shape))
    rng = tensor_rng(w.seed, t)
    scale = 10.0 ** rng.uniform(*w.scale_exp)
    if w.variant:
        # a later step of the same training run: every tensor keeps its scale, values and error
        # feedback are a fresh draw from a stream of their own (variant 0 is the recipe above)
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(w.seed), int(t), int(w.variant)])))
    if w.values == "student_t3":
        v = rng.standard_t(3, n)
    elif w.values == "laplace":
        v = rng.laplace(0.0, 1.0, n)
    elif w.values == "lowrank64":
        if len(shape) >= 2:
            m, k = shape[0], n // shape[0]
            a = rng.standard_normal((m, 64))
            b = rng.standard_normal((64, k))
            v = ((a @ b) / 8.0 + 0.05 * rng.standard_normal((m, k))).reshape(-1)
        else:
            v = rng.standard_normal(n)
    else:
        raise ValueError(w.values)
    g = (v * scale).astype(np.float32)
    if w.ef == "zeros":
        e = np.zeros(n, np.float32)
    elif w.ef == "normal0.1":
        e = (rng.standard_normal(n) * (0.1 * scale)).astype(np.float32)
    elif w.ef == "same":
        e = (rng.laplace(0.0, 1.0, n) * scale).astype(np.float32)
    elif w.ef == "none":
        e = None
    else:
        raise ValueError(w.ef)
    return g, e


def draw_q0(w: Workload, t: int) -> np.ndarray:
    """Warm-start Q for tensor t: N(0,1), [cols x r_max] row-major fp32."""
    shape = w.shapes[t]
    cols = int(np.prod(shape[1:]))
    rng = tensor_rng(w.q_seed, t)
    return rng.standard_normal((cols, w.r_max)).astype(np.float32)


def layout(w: Workload, tensors: Optional[Sequence[int]] = None):
    """Offsets of the chosen tensors packed back to back (no padding), and the layer
    table (only >=2-D tensors when w.only_2d)."""
    idx = list(range(len(w.shapes))) if tensors is None else list(tensors)
    off = 0
    offs, numels, rows, cols, tix = [], [], [], [], []
    raw = 0
    for t in idx:
        shape = w.shapes[t]
        n = int(np.prod(shape))
        if len(shape) >= 2 or not w.only_2d:
            offs.append(off)
            numels.append(n)
            rows.append(shape[0] if len(shape) >= 2 else 0)
            cols.append(n // shape[0] if len(shape) >= 2 else 0)
            tix.append(t)
        else:
            raw += 4 * n
        off += n
    return (off, np.asarray(offs, np.int64), np.asarray(numels, np.int64),
            np.asarray(rows, np.int32), np.asarray(cols, np.int32),
            np.asarray(tix, np.int64), raw)


def generate(w: Workload, tensors: Optional[Sequence[int]] = None, threads: int = 1) -> Batch:
    """Draw the whole workload (or the listed tensors of it) into one flat buffer.  Tensors have
    independent streams, so `threads` > 1 only changes how long this takes."""
    idx = list(range(len(w.shapes))) if tensors is None else list(tensors)
    total, offs, numels, rows, cols, tix, raw = layout(w, idx)
    grads = np.empty(total, np.float32)
    ef = None if w.ef == "none" else np.empty(total, np.float32)
    starts, pos = [], 0
    for t in idx:
        starts.append(pos)
        pos += int(np.prod(w.shapes[t]))

    def fill(j):
        g, e = draw_tensor(w, idx[j])
        grads[starts[j]:starts[j] + g.size] = g
        if ef is not None:
            ef[starts[j]:starts[j] + g.size] = e

    if threads > 1:
        from concurrent.futures import ThreadPoolExecutor
        order = sorted(range(len(idx)), key=lambda j: -int(np.prod(w.shapes[idx[j]])))
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, order))
    else:
        for j in range(len(idx)):
            fill(j)
    b = Batch(grads, ef, offs, numels, rows, cols, tix, raw)
    if any(f == LOWRANK for f, _ in w.candidates):
        qs, qo, qpos = [], [], 0
        for t in tix:
            q = draw_q0(w, int(t))
            qo.append(qpos)
            qs.append(q.reshape(-1))
            qpos += q.size
        b.q0 = np.concatenate(qs) if qs else np.zeros(0, np.float32)
        b.q_offsets = np.asarray(qo, np.int64)
    return b
