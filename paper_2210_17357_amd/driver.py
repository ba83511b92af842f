"""Periodic run of the algorithm around the per-step compressor (section "Implementation" and
"Parameter ranges" of the paper's experimental setup): gradients are accumulated between runs;
every `period` steps, once `warmup` steps have passed, the error table is built on the
accumulated gradients (no error feedback), the budget is the uniform default's error, the DP picks
the per-layer parameters, and the communication engine uses them until the next run.

This class only sequences calls of the C ABI (accumulate, profile_solve, payload_layout,
compress); it does no arithmetic on gradients itself.
"""
from __future__ import annotations

import numpy as np

from . import binding as B


class PeriodicRun:
    def __init__(self, handle: "B.Handle", layers, cands, default: int, n_bins: int, period: int,
                 warmup: int = 0, bucket: int = 128):
        if period < 1 or warmup < 0:
            raise ValueError("period >= 1 and warmup >= 0")
        self.h, self.layers, self.cands = handle, layers, cands
        self.default, self.n_bins, self.period, self.warmup, self.bucket = default, n_bins, period, warmup, bucket
        self.choice = np.full(len(layers), default, np.int32)       # uniform default until the first run
        self.offsets = B.payload_layout(layers, cands, self.choice, bucket)
        self.step_count = 0
        self.in_window = 0
        self.acc = None
        self.last = None            # (errors, sizes, e_max, status) of the latest run

    def payload_bytes(self) -> int:
        """Upper bound of the payload buffer over every possible choice."""
        return int(B.sizes(self.layers, self.cands, self.bucket).max(axis=1).sum()) + 16 * (len(self.layers) + 1)

    def step(self, d_grads, d_ef, d_payload, d_q=None, d_q0=None):
        """One training step: accumulate, re-run the algorithm when a window ends, compress.
        Returns (choice, offsets) the payload was written with; compression is off (returns
        None) during the warm-up steps."""
        import torch
        if self.acc is None:
            self.acc = torch.empty_like(d_grads)
        self.h.accumulate(self.acc, d_grads, reset=self.in_window == 0)
        self.in_window += 1
        self.step_count += 1
        if self.step_count >= self.warmup and self.in_window >= self.period:
            st, errors, sizes, e_max, choice, _, _ = self.h.profile_solve(
                self.acc, None, self.layers, self.cands, self.default, self.n_bins, d_q0)
            if st == B.OK:
                self.choice = choice
                self.offsets = B.payload_layout(self.layers, self.cands, choice, self.bucket)
            self.last = (errors, sizes, e_max, st)
            self.in_window = 0
        if self.step_count <= self.warmup:
            return None
        self.h.compress(d_grads, d_ef, self.layers, self.cands, self.choice, d_payload, self.offsets, d_q)
        return self.choice, self.offsets
