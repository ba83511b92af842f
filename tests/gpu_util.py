"""Helpers for the GPU parity tests: move a synthetic batch to the device and call the C ABI
through the binding."""
import numpy as np


def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def to_device(batch):
    torch = torch_cuda()
    g = torch.from_numpy(batch.grads).cuda()
    e = None if batch.ef is None else torch.from_numpy(batch.ef).cuda()
    q = None if batch.q0 is None else torch.from_numpy(batch.q0).cuda()
    return g, e, q


def tables(batch, cands):
    from paper_2210_17357_amd import binding as B
    return (B.layer_table(batch.offsets, batch.numels, batch.rows, batch.cols), B.cand_table(cands))


def rel_err(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return np.abs(a - b) / np.maximum(np.abs(b), 1e-300)
