"""GPU parity, low-rank family: errors of all ranks from one power-iteration step (1e-4 relative
against the fp64 oracle), factors within 1e-3 relative Frobenius, error feedback and the warm
start update, through the C ABI."""
import numpy as np
import pytest

from oracle import lowrank, pipeline
from paper_2210_17357_amd import workloads as W

from gpu_util import rel_err, tables, to_device, torch_cuda

pytestmark = pytest.mark.gpu


def _frob_rel(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b.astype(np.float64)) /
                 max(np.linalg.norm(b.astype(np.float64)), 1e-300))


def _check(w, batch, ranks, compress_cycle=True, power_iters=1):
    from paper_2210_17357_amd import binding as B
    torch = torch_cuda()
    cands = [(W.LOWRANK, float(r)) for r in ranks]
    layers, ctab = tables(batch, cands)
    g, e, q0 = to_device(batch)
    L = len(batch.numels)
    h = B.Handle(int(batch.grads.size), L, len(cands), r_max=w.r_max, power_iters=power_iters)
    errors, sizes = h.profile(g, e, layers, ctab, q0)
    ref = pipeline.profile(batch.grads, batch.ef, batch.offsets, batch.numels, batch.rows, batch.cols, cands,
                           q0=batch.q0, q_offsets=batch.q_offsets, r_max=w.r_max, power_iters=power_iters)
    assert np.array_equal(sizes, pipeline.sizes_table(batch.numels, batch.rows, batch.cols, cands))
    # error_r is a difference of norms: 1e-4 relative.  Only where the oracle's error is itself
    # rounding noise (below 1e-8 ||X||^2: a full-rank layer gives ~1e-30 in fp64 and exactly 0 or
    # fp32 noise here) an absolute bound of 1e-6 ||X||^2 takes its place.
    xnorm = np.array([[float(np.sum((batch.grads[o:o + n].astype(np.float64)
                                      + (0 if batch.ef is None else batch.ef[o:o + n])) ** 2))]
                      for o, n in zip(batch.offsets, batch.numels)])
    bad = (rel_err(errors, ref) > 1e-4) & ~((ref < 1e-8 * xnorm) & (np.abs(errors - ref) <= 1e-6 * xnorm))
    assert not bad.any(), (np.argwhere(bad)[:5], errors[bad][:5], ref[bad][:5])
    errors2, _ = h.profile(g, e, layers, ctab, q0)
    assert np.array_equal(errors, errors2)

    if compress_cycle:
        choice = np.array([l % len(cands) for l in range(L)], np.int32)
        offsets = B.payload_layout(layers, ctab, choice)
        payload = torch.zeros(int(offsets[-1]) + 16, dtype=torch.uint8, device="cuda")
        ef_dev = e.clone() if e is not None else torch.zeros_like(g)
        q_dev = q0.clone()
        h.compress(g, ef_dev, layers, ctab, choice, payload, offsets, q_dev)
        pay, new_ef, new_q = payload.cpu().numpy(), ef_dev.cpu().numpy(), q_dev.cpu().numpy()
        for l in range(L):
            off, n = int(batch.offsets[l]), int(batch.numels[l])
            m_, n_ = int(batch.rows[l]), int(batch.cols[l])
            r = int(cands[choice[l]][1])
            q0l = batch.q0[int(batch.q_offsets[l]):int(batch.q_offsets[l]) + n_ * w.r_max].reshape(n_, w.r_max)
            phat, q, e_ref = lowrank.compress(batch.grads[off:off + n],
                                              None if batch.ef is None else batch.ef[off:off + n], m_, n_, q0l, r,
                                              power_iters)
            got_p = pay[offsets[l]:offsets[l] + 4 * m_ * r].view(np.float32).reshape(m_, r)
            got_q = pay[offsets[l] + 4 * m_ * r:offsets[l] + 4 * (m_ + n_) * r].view(np.float32).reshape(n_, r)
            assert sizes[l, choice[l]] == 4 * (m_ + n_) * r
            assert _frob_rel(got_p, phat) < 1e-3, ("Phat", l, m_, n_, r, _frob_rel(got_p, phat))
            assert _frob_rel(got_q, q) < 1e-3, ("Q", l, m_, n_, r, _frob_rel(got_q, q))
            x = batch.grads[off:off + n].astype(np.float64)
            if batch.ef is not None:
                x = (batch.grads[off:off + n] + batch.ef[off:off + n]).astype(np.float64)
            scale = np.linalg.norm(x)
            assert np.linalg.norm(new_ef[off:off + n].astype(np.float64) - e_ref.astype(np.float64)) < 1e-3 * scale
            # the residual left in the error feedback has the profiled energy
            resid = float(np.sum(new_ef[off:off + n].astype(np.float64) ** 2))
            assert abs(resid - ref[l, choice[l]]) < 1e-3 * ref[l, choice[l]] + 1e-12 * scale ** 2
            # warm start: first r columns of the layer's block replaced by the new Q, rest untouched
            blk = new_q[int(batch.q_offsets[l]):int(batch.q_offsets[l]) + n_ * w.r_max].reshape(n_, w.r_max)
            assert np.array_equal(blk[:, :r], got_q)
            assert np.array_equal(blk[:, r:], q0l[:, r:])
    h.close()
    return errors, ref


def test_transformer_lm_workload_subset():
    # embedding (32768 x 512), one decoder block's matrices, and the next block's first matrix
    w = W.workload("c3_transformer_lm_lowrank")
    tensors = [0] + list(range(1, 18))
    batch = W.generate(w, tensors)
    assert len(batch.numels) == 7
    errors, ref = _check(w, batch, W.LOWRANK_RANKS)
    assert np.all(np.diff(errors, axis=1) <= 0)


def test_odd_shapes_and_error_feedback():
    rng = np.random.default_rng(0)
    shapes = [(37, 53), (130, 70), (64, 64), (5, 300), (300, 5), (129, 257), (256, 36)]
    w = W.Workload("lr_odd", tuple(shapes), tuple((W.LOWRANK, float(r)) for r in (1, 3, 4, 5)), 2, 100,
                   "lowrank64", "normal0.1", (-3.0, -1.0), r_max=8)
    batch = W.generate(w)
    assert batch.ef is not None
    _check(w, batch, (1, 3, 4, 5))


def test_full_workload_errors_and_solve():
    from oracle import solver
    from paper_2210_17357_amd import binding as B
    w = W.workload("c3_transformer_lm_lowrank")
    tensors = [0] + [t for t in range(1, 1 + 16 * 4) ]       # embedding + four decoder blocks
    batch = W.generate(w, tensors, threads=8)
    errors, ref = _check(w, batch, W.LOWRANK_RANKS, compress_cycle=False)
    layers, ctab = tables(batch, list(w.candidates))
    h = B.Handle(int(batch.grads.size), len(batch.numels), 5, r_max=64)
    sizes = B.sizes(layers, ctab)
    e_max = B.emax(errors, w.default)
    st, choice, tsize, _ = h.solve(errors, sizes, e_max, w.n_bins)
    rc, rs, _ = solver.solve(errors, sizes, e_max, w.n_bins)
    assert st == B.OK and np.array_equal(choice, rc) and tsize == rs
    h.close()


def test_rank_deficient_and_zero_matrices():
    from paper_2210_17357_amd import binding as B
    torch = torch_cuda()
    rng = np.random.default_rng(3)
    a = (rng.standard_normal((96, 3)) @ rng.standard_normal((3, 80))).astype(np.float32)     # rank 3
    z = np.zeros((40, 48), np.float32)
    g = np.concatenate([a.reshape(-1), z.reshape(-1)])
    q0 = np.concatenate([rng.standard_normal((80, 8)).astype(np.float32).reshape(-1),
                         rng.standard_normal((48, 8)).astype(np.float32).reshape(-1)])
    layers = B.layer_table([0, a.size], [a.size, z.size], [96, 40], [80, 48])
    cands = [(W.LOWRANK, 2.0), (W.LOWRANK, 3.0), (W.LOWRANK, 8.0)]
    ctab = B.cand_table(cands)
    h = B.Handle(g.size, 2, 3, r_max=8)
    errors, _ = h.profile(torch.from_numpy(g).cuda(), None, layers, ctab, torch.from_numpy(q0).cuda())
    total = float(np.sum(a.astype(np.float64) ** 2))
    ref2 = lowrank.error(a, q0[:640].reshape(80, 8), 2)
    assert abs(errors[0, 0] - ref2) < 1e-4 * ref2
    assert errors[0, 1] < 1e-6 * total and errors[0, 2] < 1e-6 * total      # exact rank recovered
    assert np.all(errors[1] == 0.0)
    # compress at rank 8 > true rank: the product Phat Q^T still reconstructs the matrix
    choice = np.array([2, 2], np.int32)
    offsets = B.payload_layout(layers, ctab, choice)
    payload = torch.zeros(int(offsets[-1]) + 16, dtype=torch.uint8, device="cuda")
    ef = torch.zeros(g.size, device="cuda")
    qd = torch.from_numpy(q0).cuda()
    h.compress(torch.from_numpy(g).cuda(), ef, layers, ctab, choice, payload, offsets, qd)
    pay = payload.cpu().numpy()
    p = pay[:4 * 96 * 8].view(np.float32).reshape(96, 8).astype(np.float64)
    q = pay[4 * 96 * 8:4 * (96 + 80) * 8].view(np.float32).reshape(80, 8).astype(np.float64)
    assert np.linalg.norm(p @ q.T - a) < 1e-4 * np.linalg.norm(a)
    assert float(ef.abs().max()) < 1e-4 * float(np.abs(a).max())
    assert np.all(np.isfinite(pay[:offsets[-1]].view(np.float32)))
    h.close()


def test_five_power_iteration_steps_reach_the_svd_tail():
    """Appendix "Low-rank error computation": with 5 power steps the error of every rank is
    close to the optimum sum_{i>r} sigma_i^2 of the SVD; parity with the oracle at 5 steps, and the
    GPU errors against the host SVD directly."""
    full = W.workload("c3_transformer_lm_lowrank")
    shapes = tuple(W.transformer_lm_shapes(layers=1, d=128, d_ff=512, vocab=1000)) + ((96, 200), (300, 70))
    w = W.Workload("lr_small", shapes, full.candidates, full.default, 400, full.values, full.ef, full.scale_exp,
                   only_2d=True)
    batch = W.generate(w)
    errors, ref = _check(w, batch, W.LOWRANK_RANKS, power_iters=5)
    one, _ = _check(w, batch, W.LOWRANK_RANKS, compress_cycle=False, power_iters=1)
    for l in range(len(batch.numels)):
        off, n = int(batch.offsets[l]), int(batch.numels[l])
        x = batch.grads[off:off + n].astype(np.float64).reshape(int(batch.rows[l]), int(batch.cols[l]))
        sv = np.linalg.svd(x, compute_uv=False) ** 2
        for c, r in enumerate(W.LOWRANK_RANKS):
            tail = float(sv[r:].sum())
            assert errors[l, c] >= tail * (1 - 1e-4) - 1e-7 * sv.sum()       # Eckart-Young
            assert errors[l, c] <= one[l, c] * (1 + 1e-4) + 1e-7 * sv.sum()  # more steps never hurt here
            if r < min(x.shape):
                assert errors[l, c] - tail <= 0.5 * (one[l, c] - tail) + 1e-7 * sv.sum()
