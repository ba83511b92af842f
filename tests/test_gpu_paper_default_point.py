"""GPU parity at the paper's default operating point: D = 10000 error bins, candidate lists from
the range rule (49 ranks around 32, 100 densities around 1 %, 7 bit-widths around 4), i.e. more
candidates than one pass of the Top-K path resolves and up to 100 entries per layer in the
solver.  Profile -> solve against the oracle on cut-down models."""
import numpy as np
import pytest

from oracle import pipeline, solver
from paper_2210_17357_amd import workloads as W

from gpu_util import rel_err, tables, to_device, torch_cuda

pytestmark = pytest.mark.gpu

D = 10000


def _solve_both(h, errors, sizes, default):
    from paper_2210_17357_amd import binding as B
    e_max = B.emax(errors, default)
    st, choice, tsize, terr = h.solve(errors, sizes, e_max, D)
    ref_choice, ref_size, _ = solver.solve(errors, sizes, e_max, D)
    assert st == B.OK and np.array_equal(choice, ref_choice) and tsize == ref_size
    assert tsize <= int(sizes[:, default].sum())
    return choice


def test_hundred_densities_topk():
    from paper_2210_17357_amd import binding as B
    cands, default = B.candidate_range(W.TOPK, 0.01)
    shapes = tuple(W.resnet18_shapes(num_classes=100))[:30] + ((70000,), (3, 5, 7))
    w = W.Workload("tk100", shapes, tuple(cands), default, D, "laplace", "same", (-5.0, -2.0))
    batch = W.generate(w)
    layers, ctab = tables(batch, cands)
    g, e, _ = to_device(batch)
    L = len(batch.numels)
    h = B.Handle(int(batch.grads.size), L, len(cands))
    errors, sizes = h.profile(g, e, layers, ctab)
    ref = pipeline.profile(batch.grads, batch.ef, batch.offsets, batch.numels, batch.rows, batch.cols, cands)
    assert np.array_equal(sizes, pipeline.sizes_table(batch.numels, batch.rows, batch.cols, cands))
    bad = (rel_err(errors, ref) > 1e-4) & (np.abs(errors - ref) > 1e-60)
    assert not bad.any(), np.argwhere(bad)[:5]
    assert (np.diff(errors, axis=1) <= 0).all()
    errors2, _ = h.profile(g, e, layers, ctab)
    assert np.array_equal(errors, errors2)
    _solve_both(h, errors, sizes, default)
    h.close()


def test_forty_nine_ranks_lowrank():
    from paper_2210_17357_amd import binding as B
    cands, default = B.candidate_range(W.LOWRANK, 32, r_max=64)
    full = W.workload("c3_transformer_lm_lowrank")
    shapes = tuple(W.transformer_lm_shapes(layers=2, d=128, d_ff=512, vocab=1000))
    w = W.Workload("lr49", shapes, tuple(cands), default, D, full.values, full.ef, full.scale_exp, only_2d=True)
    batch = W.generate(w)
    layers, ctab = tables(batch, cands)
    g, e, q0 = to_device(batch)
    L = len(batch.numels)
    h = B.Handle(int(batch.grads.size), L, len(cands), r_max=64)
    errors, sizes = h.profile(g, e, layers, ctab, q0)
    ref = pipeline.profile(batch.grads, batch.ef, batch.offsets, batch.numels, batch.rows, batch.cols, cands,
                           q0=batch.q0, q_offsets=batch.q_offsets, r_max=64)
    xnorm = np.array([[float(np.sum(batch.grads[o:o + n].astype(np.float64) ** 2))]
                      for o, n in zip(batch.offsets, batch.numels)])
    bad = (rel_err(errors, ref) > 1e-4) & ~((ref < 1e-8 * xnorm) & (np.abs(errors - ref) <= 1e-6 * xnorm))
    assert not bad.any(), np.argwhere(bad)[:5]
    _solve_both(h, errors, sizes, default)
    h.close()


def test_mixed_lists_from_the_range_rule_and_wide_solver_tables():
    from paper_2210_17357_amd import binding as B
    qc, qd = B.candidate_range(W.QUANT, 4)
    tc, td = B.candidate_range(W.TOPK, 0.01)
    cands = qc + tc[:40]                       # 47 candidates, two Top-K groups beyond the first
    shapes = tuple(W.gpt2_medium_shapes(layers=1, d=128, d_ff=512, vocab=1000, ctx=64))
    w = W.Workload("mix47", shapes, tuple(cands), qd, D, "student_t3", "normal0.1", (-5.0, -2.0))
    batch = W.generate(w)
    layers, ctab = tables(batch, cands)
    g, e, _ = to_device(batch)
    L = len(batch.numels)
    h = B.Handle(int(batch.grads.size), L, len(cands))
    errors, sizes = h.profile(g, e, layers, ctab)
    ref = pipeline.profile(batch.grads, batch.ef, batch.offsets, batch.numels, batch.rows, batch.cols, cands)
    assert rel_err(errors, ref).max() < 1e-4
    choice = _solve_both(h, errors, sizes, qd)
    # random wide tables: up to 128 candidates per layer, many distinct bins survive the host's pruning
    rng = np.random.default_rng(2)
    h2 = B.Handle(1024, 20, 128)
    for trial in range(6):
        Lr, P = 20, 128 if trial % 2 else 100
        err = np.sort(rng.random((Lr, P)), axis=1)[:, ::-1] * 10.0 ** rng.uniform(-3, 0, (Lr, 1))
        szs = np.sort(rng.integers(1, 1 << 20, (Lr, P)), axis=1).astype(np.int64)    # size up as error goes down
        e_max = solver.e_max_uniform(err, P // 2)
        st, ch, ts, te = h2.solve(err, szs, e_max, D)
        rc, rs, _ = solver.solve(err, szs, e_max, D)
        assert st == B.OK and np.array_equal(ch, rc) and ts == rs
    h2.close()
    # compress with the chosen mixed setting still round-trips through the oracle
    torch = torch_cuda()
    offsets = B.payload_layout(layers, ctab, choice)
    payload = torch.zeros(int(offsets[-1]) + 16, dtype=torch.uint8, device="cuda")
    ef_dev = e.clone()
    h.compress(g, ef_dev, layers, ctab, choice, payload, offsets)
    pay, new_ef = payload.cpu().numpy(), ef_dev.cpu().numpy()
    for l in range(L):
        off, n = int(batch.offsets[l]), int(batch.numels[l])
        p_ref, e_ref, _ = pipeline.compress_layer(batch.grads, batch.ef, off, n, 0, 0, cands[choice[l]], l)
        assert np.array_equal(pay[offsets[l]:offsets[l] + p_ref.size], p_ref), l
        assert np.array_equal(new_ef[off:off + n].view(np.uint32), e_ref.view(np.uint32)), l
    h.close()
