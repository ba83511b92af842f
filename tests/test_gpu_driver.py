"""GPU: the periodic driver (accumulate -> every `period` steps profile on the accumulated
gradients, solve, then compress every step with the latest choice) against the same sequence
written out with the oracle."""
import numpy as np
import pytest

from oracle import pipeline, solver
from paper_2210_17357_amd import workloads as W

from gpu_util import tables, torch_cuda

pytestmark = pytest.mark.gpu


def test_accumulate_matches_fp32_sum():
    from paper_2210_17357_amd import binding as B
    torch = torch_cuda()
    rng = np.random.default_rng(0)
    for n in (1, 3, 4, 1027, 65536 + 5):
        a = rng.standard_normal(n).astype(np.float32)
        b = rng.standard_normal(n).astype(np.float32)
        h = B.Handle(max(n, 16), 1, 1)
        acc = torch.full((n,), 7.0, dtype=torch.float32, device="cuda")
        h.accumulate(acc, torch.from_numpy(a).cuda(), reset=True)
        assert np.array_equal(acc.cpu().numpy(), a)
        h.accumulate(acc, torch.from_numpy(b).cuda())
        assert np.array_equal(acc.cpu().numpy(), a + b)
        h.close()


def test_periodic_run_against_oracle_sequence():
    from paper_2210_17357_amd import binding as B
    from paper_2210_17357_amd.driver import PeriodicRun
    torch = torch_cuda()
    full = W.workload("c4_gpt2_medium_mixed")
    shapes = tuple(W.gpt2_medium_shapes(layers=1, d=128, d_ff=512, vocab=500, ctx=64))
    w = W.Workload("drv", shapes, full.candidates, full.default, 400, full.values, "zeros", full.scale_exp)
    cands = list(w.candidates)
    base = W.generate(w)
    L = len(base.numels)
    layers, ctab = tables(base, cands)
    h = B.Handle(int(base.grads.size), L, len(cands))
    period, warmup, steps = 3, 2, 8
    run = PeriodicRun(h, layers, ctab, w.default, w.n_bins, period, warmup)
    payload = torch.zeros(run.payload_bytes(), dtype=torch.uint8, device="cuda")
    ef_dev = torch.zeros(int(base.grads.size), dtype=torch.float32, device="cuda")
    # oracle-side state
    o_ef = np.zeros(int(base.grads.size), np.float32)
    o_acc = None
    o_choice = np.full(L, w.default, np.int32)
    in_window = 0
    n_runs = 0
    for s in range(1, steps + 1):
        grads = W.generate(W.Workload("drv", shapes, full.candidates, full.default, 400, full.values, "zeros",
                                      full.scale_exp, seed=100 + s)).grads
        got = run.step(torch.from_numpy(grads).cuda(), ef_dev, payload)
        o_acc = grads.copy() if in_window == 0 else (o_acc + grads).astype(np.float32)
        in_window += 1
        if s >= warmup and in_window >= period:
            errs = pipeline.profile(o_acc, None, base.offsets, base.numels, base.rows, base.cols, cands)
            szs = pipeline.sizes_table(base.numels, base.rows, base.cols, cands)
            ch, _, _ = solver.solve(errs, szs, solver.e_max_uniform(errs, w.default), w.n_bins)
            if ch is not None:
                # the GPU tables differ from the oracle's in the last digits: compare the choice the
                # GPU made from ITS tables with the oracle's solver on those same tables
                g_err, g_szs, g_emax, st = run.last
                assert st == B.OK and np.abs(g_err - errs).max() <= 1e-4 * np.abs(errs).max()
                ref_choice, _, _ = solver.solve(g_err, g_szs, g_emax, w.n_bins)
                o_choice = ref_choice
            in_window = 0
            n_runs += 1
        if s <= warmup:
            assert got is None
            continue
        choice, offsets = got
        assert np.array_equal(choice, o_choice), s
        pay = payload.cpu().numpy()
        for l in range(L):
            off, n = int(base.offsets[l]), int(base.numels[l])
            p_ref, e_ref, _ = pipeline.compress_layer(grads, o_ef, off, n, 0, 0, cands[o_choice[l]], l)
            assert np.array_equal(pay[offsets[l]:offsets[l] + p_ref.size], p_ref), (s, l)
            o_ef[off:off + n] = e_ref
        assert np.array_equal(ef_dev.cpu().numpy().view(np.uint32), o_ef.view(np.uint32)), s
    assert n_runs == 2 and not np.array_equal(o_choice, np.full(L, w.default))
    h.close()
