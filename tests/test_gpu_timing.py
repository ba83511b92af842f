"""Kernel timing of the library (lgreco_set_timing / lgreco_get_timing_of): the brackets must not
change any result, and what they report must be consistent with the host's own clock."""
import time

import numpy as np
import pytest

from paper_2210_17357_amd import workloads as W

from gpu_util import tables, to_device, torch_cuda

pytestmark = pytest.mark.gpu


def _workload(kind):
    if kind == "mixed":
        w = W.workload("c4_gpt2_medium_mixed")
        shapes = tuple(W.gpt2_medium_shapes(layers=2, d=256, d_ff=1024, vocab=3000, ctx=64))
        return W.Workload("timing_mixed", shapes, w.candidates, w.default, 400, w.values, w.ef, w.scale_exp)
    w = W.workload("c3_transformer_lm_lowrank")
    shapes = tuple(s for s in W.transformer_lm_shapes(layers=1, d=256, d_ff=512, vocab=1024) if len(s) == 2)
    return W.Workload("timing_lowrank", shapes, w.candidates, w.default, 200, w.values, w.ef, w.scale_exp,
                      only_2d=True, r_max=w.r_max)


@pytest.mark.parametrize("kind", ["mixed", "lowrank"])
def test_brackets_leave_results_alone_and_fit_the_host_clock(kind):
    from paper_2210_17357_amd import binding as B
    torch = torch_cuda()
    w = _workload(kind)
    batch = W.generate(w)
    cands = list(w.candidates)
    layers, ctab = tables(batch, cands)
    g, e, q0 = to_device(batch)
    L = len(batch.numels)
    stream = torch.cuda.current_stream().cuda_stream
    results = {}
    for level in (0, 1, 2):
        h = B.Handle(int(batch.grads.size), L, len(cands), r_max=w.r_max)
        h.set_timing(level)
        for rep in range(2):            # the second pass reuses every cached table
            ef = e.clone() if e is not None else torch.zeros_like(g)
            q = q0.clone() if q0 is not None else None
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            st, errors, sizes, e_max, choice, tsize, terr = h.profile_solve(
                g, e, layers, ctab, w.default, w.n_bins, q0, stream=stream)
            t1 = time.perf_counter()
            assert st == B.OK
            offsets = B.payload_layout(layers, ctab, choice)
            payload = torch.zeros(int(offsets[-1]) + 16, dtype=torch.uint8, device="cuda")
            h.compress(g, ef, layers, ctab, choice, payload, offsets, q, stream=stream)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            prof = h.get_timing(B.CALL_PROFILE)
            solve = h.get_timing(B.CALL_SOLVE)
            comp = h.get_timing(B.CALL_COMPRESS)
            if level == 0:
                assert prof == [] and comp == [] and solve == []
                assert h.get_timing_totals(B.CALL_COMPRESS) == []
            else:
                names_p = [n for n, _ in prof]
                names_c = [n for n, _ in comp]
                assert "dp_solve" in [n for n, _ in solve]
                if kind == "mixed":
                    assert "quant_profile_topk_collect" in names_p
                    assert "quant_compress" in names_c or "topk_collect" in names_c
                else:
                    assert "lowrank_gemm_p" in names_p and "lowrank_gemm_q" in names_p
                    assert "lowrank_ef" in names_c
                if level == 2:
                    assert len(names_p) > sum(1 for n in names_p if n.startswith(("quant_profile", "lowrank_gemm")))
                for n, ms in prof + solve + comp:
                    assert np.isfinite(ms) and ms >= 0.0, (n, ms)
                # sections of one call do not overlap: their sum fits in the call's wall clock
                # (a phase bracket spans the sections of its call; the dotted names are parts of dp_solve)
                def inner(secs):
                    return [ms for n, ms in secs if "." not in n and not n.startswith("phase_")]
                assert sum(inner(prof + solve)) <= (t1 - t0) * 1e3 + 0.05, (level, prof, solve, t1 - t0)
                assert sum(inner(comp)) <= (t2 - t1) * 1e3 + 0.05, (level, comp, t2 - t1)
                phase_p, phase_c = dict(prof)["phase_profile"], dict(comp)["phase_compress"]
                assert sum(inner(prof)) <= phase_p + 0.02 and phase_p <= (t1 - t0) * 1e3 + 0.05, (prof, t1 - t0)
                assert sum(inner(comp)) <= phase_c + 0.02 and phase_c <= (t2 - t1) * 1e3 + 0.05, (comp, t2 - t1)
                # the main kernels do real work: none of them reads as zero
                assert all(ms > 0.0 for n, ms in prof + comp if n in
                           ("quant_profile_topk_collect", "quant_compress", "topk_collect", "lowrank_gemm_p",
                            "lowrank_gemm_q", "lowrank_ef")), (prof, comp)
                # totals since set_timing: one entry per section, `rep + 1` calls each, the last
                # call's reading included
                for call, last_read in ((B.CALL_PROFILE, prof), (B.CALL_SOLVE, solve), (B.CALL_COMPRESS, comp)):
                    totals = {n: (ms, c) for n, ms, c in h.get_timing_totals(call)}
                    assert set(totals) == {n for n, _ in last_read}, (call, totals, last_read)
                    for n, ms in last_read:
                        assert totals[n][1] == rep + 1, (n, totals[n])
                        assert totals[n][0] >= ms * (1 - 1e-6), (n, totals[n], ms)
            out = (errors.copy(), choice.copy(), payload.cpu().numpy(), ef.cpu().numpy().view(np.uint32),
                   None if q is None else q.cpu().numpy().view(np.uint32))
            if rep == 1:
                results[level] = out
        h.close()
    for level in (1, 2):
        for a, b in zip(results[0], results[level]):
            assert (a is None and b is None) or np.array_equal(a, b), level


def test_stride_times_every_nth_call_only():
    """lgreco_set_timing_stride(3): calls 0, 3, 6 of each kind carry events, the others none; the
    totals count exactly those; results are the same in every call."""
    from paper_2210_17357_amd import binding as B
    torch = torch_cuda()
    w = _workload("mixed")
    batch = W.generate(w)
    cands = list(w.candidates)
    layers, ctab = tables(batch, cands)
    g, e, _ = to_device(batch)
    L = len(batch.numels)
    h = B.Handle(int(batch.grads.size), L, len(cands))
    h.set_timing(1)
    h.set_timing_stride(3)
    first = None
    for i in range(7):
        ef = e.clone()
        st, errors, sizes, e_max, choice, tsize, terr = h.profile_solve(g, e, layers, ctab, w.default, w.n_bins)
        assert st == B.OK
        offsets = B.payload_layout(layers, ctab, choice)
        payload = torch.zeros(int(offsets[-1]) + 16, dtype=torch.uint8, device="cuda")
        h.compress(g, ef, layers, ctab, choice, payload, offsets)
        timed = i % 3 == 0
        assert (len(h.get_timing(B.CALL_PROFILE)) > 0) == timed, i
        assert (len(h.get_timing(B.CALL_COMPRESS)) > 0) == timed, i
        out = (errors.copy(), choice.copy(), payload.cpu().numpy(), ef.cpu().numpy().view(np.uint32))
        if first is None:
            first = out
        for a, b in zip(first, out):
            assert np.array_equal(a, b), i
    for call in (B.CALL_PROFILE, B.CALL_SOLVE, B.CALL_COMPRESS):
        totals = h.get_timing_totals(call)
        assert totals and all(c == 3 for _, _, c in totals), totals
    with pytest.raises(B.LgrecoError):
        h.set_timing_stride(0)
    h.close()
