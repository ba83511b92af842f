"""GPU: argument checking of the C ABI (every rejected call must return an error code, never
launch a kernel on bad shapes) and a layer near the largest supported size (2^31 - 1 elements per
layer: indices travel as 31 bits plus the sign), checked through properties that hold at any size."""
import numpy as np
import pytest

from paper_2210_17357_amd import workloads as W

from gpu_util import torch_cuda

pytestmark = pytest.mark.gpu


def test_rejected_arguments():
    from paper_2210_17357_amd import binding as B
    torch = torch_cuda()
    n = 4096
    g = torch.randn(n + 8, device="cuda")
    e = torch.zeros(n + 8, device="cuda")
    payload = torch.zeros(8 * n, dtype=torch.uint8, device="cuda")
    cands = B.cand_table([(W.QUANT, 4.0), (W.TOPK, 0.1)])
    ok_layers = B.layer_table([0, 2048], [2048, 2048], [0, 0], [0, 0])
    h = B.Handle(n, 2, 2)

    def err(fn, *a, **k):
        with pytest.raises(B.LgrecoError) as ei:
            fn(*a, **k)
        return ei.value.status

    # layer tables: empty layer, negative offset, overlap, rows*cols != numel, too many layers / elements
    for bad in (B.layer_table([0], [0], [0], [0]), B.layer_table([-4], [16], [0], [0]),
                B.layer_table([0, 1000], [2048, 100], [0, 0], [0, 0]), B.layer_table([0], [100], [10], [11])):
        assert err(h.profile, g, e, bad, cands) == B.EINVAL
    assert err(h.profile, g, e, B.layer_table([0, 8, 16], [8, 8, 8], [0] * 3, [0] * 3), cands) == B.ENOSPACE
    assert err(h.profile, g, e, B.layer_table([0], [n + 8], [0], [0]), cands) == B.ENOSPACE
    # candidates: bits out of range / fractional, density out of range, rank on a 1-D layer, unknown family
    for bad in ([(W.QUANT, 0.0)], [(W.QUANT, 9.0)], [(W.QUANT, 2.5)], [(W.TOPK, 0.0)], [(W.TOPK, 1.5)], [(5, 1.0)]):
        assert err(h.profile, g, e, ok_layers, B.cand_table(bad)) == B.EINVAL
    assert err(h.profile, g, e, ok_layers, B.cand_table([(W.LOWRANK, 4.0)]), g) == B.EINVAL
    assert err(h.profile, g, e, ok_layers, B.cand_table([(W.LOWRANK, 4.0)])) == B.EINVAL       # no warm start
    # unaligned device pointers
    assert err(h.profile, g[1:], e, ok_layers, cands) == B.EINVAL
    choice = np.zeros(2, np.int32)
    offsets = B.payload_layout(ok_layers, cands, choice)
    assert err(h.compress, g, e, ok_layers, cands, np.array([0, 7], np.int32), payload, offsets) == B.EINVAL
    assert err(h.compress, g, e, ok_layers, cands, choice, payload, offsets + 4) == B.EINVAL   # unaligned payload
    assert err(h.decompress, payload, offsets, ok_layers, cands, np.array([2, 0], np.int32), g) == B.EINVAL
    # configuration limits
    for kw in (dict(bucket=64), dict(power_iters=0), dict(power_iters=17), dict(r_max=65)):
        with pytest.raises(B.LgrecoError) as ei:
            B.Handle(n, 2, 2, **kw)
        assert ei.value.status == B.EUNSUPPORTED
    with pytest.raises(B.LgrecoError):
        B.Handle(n, 2, 129)
    # after all the rejections the handle still works
    errors, sizes = h.profile(g, e, ok_layers, cands)
    assert errors.shape == (2, 2) and (errors > 0).all()
    h.close()


def test_layer_of_more_than_2_pow_30_elements():
    from paper_2210_17357_amd import binding as B
    torch = torch_cuda()
    n = (1 << 30) + 12345                       # ragged: a slow tail tile and a partial last bucket
    gen = torch.Generator(device="cuda").manual_seed(1)
    g = torch.empty(n, device="cuda").normal_(0, 1e-3, generator=gen)
    g[::1000003] *= 50.0                        # a sprinkle of large entries
    e = torch.empty(n, device="cuda").normal_(0, 1e-4, generator=gen)
    cands_l = [(W.QUANT, 2.0), (W.QUANT, 4.0), (W.QUANT, 8.0), (W.TOPK, 0.001), (W.TOPK, 0.01), (W.TOPK, 0.1)]
    cands = B.cand_table(cands_l)
    layers = B.layer_table([0], [n], [0], [0])
    h = B.Handle(n, 1, len(cands_l))
    errors, sizes = h.profile(g, e, layers, cands)
    x = g + e
    total = float(x.double().pow(2).sum())
    assert (np.diff(errors[0, :3]) < 0).all() and (np.diff(errors[0, 3:]) < 0).all()
    assert 0 < errors[0, 5] < errors[0, 3] < total
    nb = (n + 127) // 128
    assert sizes[0, 1] == 8 * nb + (n // 128) * 64 + ((n % 128) * 4 + 7) // 8
    assert sizes[0, 4] == 8 * int(np.floor(0.01 * n + 0.5))
    for c in (1, 4):                                                   # 4 bits, density 1 %
        choice = np.array([c], np.int32)
        offsets = B.payload_layout(layers, cands, choice)
        payload = torch.zeros(int(offsets[-1]) + 16, dtype=torch.uint8, device="cuda")
        ef = e.clone()
        h.compress(g, ef, layers, cands, choice, payload, offsets)
        left = float(ef.double().pow(2).sum())
        assert abs(left - errors[0, c]) <= 1e-4 * errors[0, c]          # what is left = what was profiled
        out = torch.empty_like(g)
        h.decompress(payload, offsets, layers, cands, choice, out, accumulate=False)
        # image + new error feedback gives x back (exactly for Top-K, to one rounding for quantization)
        diff = (out + ef - x).abs().max().item()
        assert diff <= (0.0 if c == 4 else float(x.abs().max()) * 2.0 ** -22)
        if c == 4:
            k = int(np.floor(0.01 * n + 0.5))
            idx = payload[int(offsets[0]) + 4 * k:int(offsets[0]) + 8 * k].view(torch.int32)
            assert int((out != 0).sum()) == k and bool((idx[1:] > idx[:-1]).all()) and int(idx[-1]) < n
            kept_min = float(out[out != 0].abs().min())
            assert float((ef.abs() > kept_min).sum()) == 0              # nothing larger was dropped
        del payload, ef, out
    h.close()
