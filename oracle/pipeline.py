"""Oracle: the whole path - profile every (layer, candidate), size table, budget, solve,
compress with the chosen per-layer setting (the periodic L-GreCo run of the paper's
"Implementation" paragraph followed by the per-step compression of its communication
engine).  Plain loops over layers and candidates calling the per-family oracles.
"""
import numpy as np

from . import lowrank, quant, solver, topk

QUANT, TOPK, LOWRANK = 0, 1, 2


def layer_x(grads, ef, offset: int, numel: int) -> np.ndarray:
    g = np.asarray(grads[offset:offset + numel], np.float32)
    return quant.form_x(g, None if ef is None else ef[offset:offset + numel])


def sizes_table(numels, rows, cols, cands, bucket: int = 128) -> np.ndarray:
    out = np.zeros((len(numels), len(cands)), np.int64)
    for l, n in enumerate(numels):
        for p, (fam, par) in enumerate(cands):
            if fam == QUANT:
                out[l, p] = quant.size_bytes(int(n), int(par), bucket)
            elif fam == TOPK:
                out[l, p] = topk.size_bytes(int(n), float(par))
            else:
                out[l, p] = lowrank.size_bytes(int(rows[l]), int(cols[l]), int(par))
    return out


def profile(grads, ef, offsets, numels, rows, cols, cands, bucket: int = 128,
            stochastic: bool = False, seed: int = 0, q0=None, q_offsets=None, r_max: int = 64,
            power_iters: int = 1) -> np.ndarray:
    """errors[L x P] (fp64): squared L2 distance between x = g + e and its
    compress -> decompress image, for every layer and candidate; e is not updated."""
    n_layers = len(numels)
    errors = np.zeros((n_layers, len(cands)), np.float64)
    for l in range(n_layers):
        n = int(numels[l])
        x = layer_x(grads, ef, int(offsets[l]), n)
        u = quant.layer_uniforms(seed, l, n) if stochastic else None
        tk = [(p, topk.k_of(n, par)) for p, (fam, par) in enumerate(cands) if fam == TOPK]
        if tk:
            for (p, _), err in zip(tk, topk.errors_all(x, [k for _, k in tk])):
                errors[l, p] = err
        for p, (fam, par) in enumerate(cands):
            if fam == QUANT:
                errors[l, p] = quant.error(x, int(par), bucket, u)
            elif fam == LOWRANK:
                m = lowrank.matrix_view(x, int(rows[l]), int(cols[l]))
                q = np.asarray(q0[int(q_offsets[l]):int(q_offsets[l]) + int(cols[l]) * r_max])
                errors[l, p] = lowrank.error(m, q.reshape(int(cols[l]), r_max), int(par), power_iters)
    return errors


def compress_layer(grads, ef, offset, numel, rows, cols, cand, layer_index, bucket=128,
                   stochastic=False, seed=0, q0_layer=None, power_iters=1):
    """Returns (payload uint8[], new_ef f32[numel], extra) for one layer and one candidate."""
    fam, par = cand
    g = np.asarray(grads[offset:offset + numel], np.float32)
    e = None if ef is None else np.asarray(ef[offset:offset + numel], np.float32)
    if fam == QUANT:
        u = quant.layer_uniforms(seed, layer_index, numel) if stochastic else None
        payload, new_e, codes, xhat = quant.compress(g, e, int(par), bucket, u)
        return payload, new_e, {"codes": codes, "xhat": xhat}
    if fam == TOPK:
        vals, idx, new_e = topk.compress(g, e, float(par))
        return topk.payload(vals, idx), new_e, {"values": vals, "indices": idx}
    phat, q, new_e = lowrank.compress(g, e, rows, cols, q0_layer, int(par), power_iters)
    payload = np.concatenate([phat.reshape(-1).view(np.uint8), q.reshape(-1).view(np.uint8)])
    return payload, new_e, {"phat": phat, "q": q}


def decompress_layer(payload, numel, rows, cols, cand, bucket=128, out=None):
    """Receiver side of the codec (the step after compression in the paper's pipeline: every
    worker turns the payloads it received back into dense gradients and sums them).  Returns the
    dense fp32 image of one layer's payload, or fl32(out + image) when `out` is given."""
    fam, par = cand
    if fam == QUANT:
        img = quant.unpack(np.asarray(payload, np.uint8), int(numel), int(par), bucket)
    elif fam == TOPK:
        img = topk.decompress(payload, int(numel), topk.k_of(int(numel), float(par)))
    else:
        img = lowrank.decompress(payload, int(rows), int(cols), int(par))
    if out is None:
        return img
    return (np.asarray(out, np.float32) + img).astype(np.float32)


def run(grads, ef, offsets, numels, rows, cols, cands, default, n_bins, **kw):
    """profile -> budget -> solve.  Returns dict with errors, sizes, e_max, choice, totals."""
    errors = profile(grads, ef, offsets, numels, rows, cols, cands, **kw)
    sizes = sizes_table(numels, rows, cols, cands, kw.get("bucket", 128))
    e_max = solver.e_max_uniform(errors, default)
    choice, tsize, terr = solver.solve(errors, sizes, e_max, n_bins)
    return {"errors": errors, "sizes": sizes, "e_max": e_max, "choice": choice,
            "total_size": tsize, "total_error": terr}
