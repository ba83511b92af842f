#!/usr/bin/env python3
"""Benchmark of the L-GreCo hot path on one MI355X.

One "step" = one pass of the whole path over one batch of synthetic gradients:
    lgreco_profile (every candidate) -> lgreco_emax -> lgreco_solve -> lgreco_payload_layout
    -> lgreco_compress (chosen per-layer setting, error feedback updated),
by default through lgreco_profile_solve_compress, which is those calls in one (--calls two / four
go through the separate entry points; same kernels, same results).
Inputs are resident in HBM before the timed region.  Every step works on its own copy of the
error-feedback buffer, so all steps do identical work and nothing is restored inside the
timed region.

Prints ONE JSON line (metric = gradient GB/s = 4 * N bytes / step time), with
  "roofline"     achieved algorithmic GB/s of the dominant kernel, timed with HIP events on the
                 launch stream inside the timed region (the kernels of every --time-every-th step
                 carry the events; the library sums them, the loop never stops to read them),
                 against the 8 TB/s HBM peak;
  "cpu_baseline" the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP32_MFMA_PEAK_TFLOPS = 157.3

# HBM bytes per launch (read + write) of the dominant kernels, from the rocprofv3 FETCH_SIZE /
# WRITE_SIZE runs summarised under profiles/<workload>_kernels_hbm.md (FETCH_SIZE x 2.0 and
# WRITE_SIZE x 1.0, both calibrated on a copy of known size).  Counters cannot be read from inside
# this process, so the figures are carried here and apply to the default synthetic input only.
MEASURED_TRAFFIC_BYTES = {
    "c4_gpt2_medium_mixed": {"compress/topk_collect": 2186.3e6 + 1130.5e6,
                             "profile/quant_profile_topk_collect": 2983.2e6 + 200.3e6,
                             "compress/quant_compress": 656.2e6 + 382.1e6},
    "c3_transformer_lm_lowrank": {"compress/lowrank_ef": 656.6e6 + 268.5e6},
    "c2_resnet50_topk": {"compress/topk_collect": 205.3e6 + 106.7e6, "profile/topk_collect": 205.2e6 + 17.2e6},
    "c1_resnet18_quant": {"profile/quant_profile": 110.3e6, "compress/quant_compress": 93.9e6 + 52.1e6},
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--calls", choices=("one", "two", "four"), default="one",
                    help="one: lgreco_profile_solve_compress; two: lgreco_profile_solve, then layout + "
                         "lgreco_compress; four: lgreco_profile, lgreco_emax, lgreco_solve, then layout + "
                         "lgreco_compress (same results; each return to the caller between the solver and the "
                         "compression kernels leaves the GPU idle for some tens of microseconds)")
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c4_gpt2_medium_mixed")
    ap.add_argument("--power-iters", type=int, default=1,
                    help="power-iteration steps of the low-rank family (the configs use 1)")
    ap.add_argument("--sample-every-call", action="store_true",
                    help="Top-K: sample the data in every call instead of starting from the previous "
                         "call's thresholds (reuse_thresholds = 0)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="leave out the HIP-event brackets around kernel sections (no roofline in the output)")
    ap.add_argument("--time-every", type=int, default=4,
                    help="kernels carry HIP events in every n-th step only (a timed kernel leaves ~5 us of the "
                         "stream idle on either side: ~45 us per step on the largest workload when every step is timed)")
    ap.add_argument("--detail", action="store_true",
                    help="bracket every kernel section, not only the main kernels (costs ~3 %% of the step)")
    ap.add_argument("--cpu-sample-elems", type=int, default=30_000_000)
    return ap.parse_args()


def cpu_baseline(w, sample_tensors, power_iters=1):
    """Oracle (as it stands) on a bounded sample: same three phases, wall clock."""
    from oracle import pipeline, solver
    from paper_2210_17357_amd import workloads as W
    b = W.generate(w, sample_tensors)
    n = int(b.numels.sum())
    cands = list(w.candidates)
    kw = dict(bucket=w.bucket, stochastic=w.stochastic, seed=w.seed)
    if b.q0 is not None:
        kw.update(q0=b.q0, q_offsets=b.q_offsets, r_max=w.r_max, power_iters=power_iters)
    t0 = time.perf_counter()
    errors = pipeline.profile(b.grads, b.ef, b.offsets, b.numels, b.rows, b.cols, cands, **kw)
    sizes = pipeline.sizes_table(b.numels, b.rows, b.cols, cands, w.bucket)
    t1 = time.perf_counter()
    e_max = solver.e_max_uniform(errors, w.default)
    choice, _, _ = solver.solve(errors, sizes, e_max, w.n_bins)
    t2 = time.perf_counter()
    for l in range(len(b.numels)):
        q0l = None
        if b.q0 is not None:
            q0l = b.q0[int(b.q_offsets[l]):int(b.q_offsets[l]) + int(b.cols[l]) * w.r_max].reshape(-1, w.r_max)
        pipeline.compress_layer(b.grads, b.ef, int(b.offsets[l]), int(b.numels[l]), int(b.rows[l]),
                                int(b.cols[l]), cands[choice[l]], l, w.bucket, w.stochastic, w.seed, q0l,
                                power_iters)
    t3 = time.perf_counter()
    return b, errors, choice, {"profile_s": t1 - t0, "solve_s": t2 - t1, "compress_s": t3 - t2,
                               "elems": n, "total_s": t3 - t0}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2210_17357_amd import binding as B
    from paper_2210_17357_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    w = W.workload(args.workload)
    cands = list(w.candidates)
    threads = min(16, os.cpu_count() or 1)
    t_gen = time.perf_counter()
    batch = W.generate(w, threads=threads)
    t_gen = time.perf_counter() - t_gen
    N = int(batch.numels.sum())
    L = len(batch.numels)
    layers = B.layer_table(batch.offsets, batch.numels, batch.rows, batch.cols)
    ctab = B.cand_table(cands)
    dev = torch.device("cuda:0")
    g = torch.from_numpy(batch.grads).to(dev)
    has_ef = batch.ef is not None
    ef0 = torch.from_numpy(batch.ef).to(dev) if has_ef else torch.zeros_like(g)
    q0 = torch.from_numpy(batch.q0).to(dev) if batch.q0 is not None else None
    n_runs = args.steps + args.warmup
    ef_pool = [ef0.clone() for _ in range(n_runs)]
    q_pool = [q0.clone() for _ in range(n_runs)] if q0 is not None else [None] * n_runs
    h = B.Handle(int(batch.grads.size), L, len(cands), bucket=w.bucket, stochastic=w.stochastic,
                 seed=w.seed, r_max=w.r_max, power_iters=args.power_iters,
                 reuse_thresholds=not args.sample_every_call)
    # The one-call form hands one error-feedback buffer to profile and compression; a workload whose
    # profile runs without one (NULL, half the read traffic) keeps the two-call form.
    calls = "two" if (args.calls == "one" and not has_ef) else args.calls
    level = 0 if args.no_kernel_timing else (2 if args.detail else 1)
    h.set_timing(level)
    h.set_timing_stride(max(1, args.time_every))
    sizes_tab = B.sizes(layers, ctab, w.bucket)
    payload = torch.empty(int(sizes_tab.max(axis=1).sum()) + 16 * (L + 1), dtype=torch.uint8, device=dev)

    kern = {}          # name -> [total ms, calls]
    phase = {"profile": 0.0, "solve": 0.0, "compress": 0.0}
    last = {}

    stream = torch.cuda.current_stream().cuda_stream      # the stream every call of the run is given

    timing = not args.no_kernel_timing

    def step(i, record):
        ef = ef_pool[i]
        t0 = time.perf_counter()
        if calls == "one":
            # the whole path as one call: nothing runs in the caller between the solver's result
            # and the compression kernels
            st, errors, sizes, e_max, choice, tsize, terr, offsets = h.profile_solve_compress(
                g, ef, layers, ctab, w.default, w.n_bins, payload, q_pool[i], stream=stream)
            t1 = t2 = t3 = time.perf_counter()
        else:
            if calls == "four":
                errors, sizes = h.profile(g, ef if has_ef else None, layers, ctab, q0, want_sizes=True, stream=stream)
                t1 = time.perf_counter()
                e_max = B.emax(errors, w.default)
                st, choice, tsize, terr = h.solve(errors, sizes, e_max, w.n_bins, stream=stream)
            else:
                # profile, E_max and solve as one call: no host round trip between their kernels
                st, errors, sizes, e_max, choice, tsize, terr = h.profile_solve(
                    g, ef if has_ef else None, layers, ctab, w.default, w.n_bins, q0, stream=stream)
                t1 = time.perf_counter()
            t2 = time.perf_counter()
            offsets = B.payload_layout(layers, ctab, choice, w.bucket)
            h.compress(g, ef, layers, ctab, choice, payload, offsets, q_pool[i], stream=stream)
            t3 = time.perf_counter()
        if record:
            # host clocks: compress only queues its kernels, their GPU time falls into the wait of
            # the next step's profile call (or the final synchronize); with --calls two "profile"
            # covers profile + solve, with --calls one everything
            phase["profile"] += t1 - t0
            phase["solve"] += t2 - t1
            phase["compress"] += t3 - t2
        last.update(errors=errors, sizes=sizes, choice=choice, e_max=e_max, tsize=tsize, terr=terr, st=st)

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    h.set_timing(level)          # clears the library's per-section totals: the warm-up does not count
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    # Kernel times: the library keeps the events of every call (the main kernels' events ride on
    # the launches themselves) and sums them per section while it waits for the GPU anyway; the
    # loop above never asks for them, the totals over the timed steps are read here.
    if timing:
        for prefix, call in (("profile/", B.CALL_PROFILE), ("solve/", B.CALL_SOLVE), ("compress/", B.CALL_COMPRESS)):
            for name, total_ms, cnt in h.get_timing_totals(call):
                kern[prefix + name] = [total_ms, cnt]
    ms_per_step = elapsed * 1e3 / args.steps
    value = 4.0 * N / (elapsed / args.steps) / 1e9

    choice = last["choice"]
    fam = np.array([cands[c][0] for c in choice])
    par = np.array([cands[c][1] for c in choice])
    numels = batch.numels.astype(np.float64)
    nq = float(numels[fam == W.QUANT].sum())
    ntk = float(numels[fam == W.TOPK].sum())
    mean_bits = float((numels * par)[fam == W.QUANT].sum() / nq) if nq else 0.0
    mean_dens = float((numels * par)[fam == W.TOPK].sum() / ntk) if ntk else 0.0
    # algorithmic bytes per element and elements covered per launch, per timed section:
    # streaming reads of g (and e when there is one) = rd bytes per element in the profile; compress reads g and e and writes e
    rd = 8.0 if has_ef else 4.0
    algo, elems = {}, {}
    for k in ("quant_profile", "quant_profile_topk_collect", "topk_collect"):
        algo["profile/" + k], elems["profile/" + k] = rd, float(N)
    algo["compress/quant_compress"] = 12.0 + mean_bits / 8.0 + 8.0 / 128.0
    elems["compress/quant_compress"] = nq
    algo["compress/topk_collect"], elems["compress/topk_collect"] = 12.0, ntk
    nlr = float(numels[fam == W.LOWRANK].sum())
    algo["compress/lowrank_ef"], elems["compress/lowrank_ef"] = 12.0, nlr
    # dense contractions of the low-rank path: flops per launch (64 columns are computed per layer)
    flops = {}
    mn2d = float(sum(int(r) * int(c) for r, c in zip(batch.rows, batch.cols)))
    if any(f == W.LOWRANK for f, _ in cands):
        for k in ("lowrank_gemm_p", "lowrank_gemm_q"):
            flops["profile/" + k] = 2.0 * mn2d * 64
            flops["compress/" + k] = 2.0 * float(sum(int(r) * int(c) for r, c, f_ in
                                                     zip(batch.rows, batch.cols, fam) if f_ == W.LOWRANK)) * 64
    kernels = {}
    for name, (ms, cnt) in kern.items():
        avg = ms / max(cnt, 1)
        entry = {"avg_ms": round(avg, 4), "launches": cnt}
        if name in algo and avg > 0 and elems[name] > 0:
            gb = algo[name] * elems[name] / 1e9
            entry["algo_GB"] = round(gb, 4)
            entry["GBps"] = round(gb / (avg * 1e-3), 1)
        if name in flops and avg > 0 and flops[name] > 0:
            entry["TFLOPs"] = round(flops[name] / (avg * 1e-3) / 1e12, 2)
        kernels[name] = entry
    timed = {k: v for k, v in kernels.items() if "GBps" in v or "TFLOPs" in v}
    roofline = None
    if timed:
        dom = max(timed, key=lambda k: timed[k]["avg_ms"])
        if "TFLOPs" in timed[dom]:
            ach = timed[dom]["TFLOPs"]
            roofline = {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": FP32_MFMA_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(ach / FP32_MFMA_PEAK_TFLOPS, 4), "traffic": None,
                        "avg_ms": timed[dom]["avg_ms"]}
        else:
            ach = timed[dom]["GBps"]
            roofline = {"bound": "hbm", "kernel": dom, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(ach / HBM_PEAK_GBS, 4),
                        "traffic": MEASURED_TRAFFIC_BYTES.get(w.name, {}).get(dom),
                        "algorithmic_bytes": round(algo[dom] * elems[dom]),
                        "avg_ms": timed[dom]["avg_ms"], "algo_bytes_per_elem": round(algo[dom], 4)}
    out = {
        "metric": "profile+solve+compress gradient GB/s at 1 MI355X",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "elements": N, "layers": L, "candidates": len(cands),
                   "n_bins": w.n_bins, "stochastic": bool(w.stochastic), "power_iters": args.power_iters,
                   "reuse_thresholds": not args.sample_every_call,
                   "calls_per_step": calls,
                   "kernels_timed_every_n_steps": None if args.no_kernel_timing else max(1, args.time_every),
                   "host_generation_s": round(t_gen, 2)},
        "roofline": roofline,
        # host wall clock per call; compress returns with its kernels queued, so most of its GPU
        # time shows up under the next step's profile
        "phases_ms": ({"profile_solve_compress": round(phase["profile"] * 1e3 / args.steps, 4)} if calls == "one"
                      else {k: round(v * 1e3 / args.steps, 4) for k, v in phase.items()}),
        "kernels": kernels,
        "result": {"status": int(last["st"]), "total_size_bytes": int(last["tsize"]),
                   "ratio_vs_fp32": round(4.0 * N / max(int(last["tsize"]), 1), 3),
                   "uniform_default_bytes": int(last["sizes"][:, w.default].sum()),
                   "total_error_over_emax": round(float(last["terr"]) / float(last["e_max"]), 5)
                   if last["e_max"] > 0 else None,
                   "layers_quant": int((fam == W.QUANT).sum()), "layers_topk": int((fam == W.TOPK).sum()),
                   "layers_lowrank": int((fam == W.LOWRANK).sum())},
    }

    # receiver side (not part of the step): the last step's payloads back to a dense buffer
    out_buf = torch.empty_like(g)
    offsets = B.payload_layout(layers, ctab, choice, w.bucket)
    h.set_timing(0)
    for _ in range(2):
        h.decompress(payload, offsets, layers, ctab, choice, out_buf, accumulate=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        h.decompress(payload, offsets, layers, ctab, choice, out_buf, accumulate=True)
    torch.cuda.synchronize()
    dec_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    out["decompress"] = {"ms": round(dec_ms, 4), "GBps_dense_output": round(4.0 * N / dec_ms / 1e6, 1),
                         "mode": "accumulate", "payload_bytes": int(last["tsize"])}

    if not args.no_cpu_baseline:
        # bounded sample: leading tensors of the workload up to ~cpu-sample-elems elements,
        # skipping any single tensor larger than the bound
        sample, acc = [], 0
        for t, shape in enumerate(w.shapes):
            n = int(np.prod(shape))
            if n > args.cpu_sample_elems:
                continue
            if acc + n > args.cpu_sample_elems:
                break
            sample.append(t)
            acc += n
        sb, o_err, o_choice, tm = cpu_baseline(w, sample, args.power_iters)
        out["cpu_baseline"] = {
            "value": round(4.0 * tm["elems"] / tm["total_s"] / 1e9, 4), "unit": "GB/s", "cores": 1,
            "kind": "oracle",
            "sample": "tensors %d..%d of %s (%d elements): oracle profile %.2fs + solve %.2fs + compress %.2fs; "
                      "numpy element-wise code, single thread (host has %d cores)"
                      % (sample[0], sample[-1], w.name, tm["elems"], tm["profile_s"], tm["solve_s"],
                         tm["compress_s"], os.cpu_count() or 0)}
        # parity of the GPU profile on the sampled layers (same seeded inputs)
        idx = [int(np.where(batch.tensor_index == t)[0][0]) for t in sb.tensor_index]
        if not w.stochastic or idx == list(range(len(idx))):     # the RNG is keyed by layer index
            g_err = last["errors"][idx]
            rel = np.abs(g_err - o_err) / np.maximum(np.abs(o_err), 1e-300)
            out["parity"] = {"layers_checked": len(idx), "max_rel_err_profile": float(rel.max())}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
