#!/usr/bin/env python3
"""Benchmark of the L-GreCo hot path on one MI355X.

One "step" = one pass of the whole path over one batch of synthetic gradients:
    lgreco_profile (every candidate) -> lgreco_emax -> lgreco_solve -> lgreco_payload_layout
    -> lgreco_compress (chosen per-layer setting, error feedback updated),
by default through lgreco_profile_solve_compress, which is those calls in one (--calls two / four
go through the separate entry points; same kernels, same results).
Inputs are resident in HBM before the timed region.  The data MOVES from step to step as in a
training loop: the steps rotate over --grad-buffers independent draws of the workload (same
per-layer scales, fresh values and error feedback, each scaled by 1, 1.03, 0.97, ...), so the Top-K
thresholds a call remembers from the previous one are never exactly right.  Every step works on
its own copy of the error-feedback buffer, so nothing is restored inside the timed region.

Prints ONE JSON line (metric = gradient GB/s = 4 * N bytes / step time), with
  "roofline"        achieved algorithmic GB/s of the dominant kernel, timed with HIP events on the
                    launch stream inside the timed region (the kernels of every --time-every-th step
                    carry the events; the library sums them, the loop never stops to read them),
                    against the 8 TB/s HBM peak;
  "phases_gpu_ms"   GPU time of the profile, solve and compress phases (events around everything a
                    phase queues: main kernels, the Top-K chains, list building, the DP);
  "roofline_phase"  algorithmic bytes of a phase (and of the whole step) / its time / 8 TB/s;
  "cold"            the same loop with reuse_thresholds = 0 (every call samples the data first);
  "other_workloads" the smaller workloads of the benchmark spec, same measurement, a few ms each;
  "cpu_baseline"    the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import dataclasses
import gc
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP32_MFMA_PEAK_TFLOPS = 157.3
DEFAULT_WORKLOAD = "c4_gpt2_medium_mixed"
OTHER_WORKLOADS = ("c1_resnet18_quant", "c2_resnet50_topk", "c3_transformer_lm_lowrank")
DRIFT = (1.0, 1.03, 0.97, 1.015, 0.985)      # scale of gradient buffer v (and of its error feedback)
# timed sections of the library that get a roofline figure (streaming kernels in bytes, contractions in flops)
STREAMING_SECTIONS = ("profile/quant_profile", "profile/quant_profile_topk_collect", "profile/topk_collect",
                      "compress/quant_compress", "compress/topk_collect", "compress/lowrank_ef")
CONTRACTION_SECTIONS = ("profile/lowrank_gemm_p", "profile/lowrank_gemm_q", "compress/lowrank_gemm_p",
                        "compress/lowrank_gemm_q")


def measured_traffic(workload: str) -> dict:
    """HBM bytes per launch (read + write) per timed section, from the rocprofv3 FETCH_SIZE /
    WRITE_SIZE summary under profiles/ (counters cannot be read from inside this process).  The
    summary's table carries the bench section of every kernel in its last column."""
    path = os.path.join(ROOT, "profiles", workload + "_kernels_hbm.md")
    out = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) < 9 or not re.match(r"^(profile|compress)/", cells[-1]):
            continue
        try:
            out[cells[-1]] = (float(cells[-3]) + float(cells[-2])) * 1e6
        except ValueError:
            pass
    return out


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
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--grad-buffers", type=int, default=3,
                    help="independent draws of the workload the steps rotate over (1: the same data every step)")
    ap.add_argument("--power-iters", type=int, default=1,
                    help="power-iteration steps of the low-rank family (the configs use 1)")
    ap.add_argument("--sample-every-call", action="store_true",
                    help="Top-K: the main loop itself runs with reuse_thresholds = 0 (the default run reports "
                         "that case under \"cold\")")
    ap.add_argument("--no-cold", action="store_true", help="leave out the reuse_thresholds = 0 loop")
    ap.add_argument("--dp-groups", type=int, default=0,
                    help="layer groups of the solver: 0 = the library decides from the table's size, 1 = one "
                         "sequential sweep, 2 / 4 / 8 = that many groups")
    ap.add_argument("--keep-ef-on-failure", action="store_true",
                    help="create the handle with keep_ef_on_failure = 1: the profile of the one call does not "
                         "leave x in the error-feedback buffer (more memory traffic, same results)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="leave out the smaller workloads (they run only next to the default workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="leave out the HIP-event brackets around kernel sections (no roofline in the output)")
    ap.add_argument("--time-every", type=int, default=4,
                    help="kernels carry HIP events in every n-th step only (a timed kernel leaves ~5 us of the "
                         "stream idle on either side: ~45 us per step on the largest workload when every step is timed)")
    ap.add_argument("--detail", action="store_true",
                    help="bracket every kernel section, not only the main kernels (costs ~3 %% of the step)")
    ap.add_argument("--cpu-sample-elems", type=int, default=66_000_000)
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


def measure(wname, args, steps, warmup, with_cold, with_decompress):
    """The timed loop on one workload.  Returns (result dict, context for the CPU baseline)."""
    import torch
    from paper_2210_17357_amd import binding as B
    from paper_2210_17357_amd import workloads as W

    w = W.workload(wname)
    cands = list(w.candidates)
    threads = min(16, os.cpu_count() or 1)
    n_buf = max(1, min(args.grad_buffers, len(DRIFT)))
    dev = torch.device("cuda:0")
    t_gen = time.perf_counter()
    batch = None
    g_list, ef0_list = [], []
    for v in range(n_buf):
        b = W.generate(dataclasses.replace(w, variant=v), threads=threads)
        if v == 0:
            batch = b
        g_list.append(torch.from_numpy(b.grads).to(dev).mul_(DRIFT[v]))
        ef0_list.append(torch.from_numpy(b.ef).to(dev).mul_(DRIFT[v]) if b.ef is not None else None)
        if v > 0:
            del b
    t_gen = time.perf_counter() - t_gen
    N = int(batch.numels.sum())
    L = len(batch.numels)
    layers = B.layer_table(batch.offsets, batch.numels, batch.rows, batch.cols)
    ctab = B.cand_table(cands)
    has_ef = batch.ef is not None
    q0 = torch.from_numpy(batch.q0).to(dev) if batch.q0 is not None else None
    n_runs = steps + warmup
    zeros = None if has_ef else torch.zeros_like(g_list[0])

    def fresh_ef(i):
        return ef0_list[i % n_buf].clone() if has_ef else zeros.clone()
    # The one-call form hands one error-feedback buffer to profile and compression: a workload that
    # states none gets a cleared buffer every step (x = g + 0, as in the first step of a training
    # run) and the handle is told so (lgreco_set_ef_zero_on_entry): the profile does not read it,
    # the compression reads and fills it.
    calls = args.calls
    level = 0 if args.no_kernel_timing else (2 if args.detail else 1)
    sizes_tab = B.sizes(layers, ctab, w.bucket)
    payload = torch.empty(int(sizes_tab.max(axis=1).sum()) + 16 * (L + 1), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream      # the stream every call of the run is given
    has_topk = any(f == W.TOPK for f, _ in cands)

    def loop(reuse, timing_level):
        """warm-up + timed steps on a handle of its own; returns (elapsed s, kernel totals, last results)."""
        h = B.Handle(int(batch.grads.size), L, len(cands), bucket=w.bucket, stochastic=w.stochastic,
                     seed=w.seed, r_max=w.r_max, power_iters=args.power_iters, reuse_thresholds=reuse,
                     keep_ef_on_failure=args.keep_ef_on_failure, dp_groups=args.dp_groups)
        h.set_timing(timing_level)
        h.set_timing_stride(max(1, args.time_every))
        if not has_ef:
            h.set_ef_zero_on_entry(True)
        ef_pool = [fresh_ef(i) for i in range(n_runs)]
        q_pool = [q0.clone() for _ in range(n_runs)] if q0 is not None else [None] * n_runs
        last = {}

        def step(i):
            g, ef = g_list[i % n_buf], ef_pool[i]
            if calls == "one":
                st, errors, sizes, e_max, choice, tsize, terr, offsets = h.profile_solve_compress(
                    g, ef, layers, ctab, w.default, w.n_bins, payload, q_pool[i], stream=stream)
            else:
                if calls == "four":
                    errors, sizes = h.profile(g, ef if has_ef else None, layers, ctab, q0, want_sizes=True,
                                              stream=stream)
                    e_max = B.emax(errors, w.default)
                    st, choice, tsize, terr = h.solve(errors, sizes, e_max, w.n_bins, stream=stream)
                else:
                    st, errors, sizes, e_max, choice, tsize, terr = h.profile_solve(
                        g, ef if has_ef else None, layers, ctab, w.default, w.n_bins, q0, stream=stream)
                offsets = B.payload_layout(layers, ctab, choice, w.bucket)
                h.compress(g, ef, layers, ctab, choice, payload, offsets, q_pool[i], stream=stream)
            last.update(errors=errors, sizes=sizes, choice=choice, e_max=e_max, tsize=tsize, terr=terr, st=st,
                        buffer=i % n_buf)

        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        h.set_timing(timing_level)   # clears the library's per-section totals: the warm-up does not count
        t_start = time.perf_counter()
        for i in range(steps):
            step(warmup + i)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start
        # Kernel times: the library keeps the events of every timed call and sums them per section
        # while it waits for the GPU anyway; the loop above never asks for them.
        kern = {}
        if timing_level:
            for prefix, call in (("profile/", B.CALL_PROFILE), ("solve/", B.CALL_SOLVE),
                                 ("compress/", B.CALL_COMPRESS)):
                for name, total_ms, cnt in h.get_timing_totals(call):
                    kern[prefix + name] = [total_ms, cnt]
        del ef_pool, q_pool
        return h, elapsed, kern, last

    h, elapsed, kern, last = loop(not args.sample_every_call, level)
    ms_per_step = elapsed * 1e3 / steps
    value = 4.0 * N / (elapsed / steps) / 1e9

    choice = last["choice"]
    fam = np.array([cands[c][0] for c in choice])
    par = np.array([cands[c][1] for c in choice])
    numels = batch.numels.astype(np.float64)
    nq = float(numels[fam == W.QUANT].sum())
    ntk = float(numels[fam == W.TOPK].sum())
    nlr = float(numels[fam == W.LOWRANK].sum())
    mean_bits = float((numels * par)[fam == W.QUANT].sum() / nq) if nq else 0.0
    chosen_bytes = last["sizes"][np.arange(L), choice].astype(np.float64)
    # algorithmic bytes per element and elements covered per launch, per timed section.  The
    # profile reads g (and e when there is one); the compression reads g and e and writes e.  In
    # the one call over quantization / Top-K candidates the profile also WRITES x = g + e into the
    # error-feedback buffer (12 bytes per element) and the compression reads x there, 4 bytes per
    # element and 4 for the new error feedback, for a quantized layer; a Top-K layer's kept entries come from the candidates the
    # profile recorded (8 bytes per candidate written there and read here: some 13 % of the
    # elements, data dependent and not priced on either side), so nothing per element.
    lowrank = any(f == W.LOWRANK for f, _ in cands)
    in_place = calls == "one" and has_ef and not lowrank and not args.keep_ef_on_failure
    rd = (12.0 if in_place else 8.0) if has_ef else 4.0
    cq, ct = (8.0, 0.0) if in_place else (12.0, 12.0)
    algo, elems = {}, {}
    for k in ("quant_profile", "quant_profile_topk_collect", "topk_collect"):
        algo["profile/" + k], elems["profile/" + k] = rd, float(N)
    algo["compress/quant_compress"] = cq + mean_bits / 8.0 + 8.0 / 128.0
    elems["compress/quant_compress"] = nq
    algo["compress/topk_collect"], elems["compress/topk_collect"] = ct, ntk
    # (with the promise of a zero buffer the one call's low-rank update reads g and writes e' only)
    lr_ef_bytes = 8.0 if (calls == "one" and not has_ef) else 12.0
    algo["compress/lowrank_ef"], elems["compress/lowrank_ef"] = lr_ef_bytes, nlr
    # dense contractions of the low-rank path: flops per launch
    flops = {}
    mn2d = float(sum(int(r) * int(c) for r, c in zip(batch.rows, batch.cols)))
    if lowrank:
        for k in ("lowrank_gemm_p", "lowrank_gemm_q"):
            flops["profile/" + k] = 2.0 * mn2d * w.r_max
            # the compression contracts as many columns as the largest chosen rank rounded up to 32
            flops["compress/" + k] = 2.0 * float(sum(int(r) * int(c) * p for r, c, f_, p in
                                                     zip(batch.rows, batch.cols, fam, par) if f_ == W.LOWRANK))
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
                        "traffic": measured_traffic(w.name).get(dom),
                        "algorithmic_bytes": round(algo[dom] * elems[dom]),
                        "avg_ms": timed[dom]["avg_ms"], "algo_bytes_per_elem": round(algo[dom], 4)}
            if in_place and dom.startswith("profile/"):
                # what the per-element figure stands for, since it is not the profile-only 8 bytes
                roofline["note"] = ("the one call's profile pass reads g and e (8 B) and stores x = g + e into the "
                                    "error-feedback buffer (4 B), which the compression then reads instead of g and e; "
                                    "the candidate records it also writes (6 B per candidate) are not counted")

    # per phase: GPU time between the first and the last thing the phase queues, and what the phase
    # must move (profile: one read of g and e for every candidate; compress: read g, e, write e and
    # the payload; low rank: the matrix twice for the factors, read and write for the error feedback)
    phase_ms = {}
    for key, name in (("profile", "profile/phase_profile"), ("solve", "solve/dp_solve"),
                      ("compress", "compress/phase_compress")):
        if name in kern and kern[name][1] > 0:
            phase_ms[key] = kern[name][0] / kern[name][1]
    profile_bytes = rd * N * (2.0 * args.power_iters if lowrank else 1.0)
    compress_bytes = (float(((cq * numels + chosen_bytes)[fam == W.QUANT]).sum())
                      + float(((ct * numels + chosen_bytes)[fam == W.TOPK]).sum())
                      # low rank: the one call reuses the profile's factors (only the update of the error
                      # feedback moves data); the separate compression contracts the matrix again
                      + float(((lr_ef_bytes + (0.0 if calls == "one" else 8.0 * args.power_iters)) * numels
                               + chosen_bytes)[fam == W.LOWRANK].sum()))
    roofline_phase = {}
    for key, nbytes in (("profile", profile_bytes), ("compress", compress_bytes)):
        if key in phase_ms and phase_ms[key] > 0:
            gbps = nbytes / (phase_ms[key] * 1e-3) / 1e9
            roofline_phase[key] = {"algorithmic_bytes": round(nbytes), "ms": round(phase_ms[key], 4),
                                   "GBps": round(gbps, 1), "frac": round(gbps / HBM_PEAK_GBS, 4)}
    step_gbps = (profile_bytes + compress_bytes) / (ms_per_step * 1e-3) / 1e9
    roofline_phase["step"] = {"algorithmic_bytes": round(profile_bytes + compress_bytes), "ms": round(ms_per_step, 4),
                              "GBps": round(step_gbps, 1), "frac": round(step_gbps / HBM_PEAK_GBS, 4)}
    if in_place:
        # The step also against what the path moves when profile and compression each read g and e
        # (8 bytes per element, then 12 and the payload: the accounting of the separate calls): a
        # step that avoids bytes should not look worse for it.
        two_pass = 8.0 * N + float((12.0 * numels + chosen_bytes).sum())
        roofline_phase["step"].update(two_pass_bytes=round(two_pass),
                                      two_pass_frac=round(two_pass / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))
    if lowrank:
        # the contraction-bound part: flops of the factor GEMMs over the time of the whole phase
        for key, fl in (("profile", 4.0 * mn2d * w.r_max * args.power_iters),
                        ("compress", sum(flops.get("compress/" + k, 0.0) for k in ("lowrank_gemm_p", "lowrank_gemm_q"))
                         * args.power_iters + flops.get("compress/lowrank_gemm_p", 0.0))):
            if key in phase_ms and phase_ms[key] > 0:
                tf = fl / (phase_ms[key] * 1e-3) / 1e12
                roofline_phase[key].update(flops=round(fl), TFLOPs=round(tf, 2),
                                           frac_mfma=round(tf / FP32_MFMA_PEAK_TFLOPS, 4))

    out = {
        "value": round(value, 2), "unit": "GB/s", "ms_per_step": round(ms_per_step, 4),
        "config": {"workload": w.name, "elements": N, "layers": L, "candidates": len(cands),
                   "n_bins": w.n_bins, "stochastic": bool(w.stochastic), "power_iters": args.power_iters,
                   "reuse_thresholds": not args.sample_every_call, "grad_buffers": n_buf,
                   "calls_per_step": calls, "x_in_ef_buffer": bool(in_place),
                   "steps": steps, "warmup": warmup,
                   "kernels_timed_every_n_steps": None if args.no_kernel_timing else max(1, args.time_every),
                   "host_generation_s": round(t_gen, 2)},
        "roofline": roofline,
        "phases_gpu_ms": {k: round(v, 4) for k, v in phase_ms.items()},
        "roofline_phase": roofline_phase,
        "kernels": kernels,
        "result": {"status": int(last["st"]), "total_size_bytes": int(last["tsize"]),
                   "ratio_vs_fp32": round(4.0 * N / max(int(last["tsize"]), 1), 3),
                   "uniform_default_bytes": int(last["sizes"][:, w.default].sum()),
                   "total_error_over_emax": round(float(last["terr"]) / float(last["e_max"]), 5)
                   if last["e_max"] > 0 else None,
                   "layers_quant": int((fam == W.QUANT).sum()), "layers_topk": int((fam == W.TOPK).sum()),
                   "layers_lowrank": int((fam == W.LOWRANK).sum())},
    }

    errors0 = None
    if with_decompress:
        # (for the parity figure of the CPU baseline: the profile of buffer 0, the oracle's input)
        errors0, _ = h.profile(g_list[0], ef0_list[0], layers, ctab, q0, want_sizes=False, stream=stream)
        # receiver side (not part of the step): the last step's payloads back to a dense buffer
        out_buf = torch.empty_like(g_list[0])
        offsets = B.payload_layout(layers, ctab, choice, w.bucket)
        h.set_timing(0)
        for _ in range(2):
            h.decompress(payload, offsets, layers, ctab, choice, out_buf, accumulate=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            h.decompress(payload, offsets, layers, ctab, choice, out_buf, accumulate=True)
        torch.cuda.synchronize()
        dec_ms = (time.perf_counter() - t0) * 1e3 / steps
        out["decompress"] = {"ms": round(dec_ms, 4), "GBps_dense_output": round(4.0 * N / dec_ms / 1e6, 1),
                             "mode": "accumulate", "payload_bytes": int(last["tsize"])}
        del out_buf
    h.close()

    if with_cold and has_topk and not args.sample_every_call:
        # the same loop when no call may start from the previous call's thresholds
        hc, el_c, _, _ = loop(False, 0)
        hc.close()
        out["cold"] = {"reuse_thresholds": False, "ms_per_step": round(el_c * 1e3 / steps, 4),
                       "value": round(4.0 * N / (el_c / steps) / 1e9, 2), "unit": "GB/s"}
    ctx = {"w": w, "batch": batch, "last": last, "errors0": errors0}
    del g_list, ef0_list, payload
    gc.collect()
    torch.cuda.empty_cache()
    return out, ctx


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)

    res, ctx = measure(args.workload, args, args.steps, args.warmup, with_cold=not args.no_cold,
                       with_decompress=True)
    w, batch, last = ctx["w"], ctx["batch"], ctx["last"]
    out = {
        "metric": "profile+solve+compress gradient GB/s at 1 MI355X",
        "value": res["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
    }
    for k in ("config", "roofline", "phases_gpu_ms", "roofline_phase", "cold", "kernels", "result", "decompress"):
        if k in res:
            out[k] = res[k]

    if args.workload == DEFAULT_WORKLOAD and not args.no_other_workloads:
        # the other workloads of the baseline's list (the smallest one is a parity case of a few
        # microseconds): same loop, milliseconds each
        others = {}
        for name in OTHER_WORKLOADS:
            r, _ = measure(name, args, max(args.steps, 20), max(args.warmup, 3), with_cold=not args.no_cold,
                           with_decompress=False)
            others[name] = {k: r[k] for k in ("value", "unit", "ms_per_step", "roofline", "phases_gpu_ms",
                                              "roofline_phase", "cold", "result") if k in r}
            others[name]["elements"] = r["config"]["elements"]
            others[name]["kernels"] = {k: v for k, v in r["kernels"].items() if "GBps" in v or "TFLOPs" in v}
        out["other_workloads"] = others

    if not args.no_cpu_baseline:
        # bounded sample: leading tensors of the workload up to ~cpu-sample-elems elements (the
        # largest tensor first in every workload here, so the sample holds it)
        sample, acc = [], 0
        for t, shape in enumerate(w.shapes):
            n = int(np.prod(shape))
            if acc + n > args.cpu_sample_elems and sample:
                break
            sample.append(t)
            acc += n
        sb, o_err, o_choice, tm = cpu_baseline(w, sample, args.power_iters)
        lowrank_oracle = any(int(f) == 2 for f, _ in w.candidates)        # 2: the low-rank family
        try:
            from threadpoolctl import threadpool_info
            blas_threads = max([int(i.get("num_threads", 1)) for i in threadpool_info()
                                if i.get("user_api") == "blas"] or [1])
        except Exception:
            blas_threads = 1
        out["cpu_baseline"] = {
            "value": round(4.0 * tm["elems"] / tm["total_s"] / 1e9, 4), "unit": "GB/s",
            # threads the oracle's arithmetic runs on: numpy's element-wise code uses one, its matrix
            # products (the low-rank family only) the BLAS library's pool.  (CPU time of the whole
            # process over wall time would also count the runtimes' idle spinning threads.)
            "cores": blas_threads if lowrank_oracle else 1,
            "kind": "oracle",
            "sample": "tensors %d..%d of %s (%d elements, largest tensor %d): oracle profile %.2fs + solve %.3fs + "
                      "compress %.2fs; numpy: element-wise code on one thread, matrix products on %d BLAS "
                      "threads (host has %d cores)"
                      % (sample[0], sample[-1], w.name, tm["elems"], int(sb.numels.max()), tm["profile_s"],
                         tm["solve_s"], tm["compress_s"], blas_threads, os.cpu_count() or 0)}
        # parity of the GPU profile on the sampled layers (gradient buffer 0 is the oracle's input)
        idx = [int(np.where(batch.tensor_index == t)[0][0]) for t in sb.tensor_index]
        if ctx["errors0"] is not None and (not w.stochastic or idx == list(range(len(idx)))):
            g_err = ctx["errors0"][idx]
            rel = np.abs(g_err - o_err) / np.maximum(np.abs(o_err), 1e-300)
            out["parity"] = {"layers_checked": len(idx), "max_rel_err_profile": float(rel.max())}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
