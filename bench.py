#!/usr/bin/env python3
"""Benchmark of the GuidedQuant Fisher-Gram hot path on one MI355X.

A step is one pass of the whole path over one linear layer's calibration batch:
    gq_group_weights(dZ) -> s,  gq_fisher_gram(X, s) -> H (upper triangle),
    gq_fisher_mirror(H),        gq_objective(W, What, H) -> obj
on synthetic tensors of the Llama-2-7B attention-projection shape
(X[65536,4096] bf16, dZ[65536,4096] fp32, G=4), resident in HBM before timing.

Prints ONE JSON line on stdout.  `value` is the algorithmic Gram work of a step,
G*n*d_in*(d_in+1) flop (upper triangle only), divided by the whole step time;
`roofline` is the Gram kernel alone (HIP events around its launches inside the
timed region) against the bf16 dense MFMA peak; `cpu_baseline` is the fp64
oracle timed on the host cores on a bounded token sample of the same layer.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (published, no sparsity)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gram_flops(G, n, d_in):
    return float(G) * n * d_in * (d_in + 1)


def load_traffic(workload):
    """HBM bytes per Gram launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs of
    this script, scaled by a plain copy of known size); the committed summary under profiles/
    holds the figures and the commands.  (None, None) when no measurement is on file."""
    rel = os.path.join("profiles", f"fisher_gram_bf16_{workload}.traffic.json")
    try:
        with open(os.path.join(ROOT, rel)) as f:
            return json.load(f)["hbm_bytes_per_launch"], f"{rel} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command; not measured in this run)"
    except Exception:
        return None, None


def mfma_ceiling():
    """What a loop of nothing but bf16 MFMAs sustains on this GPU (constant and random operands), the shader
    clock it holds meanwhile, and what a plain read stream / copy of 1 GiB sustains, measured by the small
    stand-alone program built next to the library, as a child process."""
    import subprocess
    exe = os.path.join(ROOT, "paper_2505_07004_amd", "mfma_ceiling")
    if not os.path.exists(exe):
        return None
    try:
        out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
        return json.loads(out.stdout.strip().splitlines()[-1])
    except Exception as e:
        log("mfma_ceiling failed:", e)
        return None


def cpu_baseline(spec, X, dZ, W, What, sample_tokens):
    """Time the oracle (numpy fp64, as it stands) on the first `sample_tokens` tokens."""
    import numpy as np
    import oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    Xh = X[:sample_tokens].to("cpu").to(__import__("torch").float64).numpy()
    dZh = dZ[:sample_tokens].to("cpu").numpy()
    Wh, Whh = W.to("cpu").numpy(), What.to("cpu").numpy()
    t0 = time.perf_counter()
    s = oracle.group_weights(dZh, spec.G)
    H = oracle.fisher_gram(Xh, s)
    obj, _ = oracle.objective(Wh, Whh, H, spec.G)
    dt = time.perf_counter() - t0
    fl = gram_flops(spec.G, sample_tokens, spec.d_in)
    return {
        "value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
        "sample": f"first {sample_tokens} of {spec.n} tokens, all {spec.G} groups, whole path "
                  f"(group weights + Gram + objective) in numpy fp64, {dt:.1f} s; "
                  f"rate = algorithmic Gram flop of the sample / that time",
    }, H, obj


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama2_7b_attn")
    ap.add_argument("--cpu-sample-tokens", type=int, default=16384)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB elementwise copy kernel (reference point for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the pure-MFMA ceiling measurement")
    ap.add_argument("--no-xcd-calibration", action="store_true",
                    help="leave the Gram kernel's schedule at its default (equal XCD speeds)")
    ap.add_argument("--cd-cycles", type=int, default=1,
                    help="cycles of the coordinate-descent assignment step timed after the main loop, followed by one "
                         "codebook step (0: skip both)")
    ap.add_argument("--tokens", type=int, default=0, help="override n (debugging only; invalid as a result)")
    ap.add_argument("--groups", type=int, default=0, help="override G (the 13B sweep runs G in 1, 2, 4, 8)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (--gpus 1); the path has no multi-GPU part")

    import torch
    from paper_2505_07004_amd import binding as gq
    from paper_2505_07004_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU: libgq has no CPU path")
    dev = "cuda:0"
    torch.cuda.set_device(0)
    spec = wl.CONFIGS[args.workload]
    if args.tokens:
        spec = wl.scaled(spec, n=args.tokens)
    if args.groups:
        spec = wl.scaled(spec, G=args.groups)
    log(f"workload {spec.name}: X[{spec.n},{spec.d_in}] {spec.x_dtype}, dZ[{spec.n},{spec.d_out}] f32, G={spec.G}")
    t0 = time.perf_counter()
    X = wl.make_x(spec, dev)
    dZ = wl.make_dz_for(spec, dev)
    W, What = wl.make_weights(spec, dev)
    torch.cuda.synchronize()
    log(f"inputs generated on the GPU in {time.perf_counter() - t0:.1f} s")

    n, d_in, d_out, G = spec.n, spec.d_in, spec.d_out, spec.G
    chunks = max(1, spec.chunks)
    s = torch.empty((n, G), dtype=torch.float32, device=dev)
    H = torch.empty((G, d_in, d_in), dtype=torch.float32, device=dev)
    ws_g = torch.empty(max(1, gq.gq_fisher_gram_workspace_bytes(X.dtype, n, d_in, G)), dtype=torch.uint8, device=dev)
    lib = gq.load_library()
    ws_o = torch.empty(max(1, int(lib.gq_objective_workspace_bytes(d_out, d_in, G))), dtype=torch.uint8, device=dev)

    names = ["group_weights", "fisher_gram", "mirror", "objective"]

    def step(events=None):
        ev = events
        if ev is not None:
            ev[0].record()
        gq.gq_group_weights(dZ, G, out=s)
        if ev is not None:
            ev[1].record()
        if chunks == 1:
            gq.gq_fisher_gram(X, s, H=H, workspace=ws_g)
        else:                                   # streamed over token chunks: overwrite, then accumulate
            c = n // chunks
            for i in range(chunks):
                gq.gq_fisher_gram(X[i * c:(i + 1) * c], s[i * c:(i + 1) * c], H=H, accumulate=i > 0, workspace=ws_g)
        if ev is not None:
            ev[2].record()
        gq.gq_fisher_mirror(H)
        if ev is not None:
            ev[3].record()
        obj = gq.gq_objective(W, What, H, workspace=ws_o)
        if ev is not None:
            ev[4].record()
        return obj

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)        # a plain elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # Schedule tuning, part of the warm-up (outside the timed region): the eight XCDs of a chip run the Gram
    # kernel at different speeds; every call records them in its workspace, and the library cuts the left-over
    # work accordingly once it is told.  The Gram call is timed before and after so that both figures are on
    # record; the timed steps below run with the measured speeds unless --no-xcd-calibration is given.
    def gram_call():
        if chunks == 1:
            gq.gq_fisher_gram(X, s, H=H, workspace=ws_g)
        else:
            c = n // chunks
            for i in range(chunks):
                gq.gq_fisher_gram(X[i * c:(i + 1) * c], s[i * c:(i + 1) * c], H=H, accumulate=i > 0, workspace=ws_g)

    def gram_median_ms(reps=5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ts = []
        for _ in range(reps):
            e0.record()
            gram_call()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return sorted(ts)[len(ts) // 2]

    schedule = {"xcd_speeds": None, "note": "default schedule (equal XCD speeds)"}
    if not args.no_xcd_calibration:
        try:
            default_ms = gram_median_ms()
            acc = [0.0] * 8
            for _ in range(3):
                gram_call()
                m = gq.gq_fisher_gram_measured_xcd_speeds(n // chunks, d_in, G, ws_g)
                acc = [a + v / 3.0 for a, v in zip(acc, m)]
            gq.gq_fisher_gram_set_xcd_speeds(acc)
            gram_call()
            tuned_ms = gram_median_ms()
            # The speeds are coupled (an XCD runs faster while others wait), so what is measured under the tuned
            # schedule differs a little from what was measured under the default one: a few rounds of measuring again
            # and averaging, keeping the setting that timed best.
            best = list(acc)
            for _ in range(3):
                m = gq.gq_fisher_gram_measured_xcd_speeds(n // chunks, d_in, G, ws_g)
                acc = [0.5 * (a + v) for a, v in zip(acc, m)]
                gq.gq_fisher_gram_set_xcd_speeds(acc)
                gram_call()
                t = gram_median_ms()
                if t < tuned_ms:
                    tuned_ms, best = t, list(acc)
            acc = best
            gq.gq_fisher_gram_set_xcd_speeds(acc)
            gram_call()
            if tuned_ms > default_ms:             # speeds that do not hold from call to call: keep the default schedule
                gq.gq_fisher_gram_set_xcd_speeds(None)
                gram_call()
            schedule = {"xcd_speeds": acc if tuned_ms <= default_ms else None, "measured_xcd_speeds": acc,
                        "fisher_gram_ms_default_schedule": default_ms,
                        "fisher_gram_ms_with_measured_speeds": tuned_ms,
                        "note": "relative XCD speeds measured during the warm-up from the records the Gram kernel leaves "
                                "in its workspace and set with gq_fisher_gram_set_xcd_speeds; they only move the cuts "
                                "between the runs of the left-over work items"}
            log("schedule:", json.dumps(schedule))
        except gq.GQError as err:                 # shapes without left-over items to cut record nothing
            schedule = {"xcd_speeds": None, "note": f"default schedule ({err})"}
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        obj = step(evs[k])
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    ms_per_step = total_s * 1e3 / args.steps
    import statistics
    samples = {nm: [e[i].elapsed_time(e[i + 1]) for e in evs] for i, nm in enumerate(names)}
    samples["step"] = [e[0].elapsed_time(e[4]) for e in evs]
    per_kernel = {nm: sum(v) / len(v) for nm, v in samples.items() if nm != "step"}
    per_kernel_median = {nm: statistics.median(v) for nm, v in samples.items()}
    per_kernel_min = {nm: min(v) for nm, v in samples.items()}
    log("per-call ms (HIP events, mean over timed steps):", json.dumps(per_kernel))
    log("per-call ms (median):", json.dumps(per_kernel_median))

    fl = gram_flops(G, n, d_in)
    value = fl / (ms_per_step * 1e-3) / 1e12
    gram_ms = per_kernel["fisher_gram"]
    achieved = fl / (gram_ms * 1e-3) / 1e12
    dz_bytes = dZ.numel() * 4 + s.numel() * 4                       # K1: dZ once, s written
    mirror_bytes = 4.0 * G * d_in * (d_in - 1)                      # mirror: strict upper triangle read, strict lower written
    dz_gbs = dz_bytes / (per_kernel["group_weights"] * 1e-3) / 1e9
    mirror_gbs = mirror_bytes / (per_kernel["mirror"] * 1e-3) / 1e9
    props = torch.cuda.get_device_properties(0)
    traffic, traffic_source = load_traffic(spec.name)

    result = {
        "metric": "Fisher-Gram TFLOP/s (algorithmic, upper triangle) over one linear layer's whole GuidedQuant pass",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{spec.name}: X[{n},{d_in}] bf16, dZ[{n},{d_out}] f32, G={G}, "
                               f"W[{d_out},{d_in}] f32 with 3-bit per-row codebook What",
                   "tokens": n, "d_in": d_in, "d_out": d_out, "G": G, "token_chunks": chunks},
        "pct_of_mfma_peak": 100.0 * achieved / PEAK_BF16_TFLOPS,
        "ms_per_call": per_kernel, "ms_per_call_median": per_kernel_median, "ms_per_call_min": per_kernel_min,
        "ms_per_step_median": per_kernel_median["step"], "ms_per_step_min": per_kernel_min["step"],
        "schedule": schedule,
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "hbm_GiB": round(props.total_memory / 2 ** 30, 1)},
        "group_weights_GBps": dz_gbs,
        "hbm_kernels": {
            "group_weights": {"bytes_per_launch": dz_bytes, "GBps": dz_gbs, "frac_of_8TBps": dz_gbs / 8000.0},
            "mirror": {"bytes_per_launch": mirror_bytes, "GBps": mirror_gbs, "frac_of_8TBps": mirror_gbs / 8000.0}},
        "roofline": {"bound": "mfma", "kernel": "fisher_gram_bf16", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "traffic_source": traffic_source,
                     "flop_per_launch": fl, "ms_per_launch": gram_ms, "ms_per_launch_median": per_kernel_median["fisher_gram"],
                     "ms_per_launch_min": per_kernel_min["fisher_gram"],
                     "note": "one launch = one gq_fisher_gram call (weight repack + Gram kernel + second pass of the split tiles), "
                             "HIP events on the launch stream around the call"},
    }

    if args.cd_cycles > 0:
        # The step that consumes H (Section 4.2): timed on its own, after the hot path, on the H just
        # built (diagonal damped by 1 % of its mean, as every user of H does) and the 3-bit grids.
        Hd = gq.gq_damp_diagonal(H.clone(), 0.01, 0.0)
        _, C = wl.quantize_codebook_per_row(W, 3, return_codebook=True)
        ws_c = torch.empty(int(lib.gq_cd_workspace_bytes(d_out, d_in, G)), dtype=torch.uint8, device=dev)
        Wq = What.clone()
        gq.gq_cd_assign(W, Wq, C, Hd, n_cycles=1, want_codes=False, workspace=ws_c)      # warm-up
        Wq = What.clone()
        o_before = gq.gq_objective(W, Wq, Hd, workspace=ws_o)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        Qc = gq.gq_cd_assign(W, Wq, C, Hd, n_cycles=args.cd_cycles, want_codes=True, workspace=ws_c)
        e1.record()
        o_after = gq.gq_objective(W, Wq, Hd, workspace=ws_o)
        torch.cuda.synchronize()
        cd_ms = e0.elapsed_time(e1)
        cd_fl = 2.0 * d_out * d_in * d_in * args.cd_cycles          # the sums of Eq. (cd_closed), once per coordinate and cycle
        result["cd_assign"] = {
            "cycles": args.cd_cycles, "ms": cd_ms, "ms_per_cycle": cd_ms / args.cd_cycles, "levels": 8,
            "objective_before": [float(v) for v in o_before.tolist()], "objective_after": [float(v) for v in o_after.tolist()],
            "roofline": {"bound": "mfma", "achieved": cd_fl / (cd_ms * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS / 3,
                         "unit": "TFLOP/s", "frac": cd_fl / (cd_ms * 1e-3) / 1e12 / (PEAK_BF16_TFLOPS / 3), "traffic": None,
                         "note": "fp32-grade multiply-adds (three bf16 MFMA products each), 2*d_out*d_in^2 per cycle; "
                                 "the walk inside a block of 128 coordinates is sequential"},
        }
        log(f"cd_assign: {cd_ms / args.cd_cycles:.2f} ms per cycle; objective {result['cd_assign']['objective_before']} -> "
            f"{result['cd_assign']['objective_after']}")
        del ws_c
        # ... and the other half of the alternation: the closed-form grids for the assignments just made.
        m = 8
        ws_l = torch.empty(int(lib.gq_lnq_codebook_workspace_bytes(d_out, d_in, G, m)), dtype=torch.uint8, device=dev)
        Wl = torch.empty_like(W)
        gq.gq_lnq_codebook(W, Qc, Hd, m, 1e-7, What=Wl, workspace=ws_l)                  # warm-up
        e0.record()
        gq.gq_lnq_codebook(W, Qc, Hd, m, 1e-7, What=Wl, workspace=ws_l)
        e1.record()
        o_grid = gq.gq_objective(W, Wl, Hd, workspace=ws_o)
        torch.cuda.synchronize()
        lnq_ms = e0.elapsed_time(e1)
        lnq_fl = 2.0 * d_out * m * d_in * d_in                       # P^T H for every channel: the contraction that dominates
        result["lnq_codebook"] = {
            "ms": lnq_ms, "levels": m, "objective_before": [float(v) for v in o_after.tolist()],
            "objective_after": [float(v) for v in o_grid.tolist()],
            "roofline": {"bound": "mfma", "achieved": lnq_fl / (lnq_ms * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS / 3,
                         "unit": "TFLOP/s", "frac": lnq_fl / (lnq_ms * 1e-3) / 1e12 / (PEAK_BF16_TFLOPS / 3), "traffic": None,
                         "note": "fp32-grade multiply-adds (three bf16 MFMA products each), 2*d_out*levels*d_in^2; "
                                 "the whole call: split of H, contraction, binning and the fp64 solves"},
        }
        log(f"lnq_codebook: {lnq_ms:.2f} ms; objective -> {result['lnq_codebook']['objective_after']}")
        # ... and the whole alternation of Algorithm 2 with the paper's T and K (T = 1 for the 70B shapes), from plain rounding.
        T_lnq = 1 if "70b" in spec.name else 2
        Q0 = torch.argmin((C[:, None, :] - What[:, :, None]).abs(), dim=2).to(torch.uint8).contiguous() if d_out * d_in * m <= (1 << 31) \
            else torch.cat([torch.argmin((C[r:r + 1024, None, :] - What[r:r + 1024, :, None]).abs(), dim=2).to(torch.uint8)
                            for r in range(0, d_out, 1024)]).contiguous()
        ws_a = torch.empty(int(lib.gq_lnq_workspace_bytes(d_out, d_in, G, m)), dtype=torch.uint8, device=dev)
        Qa = Q0.clone()
        gq.gq_lnq(W, Qa, Hd, m, n_iters=T_lnq, n_cycles=4, What=Wl, workspace=ws_a)     # warm-up
        Qa = Q0.clone()
        e0.record()
        gq.gq_lnq(W, Qa, Hd, m, n_iters=T_lnq, n_cycles=4, What=Wl, workspace=ws_a)
        e1.record()
        o_lnq = gq.gq_objective(W, Wl, Hd, workspace=ws_o)
        torch.cuda.synchronize()
        result["lnq"] = {"ms": e0.elapsed_time(e1), "T": T_lnq, "K": 4, "levels": m,
                         "objective_plain_rounding": [float(v) for v in o_before.tolist()],
                         "objective_after": [float(v) for v in o_lnq.tolist()]}
        log(f"lnq (T={T_lnq}, K=4): {result['lnq']['ms']:.2f} ms; objective -> {result['lnq']['objective_after']}")
        del Wq, ws_l, ws_a, Wl, Qc, Qa, Q0
        # ... and the sequential-rounding alternative (GPTQ / LDLQ): factor the damped H, round with feedback.
        # A factorization needs a positive definite H; the one-term H of the step above is indefinite beyond
        # 1 % damping for most shapes.  Two remedies are timed: the scaled operand in two bf16 terms for every
        # token, and for the heaviest tokens only (the H that is factored below).
        def gram_mode(**mode):
            if chunks == 1:
                gq.gq_fisher_gram(X, s, H=H, workspace=ws_g, **mode)
            else:
                c = n // chunks
                for i in range(chunks):
                    gq.gq_fisher_gram(X[i * c:(i + 1) * c], s[i * c:(i + 1) * c], H=H, accumulate=i > 0, workspace=ws_g,
                                      **mode)
        mode_ms = {}
        for label, mode in (("two_terms", {"two_terms": True}), ("heavy_two_terms", {"heavy_two_terms": True})):
            gram_mode(**mode)                                                             # warm-up
            ts = []
            for _ in range(5):
                e0.record()
                gram_mode(**mode)
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            mode_ms[label] = statistics.median(ts)
        if chunks > 1:
            # chunked calls: the heavy rows of all chunks gathered in a pool, ONE two-term pass at the end instead of
            # a read-modify-write of the whole H per chunk
            c = n // chunks
            pool_rows = 32 * chunks * max(1, -(-c // 2048))
            pool = gq.gq_fisher_gram_heavy_pool(d_in, G, pool_rows, dev)
            ws_p = torch.empty(max(int(lib.gq_fisher_gram_workspace_bytes(gq.GQ_BF16, pool_rows, d_in, G)), 256),
                               dtype=torch.uint8, device=dev)

            def gram_deferred():
                for i in range(chunks):
                    gq.gq_fisher_gram_heavy_deferred(X[i * c:(i + 1) * c], s[i * c:(i + 1) * c], pool, pool_rows, H=H,
                                                     accumulate=i > 0, workspace=ws_g)
                gq.gq_fisher_gram_heavy_flush(pool, pool_rows, H, workspace=ws_p)
            gram_deferred()                                                               # warm-up
            ts = []
            for _ in range(5):
                e0.record()
                gram_deferred()
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            mode_ms["heavy_deferred"] = statistics.median(ts)
            result["fisher_gram_heavy_deferred"] = {
                "ms": mode_ms["heavy_deferred"], "pool_rows": pool_rows,
                "frac_of_peak": fl / (mode_ms["heavy_deferred"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                "note": "gq_fisher_gram_heavy_deferred per chunk + one gq_fisher_gram_heavy_flush: the same heavy rows in "
                        "two bf16 terms, their pass once instead of once per chunk; this H is the one factored below"}
        gq.gq_fisher_mirror(H)
        torch.cuda.synchronize()
        gram2_ms = mode_ms["two_terms"]
        result["fisher_gram_two_terms"] = {"ms": gram2_ms, "TFLOPs_algorithmic": fl / (gram2_ms * 1e-3) / 1e12,
                                           "TFLOPs_executed_over_peak": 2 * fl / (gram2_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                                           "note": "every product with the scaled operand in two bf16 terms: within ~1e-5 of "
                                                   "the fp32 path, positive semidefinite to that level"}
        gram_h_ms = mode_ms["heavy_two_terms"]
        result["fisher_gram_heavy_two_terms"] = {
            "ms": gram_h_ms, "TFLOPs_algorithmic": fl / (gram_h_ms * 1e-3) / 1e12,
            "frac_of_peak": fl / (gram_h_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "note": "the H a factorization can consume (factored below at 1 % damping): two bf16 terms only for the "
                    "tokens whose weight exceeds 16 times the mean; the one-term H of the timed step is within 3e-3 "
                    "but indefinite at that damping for most shapes"}
        ws_f = torch.empty(int(lib.gq_cholesky_workspace_bytes(d_in, G)), dtype=torch.uint8, device=dev)
        ws_c = torch.empty(int(lib.gq_cd_workspace_bytes(d_out, d_in, G)), dtype=torch.uint8, device=dev)
        gq.gq_damped_cholesky(H, 0.01, 0.0, reverse=True, workspace=ws_f)                 # warm-up
        e0.record()
        Rf, info = gq.gq_damped_cholesky(H, 0.01, 0.0, reverse=True, workspace=ws_f)
        e1.record()
        gq.gq_ldlq_assign(W, C, Rf, workspace=ws_c)                                       # warm-up
        e2, e3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e2.record()
        Ws, _ = gq.gq_ldlq_assign(W, C, Rf, want_codes=False, workspace=ws_c)
        e3.record()
        o_seq = gq.gq_objective(W, Ws, Hd, workspace=ws_o)
        torch.cuda.synchronize()
        chol_ms, seq_ms = e0.elapsed_time(e1), e2.elapsed_time(e3)
        chol_fl = G * d_in ** 3 / 3.0                                   # flop of the factorization (d^3/3 per group)
        result["sequential_rounding"] = {
            "cholesky_ms": chol_ms, "ldlq_assign_ms": seq_ms, "levels": 8, "info": [int(v) for v in info.tolist()],
            "positive_definite": not any(info.tolist()),
            "objective_plain_rounding": [float(v) for v in o_before.tolist()],
            "objective_after": [float(v) for v in o_seq.tolist()] if not any(info.tolist()) else None,
            "note": None if not any(info.tolist()) else
                    "H is not positive definite at 1 % damping for this shape: the factor is invalid, only the times "
                    "are meaningful",
            "roofline": {"bound": "mfma", "kernel": "cholesky (fp32)", "achieved": chol_fl / (chol_ms * 1e-3) / 1e12,
                         "peak": 157.3, "unit": "TFLOP/s", "frac": chol_fl / (chol_ms * 1e-3) / 1e12 / 157.3, "traffic": None,
                         "note": "fp32 matrix-core peak; the 128 sequential pivots of every diagonal block and panel "
                                 "bound the small sizes, the trailing update the large ones"},
        }
        log(f"two-term Gram {gram2_ms:.2f} ms, heavy-token two-term Gram {gram_h_ms:.2f} ms; sequential rounding: cholesky {chol_ms:.2f} ms, ldlq_assign {seq_ms:.2f} ms; objective -> "
            f"{result['sequential_rounding']['objective_after']}")
        del Hd, ws_f, ws_c, Rf, Ws

    if not args.no_ceiling:
        ceil = mfma_ceiling()
        if ceil:
            result["mfma_ceiling"] = ceil
            result["roofline"]["frac_of_measured_ceiling"] = achieved / ceil["random_operands_tflops"]
            result["device"]["shader_clock_GHz_under_bf16_mfma_load"] = ceil.get("shader_clock_GHz_random_operands")
            result["device"]["max_clock_MHz"] = ceil.get("max_clock_MHz")
            rd, cp = ceil.get("hbm_read_stream_GBps"), ceil.get("hbm_copy_GBps")
            if rd:
                result["hbm_kernels"]["read_stream_ceiling_GBps"] = rd
                result["hbm_kernels"]["group_weights"]["frac_of_read_stream_ceiling"] = dz_gbs / rd
            if cp:
                result["hbm_kernels"]["copy_ceiling_GBps"] = cp
                result["hbm_kernels"]["mirror"]["frac_of_copy_ceiling"] = mirror_gbs / cp

    if not args.no_cpu_baseline:
        import numpy as np
        ns = min(args.cpu_sample_tokens, n)
        base, H_ref, obj_ref = cpu_baseline(spec, X, dZ, W, What, ns)
        result["cpu_baseline"] = base
        # the same sample through the HIP path, compared with what the oracle just computed
        s2 = gq.gq_group_weights(dZ[:ns], G)
        H2 = gq.gq_fisher_gram(X[:ns], s2, mirror=True)
        obj2 = gq.gq_objective(W, What, H2)
        torch.cuda.synchronize()
        Hg = H2.to("cpu").to(torch.float64).numpy()
        eh = max(float(np.linalg.norm(Hg[k] - H_ref[k]) / np.linalg.norm(H_ref[k])) for k in range(G))
        eo = float(np.max(np.abs(obj2.cpu().numpy() - obj_ref) / obj_ref))
        result["check"] = {"sample_tokens": ns, "H_rel_fro_max": eh, "obj_rel_max": eo, "tolerance": 3e-3}
        log(f"check on the oracle's sample: H rel-Frobenius {eh:.2e}, objective {eo:.2e}")
        if not (eh <= 3e-3 and eo <= 3e-3):
            log("PARITY CHECK FAILED")
            print(json.dumps(result))
            sys.exit(2)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
