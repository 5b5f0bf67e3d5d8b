#!/usr/bin/env python3
"""Benchmark of the ELSA attention hot path on one MI355X.

A step is one pass of the whole path (one ``elsa_attn_fwd`` call: score tiles, monoid fold,
PV accumulation, normalise/store; plus the combine pass when the library splits keys) over
one batch of seeded synthetic input that is already resident in HBM.  The default workload is
the one the headline metric is quoted on: the long-sequence sweep at n = 16384, d = 64
(B = 1, H = 16), FP32.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--path auto|fma|mfma|mfma16]

``--workload`` takes any name of ``paper_2604_23798_amd.inputs.WORKLOADS``, ``decode_32k[_fp16]``, ``dv_<d>_<d_v>_<n>[_causal][_fp16]`` or ``varlen_8x1792``
(8 packed sequences with lengths uniform on [256, 1792], H = 12, d = 64; add ``_fp16`` for FP16).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_TFLOPS = 157.3        # MI355X dense FP32 (matrix = vector peak): 256 CU x 256 flop/clk x 2.4 GHz
PEAK_FP32_VALU_UNPACKED = 78.6  # plain v_fma_f32 (packed FP32 is disabled in this build): half of the above
PEAK_FP16_TFLOPS = 2500.0       # MI355X dense FP16 MFMA
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by what the same
# counter reads for a plain copy of known size in the same run (profiles/*_counters.md).
# Keyed by (workload, kernel actually launched); the value names the summary the figure comes from.
MEASURED_TRAFFIC = {("sweep_n16384", "mfma_q128_k32"): (1.38e9, "profiles/fwd_mfma_sweep_n16384_counters.md"),
                    ("sweep_n16384_fp16", "mfma16_q256_w4"): (3.06e8, "profiles/fwd_mfma16_experiments.md"),
                    ("sweep_n16384", "mfma_q256_w4"): (6.606e8, "profiles/fwd_mfma_sweep_n16384_counters.md"),
                    ("decode_32k", "fma_decode_q1"): (2.685e9, "profiles/fwd_decode_decode_32k.md")}
# the other workloads, appended to the default run's JSON line as `configs` (each timed briefly after the headline)
CONFIG_WORKLOADS = ["vit_b16_224", "bert_base", "bert_base_padded", "sweep_n1024", "sweep_n2048", "sweep_n4096", "sweep_n8192",
                    "sweep_n1024_fp16", "sweep_n2048_fp16", "sweep_n4096_fp16", "sweep_n8192_fp16", "sweep_n16384_fp16",
                    "llama13b_32k", "llama13b_32k_fp16", "hires_vit_64k"]


def host_cores():
    """(logical cores of the box, cores this process may run on)."""
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return os.cpu_count() or 1, usable


def traffic_of(name, kernel):
    t = MEASURED_TRAFFIC.get((name, kernel))
    return (t[0], t[1]) if t else (None, None)


def roof_of(kernel):
    if kernel.startswith("fma"):
        return "alu", PEAK_FP32_VALU_UNPACKED
    if kernel.startswith("mfma16"):
        return "mfma", PEAK_FP16_TFLOPS
    return "mfma", PEAK_FP32_TFLOPS


def spot_parity(w, q, k, v, kv_len, gpu_out, per_head):
    """Oracle and CPU ladder on a seeded row sample of the workload; error measures of the GPU output against
    the oracle, plus the literal-tolerance violations of the ladder on the same rows.  Returns (parity, seconds
    the FP64 oracle took, visible-key flops of the sample)."""
    import numpy as np
    import oracle
    from paper_2604_23798_amd import inputs
    from paper_2604_23798_amd.metrics import ladder_check, metrics, passes, tolerance
    rows = inputs.sample_rows(w, per_head=per_head)
    f32 = lambda t: t.astype(np.float32)
    qq, kk, vv = f32(q), f32(k), f32(v)
    oracle.attn_rows(qq, kk, vv, w.scale, causal=w.causal, kv_len=kv_len, rows=rows[:2])   # page in
    t0 = time.perf_counter()
    ref = oracle.attn_rows(qq, kk, vv, w.scale, causal=w.causal, kv_len=kv_len, rows=rows)
    dt = time.perf_counter() - t0
    if w.fp16:
        lad = oracle.ladder_f16_rows(qq, kk, vv, w.scale, causal=w.causal, kv_len=kv_len, rows=rows)
    else:
        lad = oracle.ladder_f32_fold_rows(qq, kk, vv, w.scale, causal=w.causal, kv_len=kv_len, rows=rows).astype(np.float64)
    tol = tolerance(w.n, w.fp16)
    par = metrics(gpu_out.reshape(-1, w.d)[rows], ref, tol)
    ml = metrics(lad, ref, tol)
    par.update({"tol": tol, "rows": int(rows.size), "pass": passes(par, tol), "e_elem_wellcond": par["e_well"],
                "ladder": "fp16 weights and output" if w.fp16 else "fp32 fold", "ladder_frac_elem_viol": ml["frac_elem_viol"],
                "ladder_e_elem": ml["e_elem"], "literal_form_as_ladder": ladder_check(par, ml)})
    i = rows % w.n
    vis = np.minimum(i + 1, w.n) if w.causal else np.full(rows.shape, w.n)
    if kv_len is not None:
        vis = np.minimum(vis, kv_len[rows // (w.n * w.H)])
    return par, dt, float(4 * w.d * vis.sum())


def bench_configs(names, launches, per_head):
    """Time each workload briefly (library defaults, 256 MiB workspace lent, inputs resident) and spot-check it."""
    import numpy as np
    import torch
    from paper_2604_23798_amd import elsa, inputs
    out_rows = []
    cache = {}
    for name in names:
        w = inputs.WORKLOADS[name]
        base = name[:-5] if name.endswith("_fp16") else name
        if base not in cache:                      # the FP16 variant is the same draw, rounded
            cache.clear()
            wb = inputs.WORKLOADS[base]
            cache[base] = inputs.make(wb)
        q, k, v, kv_len = cache[base]
        if w.fp16:
            q, k, v = (t.astype(np.float16) for t in (q, k, v))
        tq, tk, tv = (torch.from_numpy(t).cuda() for t in (q, k, v))
        tl = None if kv_len is None else torch.from_numpy(kv_len).cuda()
        out = torch.full_like(tq, float("nan"))
        step = lambda: elsa.elsa_attn_fwd_masked(tq, tk, tv, out, w.scale, w.causal, tl)
        step()
        torch.cuda.synchronize()
        kernel, splits = elsa.elsa_last_kernel(), elsa.elsa_last_splits()
        # short workloads: enough launches for 20 ms of work, so that one launch's latency is not the figure
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); step(); e1.record(); torch.cuda.synchronize()
        reps = max(launches, min(2000, int(20.0 / max(e0.elapsed_time(e1), 1e-3))))
        tw = time.perf_counter()                   # untimed launches for a quarter second: short workloads otherwise
        while time.perf_counter() - tw < 0.25:     # run before the clocks have ramped up again after the host-side work
            for _ in range(min(reps, 50)):
                step()
            torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            step()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        exec_flops = float(w.flops)
        if w.causal:
            exec_flops = 4.0 * w.B * w.H * w.d * (w.n * (w.n + 1) / 2)
        elif kv_len is not None:
            exec_flops = 4.0 * w.H * w.n * w.d * float(np.minimum(kv_len, w.n).sum())
        bound, peak = roof_of(kernel)
        achieved = exec_flops / (ms * 1e-3) / 1e12
        rec = {"workload": name, "B": w.B, "H": w.H, "n": w.n, "d": w.d, "causal": bool(w.causal), "padded": bool(w.padded),
               "dtype": "f16 io / f32 state" if w.fp16 else "f32", "kernel": kernel, "splits": splits, "launches": reps,
               "ms": ms, "tflops": w.flops / (ms * 1e-3) / 1e12,
               "roofline": {"bound": bound, "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                            "flops_counted": "visible keys only" if (w.causal or kv_len is not None) else "4*B*H*n^2*d"}}
        if per_head > 0:
            assert bool(torch.isfinite(out).all()), name
            par, _, _ = spot_parity(w, q, k, v, kv_len, out.double().cpu().numpy(), min(per_head, w.n))
            rec["parity"] = par
        out_rows.append(rec)
        print("config %s: %s x%d %.4f ms %.1f TFLOP/s (%.3f of the %s roof)%s" % (
            name, kernel, splits, ms, rec["tflops"], achieved / peak, bound,
            "" if per_head <= 0 else " parity pass=%s" % rec["parity"]["pass"]), file=sys.stderr, flush=True)
        del tq, tk, tv, out
    return out_rows




def cpu_baseline(w, q, k, v, kv_len, gpu_out, budget_rows):
    """Time the FP64 oracle (single thread, as it stands) on a bounded row sample of the same
    workload, and use the same rows as a parity spot check of the timed GPU output."""
    per_head = max(2, budget_rows // (w.B * w.H))
    par, dt, flops = spot_parity(w, q, k, v, kv_len, gpu_out, per_head)
    box, usable = host_cores()
    base = {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": 1, "host_cores": box, "host_cores_usable": usable,
            "kind": "oracle",
            "sample": "%d query rows (%d per head: first, last, neighbours of 32/64/128/256-row boundaries, random) of %s, "
                      "all their keys, FP64 single thread, %.1f s" % (par["rows"], per_head, w.name, dt)}
    return base, par


def cpu_baseline_varlen(q, k, v, cu, scale, gpu_out, fp16):
    """Oracle on the first heads of the packed batch (bounded), timed; parity on the same slice."""
    import numpy as np
    import oracle
    from paper_2604_23798_amd.metrics import metrics, passes
    hs = 2
    f32 = lambda t: np.ascontiguousarray(t[:, :hs].astype(np.float32))
    t0 = time.perf_counter()
    ref = oracle.attn_varlen(f32(q), f32(k), f32(v), cu, scale)
    dt = time.perf_counter() - t0
    lens = np.diff(cu).astype(np.float64)
    flops = float(4 * hs * q.shape[2] * np.sum(lens * lens))
    tol = 2e-3 if fp16 else 2e-5
    par = metrics(gpu_out[:, :hs].reshape(-1, q.shape[2]), ref.reshape(-1, q.shape[2]), tol)
    par["tol"] = tol
    par["pass"] = passes(par, tol)
    box, usable = host_cores()
    base = {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": 1, "host_cores": box, "host_cores_usable": usable, "kind": "oracle",
            "sample": "all rows of the first %d heads of the packed batch, FP64 single thread, %.1f s" % (hs, dt)}
    return base, par


def scaling_fit(a):
    """Per-head latency over n = 2^10..2^15 and the fit T(n) = a*L(n,B) + b*n^2 + c with B = 128
    (the paper's empirical scaling validation; FP16 and FP32 I/O, H = 16, d = 64, no key split)."""
    import math
    import numpy as np
    import torch
    from paper_2604_23798_amd import elsa, inputs
    H, d = 16, 64
    res = {"metric": "per-head attention latency fit T(n) = a*L(n,128) + b*n^2 + c", "unit": "ms", "n_gpus": 1,
           "H": H, "d": d, "steps": a.steps, "warmup": a.warmup, "fits": {}}
    for fp16 in (True, False):
        ns, ts = [], []
        for lg in range(10, 16):
            n = 1 << lg
            w = inputs.Workload("fit", B=1, H=H, n=n, d=d, seed=1200 + lg, fp16=fp16)
            q, k, v, _ = inputs.make(w)
            tq, tk, tv = (torch.from_numpy(t).cuda() for t in (q, k, v))
            out = torch.empty_like(tq)
            for _ in range(a.warmup):
                elsa.elsa_attn_fwd(tq, tk, tv, out, w.scale, False)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(a.steps):
                elsa.elsa_attn_fwd(tq, tk, tv, out, w.scale, False)
            e1.record()
            torch.cuda.synchronize()
            ns.append(n)
            ts.append(e0.elapsed_time(e1) / a.steps / H)
        fit = fit_scaling_law(ns, ts)
        fit["ms_per_head"] = ts
        res["fits"]["fp16" if fp16 else "fp32"] = fit
    return res


def tile_sweep(a):
    """Small dense problems: the library's own choice of tile shape and key chunks against forced
    configurations, each timed in this process (microseconds per launch, 256 MiB workspace lent).
    One JSON object: per shape the default's kernel / chunks / time, every forced time, and the
    ratio default / best forced."""
    import torch
    from paper_2604_23798_amd import elsa, inputs
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)

    def run(B, H, n, d, causal, fp16, path, variant, splits):
        dt = torch.float16 if fp16 else torch.float32
        q, k, v = (torch.from_numpy(inputs.normal(1300 + n + d, st, 0, B * H * n * d).reshape(B, H, n, d)).cuda().to(dt)
                   for st in (inputs.STREAM_Q, inputs.STREAM_K, inputs.STREAM_V))
        out = torch.empty_like(q)
        for o, val in ((elsa.OPT_PATH, path), (elsa.OPT_VARIANT, variant), (elsa.OPT_SPLITS, splits)):
            elsa.elsa_set_option(o, val)
        f = lambda: elsa.elsa_attn_fwd(q, k, v, out, d ** -0.5, causal)
        for _ in range(max(a.warmup, 100)):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(max(a.steps, 200)):
            f()
        e1.record()
        torch.cuda.synchronize()
        for o in (elsa.OPT_PATH, elsa.OPT_VARIANT, elsa.OPT_SPLITS):
            elsa.elsa_set_option(o, 0)
        return e0.elapsed_time(e1) / max(a.steps, 200) * 1e3, elsa.elsa_last_kernel(), elsa.elsa_last_splits()

    f32_narrow = [(2, 7, 1), (2, 7, 2), (2, 7, 4), (2, 11, 1), (2, 11, 2), (2, 3, 1)]
    f32_wide = [(2, 1, 1), (2, 1, 2), (2, 1, 4), (2, 11, 1), (2, 11, 2), (2, 13, 1)]
    f16 = [(3, 1, 1), (3, 2, 1), (3, 3, 1), (3, 4, 1)]
    f32_other = [(2, 1, 1), (2, 1, 2), (2, 1, 4), (2, 3, 1), (2, 3, 2)]       # d = 96, 256: the 128-row tile and (d = 96) the key-splitting one
    shapes = [(1, 16, n, 64, False) for n in (256, 512, 768, 1024, 1536, 2048, 3072)] + \
             [(B, 12, 197, 64, False) for B in (1, 4, 8, 16)] + [(1, 32, 1024, 32, False), (1, 8, 2048, 64, False), (1, 8, 4096, 64, False)] + \
             [(1, 40, n, 128, False) for n in (256, 512, 1024, 2048)] + [(1, 16, 1024, 128, False), (1, 32, 1536, 128, False), (1, 16, 3072, 128, False), (1, 24, 2048, 128, False)] + \
             [(1, 16, n, 64, True) for n in (1024, 2048, 3072, 4096, 8192)] + [(4, 12, 197, 64, True), (1, 8, 4096, 64, True), (1, 16, 2048, 128, True), (1, 8, 4096, 128, True), (1, 40, 1024, 128, True)] + \
             [(1, H, n, d, f) for f in (False, True) for d in (96, 256) for (H, n) in ((16, 2048), (32, 1024), (8, 2048))] + \
             [(B, 12, n, 64, f) for f in (False, True) for (B, n) in ((16, 128), (16, 512), (64, 128), (8, 512))]   # batches of short sequences
    rows = []
    for (B, H, n, d, fp16) in shapes:
        forced = f16 if fp16 else (f32_wide if d == 128 else f32_other if d in (96, 256) else f32_narrow)
        for causal in (False, True):
            us, kern, C = run(B, H, n, d, causal, fp16, 0, 0, 0)
            alts = {}
            for (path, variant, splits) in forced:
                if splits > 1 and n // splits < 256:
                    continue
                t, name, _ = run(B, H, n, d, causal, fp16, path, variant, splits)
                alts["%s x%d" % (name, splits)] = round(t, 1)
            best = min(alts.values())
            rows.append({"B": B, "H": H, "n": n, "d": d, "causal": causal, "fp16": fp16, "default_us": round(us, 1),
                         "default": "%s x%d" % (kern, C), "forced_us": alts, "default_over_best": round(us / best, 3)})
            print("tile-sweep B%d H%d n%d d%d causal=%d fp16=%d: %s %.1f us, best forced %.1f" %
                  (B, H, n, d, causal, fp16, rows[-1]["default"], us, best), file=sys.stderr, flush=True)
    elsa.elsa_set_workspace(None)
    r = [x["default_over_best"] for x in rows]
    return {"metric": "library default / best forced configuration (time per launch)", "n_gpus": 1, "cases": len(rows),
            "mean": sum(r) / len(r), "max": max(r), "rows": rows}


def issue_rates(a):
    """Issue cost of the instruction kinds the fold is made of (``elsa_debug_issue_probe``): alone at one and two
    waves per SIMD, and beside the FP32 / FP16 matrix-core instructions of the other wave of the SIMD.  Reported
    in nanoseconds per instruction and SIMD (constant 100 MHz counter inside the kernel) and in cycles at the
    nominal 2.4 GHz; the clock the part sustains under each load is not read, so the cycle figures are upper bounds."""
    import torch
    from paper_2604_23798_amd import elsa
    kinds = ["v_exp_f32", "v_fma_f32", "v_add_f32", "v_max3_f32", "v_cvt_pk_f16_f32", "v_mfma_f32_32x32x2_f32",
             "v_mfma_f32_32x32x16_f16", "none"]
    per_iter = [16, 16, 16, 16, 16, 8, 8, 0]
    out = torch.zeros(8 + 256 * 512, device="cuda")
    iters = 4000

    def run(ka, kb, waves):
        for _ in range(2):
            elsa.elsa_debug_issue_probe(out, ka, kb, waves, iters)
        torch.cuda.synchronize()
        t = out[:8].cpu().numpy() * 10.0                      # ns per wave of block 0
        ns_a = float(t[:4].mean()) / iters
        ns_b = float(t[4:8].mean()) / iters if waves == 2 else 0.0
        return ns_a, ns_b
    rows = []
    for k in range(7):
        for waves in (1, 2):
            ns_a, ns_b = run(k, k, waves)
            # two waves share the SIMD: per instruction and SIMD it is the longer wave's time over both streams
            ns = max(ns_a, ns_b) / (per_iter[k] * waves)
            rows.append({"a": kinds[k], "b": kinds[k] if waves == 2 else None, "waves_per_simd": waves,
                         "ns_per_instr_and_simd": ns, "cycles_at_2.4GHz": ns * 2.4})
    for m in (5, 6):
        base_a, _ = run(m, 7, 2)
        for k in range(5):
            alone, _ = run(k, 7, 2)
            ns_a, ns_b = run(m, k, 2)
            rows.append({"a": kinds[m], "b": kinds[k], "waves_per_simd": 2,
                         "mfma_ns_per_instr": ns_a / 8, "mfma_alone_ns_per_instr": base_a / 8,
                         "b_ns_per_instr": ns_b / 16, "b_alone_ns_per_instr": alone / 16,
                         "b_slowdown": ns_b / alone, "mfma_slowdown": ns_a / base_a})
    # register-only model of one fold step of the FP16 256-row tile (kinds 8 = its MFMAs, 9 = its fold, 10 = whole step;
    # two query groups per wave and iteration): ns per 32 x 32 step and SIMD at one and two waves per SIMD
    model = []
    names = {8: "MFMAs alone (8 per 32x32 step)", 9: "fold alone", 10: "whole step"}
    for k in (8, 9, 10):
        for waves in (1, 2):
            ns_a, ns_b = run(k, k if waves == 2 else 7, waves)
            ns = max(ns_a, ns_b) / (2 * waves)
            model.append({"part": names[k], "waves_per_simd": waves, "ns_per_step_and_simd": ns, "cycles_at_2.4GHz": ns * 2.4})
    return {"metric": "instruction issue cost on one SIMD (ns per instruction; 16 independent instructions per iteration)",
            "n_gpus": 1, "iters": iters, "rows": rows, "fp16_step_model": model}


def fit_scaling_law(ns, ts, block=128):
    """Least-squares fit of T(n) = a*L(n,B) + b*n^2 + c (the paper's scaling model, L from Eq. 5)
    to latencies ``ts`` at lengths ``ns``.  Returns n, L, a, b, c and R^2."""
    import math
    import numpy as np
    L = [math.ceil(math.log2(block)) + 2 * max(0, math.ceil(math.log2(n / block))) + 3 for n in ns]
    A = np.array([[l, float(n) * n, 1.0] for l, n in zip(L, ns)])
    y = np.asarray(ts, dtype=np.float64)
    coef, *_ = np.linalg.lstsq(A, y, rcond=None)
    pred = A @ coef
    ss_res = float(np.sum((y - pred) ** 2))
    ss_tot = float(np.sum((y - np.mean(y)) ** 2))
    return {"n": list(ns), "L": L, "a": float(coef[0]), "b": float(coef[1]), "c": float(coef[2]),
            "r2": 1.0 - ss_res / ss_tot if ss_tot > 0 else 1.0}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="sweep_n16384")
    ap.add_argument("--path", default="auto", choices=["auto", "fma", "mfma", "mfma16"])
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--xcd-map", type=int, default=0)
    ap.add_argument("--splits", type=int, default=0, help="key chunks per (batch, head): 0 = the library's choice, 1 = single pass")
    ap.add_argument("--oracle-rows", type=int, default=16384, help="row budget of the cpu_baseline leg (0 = skip)")
    ap.add_argument("--pre-warm-ms", type=float, default=0.0,
                    help="run untimed steps for this long before the W warm-up steps (short workloads otherwise "
                         "run before the GPU clocks have ramped up)")
    ap.add_argument("--stream-chunks", type=int, default=0,
                    help="memory-lean mode: feed K and V in this many equal chunks through elsa_attn_stream_step "
                         "(eta = 1/chunks) and finish; dense workloads only")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time replays (launch-bound workloads)")
    ap.add_argument("--scaling-fit", action="store_true",
                    help="instead of one workload: per-head latency for n = 2^10..2^15 (H=16, d=64) and the "
                         "least-squares fit T(n) = a*L(n,128) + b*n^2 + c of the paper's scaling study")
    ap.add_argument("--tile-sweep", action="store_true",
                    help="small problems: the library's tile / chunk choice against forced configurations (about a minute)")
    ap.add_argument("--configs", default="auto",
                    help="after the headline, time the other workloads briefly and append them as `configs`: auto = all of "
                         "them in the default run (no --workload / --path / --variant given), none, or a comma-separated list")
    ap.add_argument("--config-rows", type=int, default=8, help="oracle rows per head of each `configs` entry (0 = no parity)")
    ap.add_argument("--issue-rates", action="store_true",
                    help="instead of a workload: issue cost of the fold's instruction kinds, alone and beside another wave's MFMAs")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference point for rocprofv3 byte counters)")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding)."
              % a.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_23798_amd import elsa, inputs          # fails loudly if libelsa.so is missing

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if a.scaling_fit:
        print(json.dumps(scaling_fit(a)))
        return
    if a.tile_sweep:
        print(json.dumps(tile_sweep(a)))
        return
    if a.issue_rates:
        print(json.dumps(issue_rates(a)))
        return
    varlen = a.workload.startswith("varlen_8x1792")
    decode = a.workload.startswith("decode_32k")
    dvw = a.workload.startswith("dv_")
    if dvw:
        # values of their own width: dv_<d>_<d_v>_<n>[_causal][_fp16], B = 1, H = 16, n queries = n keys
        parts = a.workload.split("_")
        d, dv, n_dv = int(parts[1]), int(parts[2]), int(parts[3])
        fp16, causal = "fp16" in parts[4:], "causal" in parts[4:]
        B, H, nq, nk = 1, 16, n_dv, n_dv
        q = inputs.normal(1012, 0, 0, B * H * nq * d).reshape(B, H, nq, d)
        k = inputs.normal(1012, 1, 0, B * H * nk * d).reshape(B, H, nk, d)
        v = inputs.normal(1012, 2, 0, B * H * nk * dv).reshape(B, H, nk, dv)
        if fp16:
            q, k, v = (t.astype(np.float16) for t in (q, k, v))
        scale = float(np.float32(d ** -0.5))
        flops = 2 * B * H * nq * nk * (d + dv)           # scores contract over d, the weighted sum over d_v
        kv_len = None
    elif decode:
        # one new position per sequence against a 32K-token cache, LLaMA-13B head shape
        fp16 = a.workload.endswith("_fp16")
        B, H, d, nq, nk = 2, 40, 128, 1, 32768
        q = inputs.normal(1007, 0, 0, B * H * nq * d).reshape(B, H, nq, d)
        k = inputs.normal(1007, 1, 0, B * H * nk * d).reshape(B, H, nk, d)
        v = inputs.normal(1007, 2, 0, B * H * nk * d).reshape(B, H, nk, d)
        if fp16:
            q, k, v = (t.astype(np.float16) for t in (q, k, v))
        scale = float(np.float32(d ** -0.5))
        flops = 4 * B * H * nq * nk * d
        causal, kv_len = True, None
    elif varlen:
        fp16 = a.workload.endswith("_fp16")
        H, d = 12, 64
        q, k, v, cu = inputs.make_varlen(1006, 8, 256, 1792, H=H, d=d, fp16=fp16)
        lens = np.diff(cu).astype(np.int64)
        tcu = torch.from_numpy(cu).cuda()
        scale = float(np.float32(d ** -0.5))
        flops = int(4 * H * d * np.sum(lens * lens))
        causal, kv_len = False, None
    else:
        if a.workload not in inputs.WORKLOADS and a.workload.endswith("_fp16") and a.workload[:-5] in inputs.WORKLOADS:
            w = inputs.WORKLOADS[a.workload[:-5]].with_(fp16=True, name=a.workload)     # any workload with FP16 I/O
        else:
            w = inputs.WORKLOADS[a.workload]
        q, k, v, kv_len = inputs.make(w)
        fp16, causal, scale, flops = w.fp16, w.causal, w.scale, w.flops
    # multiply-adds the kernels have to execute (visible keys only): what the roofline fraction is taken on
    exec_flops = float(flops)
    if dvw and causal:
        exec_flops = 2.0 * B * H * (d + dv) * (nq * (nq + 1) / 2)
    elif not (dvw or decode or varlen):
        if w.causal:
            exec_flops = 4.0 * w.B * w.H * w.d * (w.n * (w.n + 1) / 2)
        elif kv_len is not None:
            exec_flops = 4.0 * w.H * w.n * w.d * float(np.minimum(kv_len, w.n).sum())
    tq, tk, tv = (torch.from_numpy(t).cuda() for t in (q, k, v))
    tl = None if kv_len is None else torch.from_numpy(kv_len).cuda()
    out = torch.empty(tq.shape[:-1] + (tv.shape[-1],), dtype=tq.dtype, device="cuda")
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)
    elsa.elsa_set_option(elsa.OPT_PATH, {"auto": 0, "fma": 1, "mfma": 2, "mfma16": 3}[a.path])
    elsa.elsa_set_option(elsa.OPT_VARIANT, a.variant)
    elsa.elsa_set_option(elsa.OPT_XCD_MAP, a.xcd_map)
    elsa.elsa_set_option(elsa.OPT_SPLITS, a.splits)

    if a.calibrate_copy:               # a copy kernel of known size: 256 MiB read + 256 MiB written
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    if a.stream_chunks > 0:
        assert not decode and not varlen and kv_len is None and w.n % a.stream_chunks == 0
        nc = w.n // a.stream_chunks
        kcs = [tk[:, :, i * nc:(i + 1) * nc].contiguous() for i in range(a.stream_chunks)]
        vcs = [tv[:, :, i * nc:(i + 1) * nc].contiguous() for i in range(a.stream_chunks)]
        state = torch.empty(elsa.elsa_stream_state_bytes(w.B, w.H, w.n, w.d), dtype=torch.uint8, device="cuda")

        def step():
            for i in range(a.stream_chunks):
                elsa.elsa_attn_stream_step(tq, kcs[i], vcs[i], state, scale, first=(i == 0), causal=causal,
                                           causal_shift=-i * nc)
            elsa.elsa_attn_stream_finish(state, out)
    elif dvw:
        def step():
            elsa.elsa_attn_fwd_dv(tq, tk, tv, out, scale, causal, tl)
    elif decode:
        def step():
            elsa.elsa_attn_fwd_cross(tq, tk, tv, out, scale, causal, tl)
    elif varlen:
        def step():
            elsa.elsa_attn_fwd_varlen(tq, tk, tv, out, tcu, int(lens.max()), scale, causal)
    else:
        def step():
            elsa.elsa_attn_fwd_masked(tq, tk, tv, out, scale, causal, tl)

    if a.graph:
        eager_step = step
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            eager_step()                       # first launch outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            eager_step()
        step = graph.replay

    if a.pre_warm_ms > 0:
        tw = time.perf_counter()
        while (time.perf_counter() - tw) * 1e3 < a.pre_warm_ms:
            for _ in range(20):
                step()
            torch.cuda.synchronize()
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()                       # on torch's current stream: the stream the kernels are launched on
    for _ in range(a.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / a.steps
    ms_kernel = ev0.elapsed_time(ev1) / a.steps
    kernel = elsa.elsa_last_kernel()
    splits_used = elsa.elsa_last_splits()
    # per-launch spread, from a second pass with one event pair per step (not part of the figure above)
    n_lat = max(a.steps, 20)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_lat + 1)]
    evs[0].record()
    for i in range(n_lat):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    lat = np.sort(np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(n_lat)]))
    latency = {"median": float(np.median(lat)), "p10": float(lat[int(0.1 * (n_lat - 1))]),
               "p90": float(lat[int(0.9 * (n_lat - 1))]), "launches": n_lat}

    # flops: 4 B H n^2 d, the square count the metric is defined on (sum of len^2 for packed batches)
    value = flops / (ms_step * 1e-3) / 1e12
    achieved = exec_flops / (ms_kernel * 1e-3) / 1e12
    bound, peak = roof_of(kernel)
    name = a.workload
    traffic, traffic_src = traffic_of(name, kernel)
    rec = {
        "metric": "FP32 attention TFLOP/s at n=16K, d=64 (4*B*H*n^2*d / time)" if name == "sweep_n16384"
        else "attention TFLOP/s (4*B*H*n^2*d / time)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 io / f32 state" if fp16 else "f32", "data": "synthetic",
        "pct_of_fp32_peak": 100.0 * value / PEAK_FP32_TFLOPS,
        "config": {"workload": name, "causal": bool(causal), "kernel": kernel, "path": a.path, "graph": bool(a.graph),
                   "stream_chunks": a.stream_chunks, "splits": splits_used, "splits_requested": a.splits},
        "roofline": {"bound": bound, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": traffic, "traffic_source": traffic_src,
                     "kernel_ms": ms_kernel},
        "latency_ms": latency,
    }
    if decode:
        # every K and V element is read once: the kernel is bound by HBM, not by the matrix cores
        kv_bytes = 2.0 * B * H * nk * d * (2 if fp16 else 4)
        rec["metric"] = "decode attention: K/V cache bytes consumed per second"
        rec["value"], rec["unit"] = kv_bytes / (ms_step * 1e-3) / 1e9, "GB/s"
        rec["roofline"] = {"bound": "hbm", "achieved": kv_bytes / (ms_kernel * 1e-3) / 1e9, "peak": 8000.0,
                           "unit": "GB/s", "frac": kv_bytes / (ms_kernel * 1e-3) / 1e9 / 8000.0,
                           "traffic": traffic, "traffic_source": traffic_src,
                           "kernel_ms": ms_kernel}
        rec["config"].update({"B": B, "H": H, "n_q": nq, "n_k": nk, "d": d})
        rec["tokens_per_s"] = B * nq / (ms_step * 1e-3)
        del rec["pct_of_fp32_peak"]
    elif dvw:
        rec["metric"] = "attention TFLOP/s (2*B*H*n^2*(d + d_v) / time)"
        rec["config"].update({"B": B, "H": H, "n": nq, "d": d, "d_v": dv})
        if causal:
            rec["causal_effective_tflops"] = 2.0 * B * H * (d + dv) * (nq * (nq + 1) / 2) / (ms_step * 1e-3) / 1e12
    elif varlen:
        rec["config"].update({"num_seqs": 8, "lengths": [int(x) for x in lens], "H": H, "d": d})
        rec["tokens_per_s"] = float(lens.sum()) / (ms_step * 1e-3)
    else:
        rec["config"].update({"B": w.B, "H": w.H, "n": w.n, "d": w.d, "padded": w.padded})
        if kv_len is not None:         # the nominal figure counts padded keys; this one only the visible ones
            rec["visible_keys_tflops"] = 4.0 * w.H * w.n * w.d * float(np.minimum(kv_len, w.n).sum()) / (ms_step * 1e-3) / 1e12
        if w.causal:
            rec["causal_effective_tflops"] = 4.0 * w.B * w.H * w.d * (w.n * (w.n + 1) / 2) / (ms_step * 1e-3) / 1e12
    if a.oracle_rows > 0:
        host = out.double().cpu().numpy()
        if decode:
            import oracle
            t0 = time.perf_counter()
            f32 = lambda x: x.astype(np.float32)
            rows = np.arange(0, B * H, 5, dtype=np.int64)          # one (batch, head) in five
            ref, _ = oracle.cross_rows(f32(q), f32(k), f32(v), scale, causal=True, rows=rows)
            dt = time.perf_counter() - t0
            err = np.linalg.norm(host.reshape(-1, d)[rows] - ref, axis=1) / np.linalg.norm(ref, axis=1)
            base = {"value": rows.size * 2.0 * nk * d * (2 if fp16 else 4) / dt / 1e9, "unit": "GB/s", "cores": 1,
                    "host_cores": host_cores()[0], "kind": "oracle", "sample": "%d of %d (batch, head) rows, all %d keys" % (rows.size, B * H, nk)}
            par = {"rows": int(rows.size), "e_row": float(err.max())}
        elif dvw:
            import oracle
            f32 = lambda x: x.astype(np.float32)
            rows = np.linspace(0, B * H * nq - 1, min(a.oracle_rows, 2048)).astype(np.int64)
            t0 = time.perf_counter()
            ref, _ = oracle.dv_rows(f32(q), f32(k), f32(v), scale, causal=causal, rows=rows)
            dt = time.perf_counter() - t0
            err = np.linalg.norm(host.reshape(-1, dv)[rows] - ref, axis=1) / np.linalg.norm(ref, axis=1)
            vis = (rows % nq + 1).sum() if causal else rows.size * nk
            base = {"value": 2.0 * (d + dv) * float(vis) / dt / 1e12, "unit": "TFLOP/s", "cores": 1, "host_cores": host_cores()[0], "kind": "oracle",
                    "sample": "%d of %d rows (evenly spaced), visible keys only" % (rows.size, B * H * nq)}
            par = {"rows": int(rows.size), "e_row": float(err.max())}
        elif varlen:
            base, par = cpu_baseline_varlen(q, k, v, cu, scale, host, fp16)
        else:
            base, par = cpu_baseline(w, q, k, v, kv_len, host, a.oracle_rows)
        rec["cpu_baseline"] = base
        rec["parity"] = par
    default_run = (a.workload == "sweep_n16384" and a.path == "auto" and a.variant == 0 and a.splits == 0 and a.xcd_map == 0 and
                   a.stream_chunks == 0 and not a.graph)
    names = CONFIG_WORKLOADS if (a.configs == "auto" and default_run) else \
        [] if a.configs in ("auto", "none", "") else [x for x in a.configs.split(",") if x]
    if names:
        del tq, tk, tv, out
        for o in (elsa.OPT_PATH, elsa.OPT_VARIANT, elsa.OPT_XCD_MAP, elsa.OPT_SPLITS):
            elsa.elsa_set_option(o, 0)
        rec["configs"] = bench_configs(names, 5, a.config_rows)
    elsa.elsa_set_workspace(None)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
