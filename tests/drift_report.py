"""The six drift metrics of the paper's numerical-equivalence section at a workload's full size.

    python -m tests.drift_report --workload sweep_n16384 [--rows 512]

Runs the GPU path once (elsa_attn_fwd_lse, library defaults) and compares sampled query rows with the
FP64 oracle.  Prints one JSON line.  Test infrastructure: it may use the oracle, the product may not."""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def drift_report(workload, nrows):
    """The six drift metrics of the paper's numerical-equivalence section at a workload's full size,
    on sampled query rows: the GPU's output and row log-normaliser (elsa_attn_fwd_lse) against the
    FP64 oracle; probabilities are P_ij = exp(s_ij - lse_i) with FP64 scores on both sides (the
    kernels never materialise P).  (median, 95th, 99th percentile) over the sampled rows."""
    import numpy as np
    import torch
    import oracle
    from paper_2604_23798_amd import elsa, inputs
    from tests.parity import drift_metrics
    name = workload
    if name not in inputs.WORKLOADS and name.endswith("_fp16") and name[:-5] in inputs.WORKLOADS:
        w = inputs.WORKLOADS[name[:-5]].with_(fp16=True, name=name)
    else:
        w = inputs.WORKLOADS[name]
    q, k, v, kv_len = inputs.make(w)
    tq, tk, tv = (torch.from_numpy(t).cuda() for t in (q, k, v))
    tl = None if kv_len is None else torch.from_numpy(kv_len).cuda()
    out = torch.empty_like(tq)
    lse = torch.empty(tq.shape[:3], dtype=torch.float32, device="cuda")
    elsa.elsa_attn_fwd_lse(tq, tk, tv, out, lse, w.scale, w.causal, tl)
    torch.cuda.synchronize()
    kernel = elsa.elsa_last_kernel()
    per_head = max(1, min(w.n, nrows // (w.B * w.H)))
    rows = inputs.sample_rows(w, per_head=per_head)
    f32 = lambda t: t.astype(np.float32)
    ref_y = oracle.attn_rows(f32(q), f32(k), f32(v), w.scale, causal=w.causal, kv_len=kv_len, rows=rows)
    ref_lse = oracle.lse_rows(f32(q), f32(k), w.scale, causal=w.causal, kv_len=kv_len, rows=rows)
    got_y = out.reshape(-1, w.d)[torch.from_numpy(rows).cuda()].double().cpu().numpy()
    got_lse = lse.reshape(-1)[torch.from_numpy(rows).cuda()].double().cpu().numpy()
    qd, kd = q.astype(np.float64).reshape(-1, w.d), k.astype(np.float64).reshape(w.B * w.H, w.n, w.d)
    P_hat, P_ref = np.empty((rows.size, w.n)), np.empty((rows.size, w.n))
    for r, row in enumerate(rows):
        bh, i = divmod(int(row), w.n)
        sc = w.scale * (kd[bh] @ qd[row])
        lim = w.n if kv_len is None else int(min(max(kv_len[bh // w.H], 0), w.n))
        if w.causal:
            lim = min(lim, i + 1)
        sc[lim:] = -np.inf
        P_hat[r], P_ref[r] = np.exp(sc - got_lse[r]), np.exp(sc - ref_lse[r])
    keep = np.isfinite(ref_lse)                      # rows with at least one visible key
    m = drift_metrics(P_hat[keep], P_ref[keep], got_y[keep], ref_y[keep])
    return {"metric": "drift against the FP64 oracle: (median, p95, p99) over sampled rows", "workload": name, "kernel": kernel,
            "dtype": "f16 io / f32 state" if w.fp16 else "f32", "rows": int(keep.sum()), "n": w.n, "d": w.d, "n_gpus": 1,
            "max_abs_dP": m["dP_inf"], "rel_l2_dP": m["dP_l2_rel"], "jensen_shannon": m["js"], "argmax_disagreement": m["arg_rate"],
            "max_abs_dY": m["dY_inf"], "rel_l2_dY": m["dY_l2_rel"]}


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="sweep_n16384")
    ap.add_argument("--rows", type=int, default=512, help="sampled query rows in total")
    a = ap.parse_args()
    print(json.dumps(drift_report(a.workload, a.rows)))
