"""Error measures and tolerances for comparing an attention output with a reference (numpy only; no
attention arithmetic lives here).  Shared by the GPU tests, the smoke check and the benchmark.

Tolerances (max over elements / rows, FP64 reference):
  FP32 I/O: 2e-5 for n <= 4096, 1e-4 for n <= 65536;  FP16 I/O (FP32 accumulation): 2e-3.

Measures, all from the same two arrays:
  e_elem   max |d| / (|ref| + 1e-6)           -- the literal elementwise form.  Ill-conditioned on output
           elements that are near zero by cancellation: any FP32-accumulating evaluation (the single-precision
           fold of Alg. 1 included) exceeds 2e-5 on 1-2 % of the elements of the N(0,1) workloads.
  e_well   the same maximum over the WELL-CONDITIONED elements only, |ref| >= rms(ref row): there the literal
           tolerance is attainable and is binding.
  e_row    max over rows of ||d||_2 / ||ref||_2    -- the form of the paper's bound (Thm 1).
  e_mix    max |d| / (|ref| + rms(ref row))        -- elementwise with the row's own scale as the floor.
"""
import numpy as np

U32 = 2.0 ** -24


def tolerance(n, fp16=False):
    if fp16:
        return 2e-3
    return 2e-5 if n <= 4096 else 1e-4


def metrics(out, ref, tol):
    out = np.asarray(out, np.float64)
    ref = np.asarray(ref, np.float64)
    assert out.shape == ref.shape and out.ndim == 2
    assert np.all(np.isfinite(out)), "non-finite output"
    d = np.abs(out - ref)
    e_elem = d / (np.abs(ref) + 1e-6)
    rn = np.linalg.norm(ref, axis=1)
    dn = np.linalg.norm(out - ref, axis=1)
    e_row = np.where(rn > 0, dn / np.where(rn > 0, rn, 1.0), dn)
    rms = np.sqrt(np.mean(ref * ref, axis=1, keepdims=True))
    e_mix = d / (np.abs(ref) + rms + 1e-300)
    well = np.abs(ref) >= rms
    return {"e_elem": float(e_elem.max(initial=0.0)), "frac_elem_viol": float(np.mean(e_elem > tol)) if d.size else 0.0,
            "e_well": float(e_elem[well].max(initial=0.0)), "frac_well": float(np.mean(well)) if d.size else 0.0,
            "e_row": float(e_row.max(initial=0.0)), "e_mix": float(e_mix.max(initial=0.0)),
            "max_abs": float(d.max(initial=0.0))}


def passes(m, tol):
    """The binding check: row-norm and mixed elementwise error within the tolerance everywhere, and the
    literal elementwise error within it on the well-conditioned elements."""
    return bool(m["e_row"] <= tol and m["e_mix"] <= tol and m["e_well"] <= tol)


def ladder_check(m_out, m_ladder, frac_slack=1.25, elem_slack=4.0):
    """Are the violations of the literal elementwise tolerance those that the reduced-precision format itself
    causes?  ``m_ladder``: metrics of a plain CPU evaluation in the same format (a 'ladder') on the same rows.
    True when the fraction of violating elements is at most ``frac_slack`` times the ladder's (plus one part in
    ten thousand) and the worst element at most ``elem_slack`` times the ladder's worst."""
    return bool(m_out["frac_elem_viol"] <= frac_slack * m_ladder["frac_elem_viol"] + 1e-4 and
                m_out["e_elem"] <= elem_slack * m_ladder["e_elem"])


def drift_metrics(P_hat, P_ref, Y_hat, Y_ref):
    """The six drift metrics of the paper's numerical-equivalence section, per query row
    (P: [R, n] attention probabilities, Y: [R, d] outputs), each summarised as
    (median, 95th, 99th percentile) over rows: max |dP|, ||dP||_2/||P||_2, Jensen-Shannon
    divergence, argmax disagreement (rate), max |dY|, ||dY||_2/||Y||_2."""
    P_hat, P_ref = np.asarray(P_hat, np.float64), np.asarray(P_ref, np.float64)
    Y_hat, Y_ref = np.asarray(Y_hat, np.float64), np.asarray(Y_ref, np.float64)
    dP, dY = P_hat - P_ref, Y_hat - Y_ref

    def kl(a, b):
        with np.errstate(divide="ignore", invalid="ignore"):
            t = np.where(a > 0, a * (np.log(a) - np.log(b)), 0.0)
        return t.sum(axis=1)
    M = 0.5 * (P_hat + P_ref)
    js = 0.5 * kl(P_hat, M) + 0.5 * kl(P_ref, M)
    rows = {
        "dP_inf": np.abs(dP).max(axis=1),
        "dP_l2_rel": np.linalg.norm(dP, axis=1) / np.linalg.norm(P_ref, axis=1),
        "js": np.maximum(js, 0.0),
        "dY_inf": np.abs(dY).max(axis=1),
        "dY_l2_rel": np.linalg.norm(dY, axis=1) / np.linalg.norm(Y_ref, axis=1),
    }
    out = {k: tuple(float(np.percentile(v, p)) for p in (50, 95, 99)) for k, v in rows.items()}
    out["arg_rate"] = float(np.mean(P_hat.argmax(axis=1) != P_ref.argmax(axis=1)))
    return out
