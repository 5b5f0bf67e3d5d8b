"""Parity assertions of the GPU tests.  The error measures and tolerances themselves live in
``paper_2604_23798_amd.metrics`` (the benchmark reports the same numbers).

Binding everywhere: e_row <= tol, e_mix <= tol, and the literal elementwise form |d| / (|ref| + 1e-6) <= tol on
the well-conditioned elements (|ref| >= rms of the reference row).  The literal form over ALL elements is
reported with the fraction above the tolerance; the full-size tests additionally require that this fraction
and the worst element stay within a small factor of a plain CPU evaluation in the same precision."""
from paper_2604_23798_amd.metrics import U32, drift_metrics, ladder_check, metrics, passes, tolerance  # noqa: F401


def assert_parity(out, ref, tol, what=""):
    m = metrics(out, ref, tol)
    msg = "%s e_row=%.3g e_mix=%.3g e_well=%.3g e_elem=%.3g (%.3g%% of elements above %.0e) tol=%.0e" % (
        what, m["e_row"], m["e_mix"], m["e_well"], m["e_elem"], 100 * m["frac_elem_viol"], tol, tol)
    print(msg)
    assert passes(m, tol), msg
    return m
