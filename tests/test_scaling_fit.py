"""The least-squares fit of the paper's scaling model T(n) = a*L(n,B) + b*n^2 + c, pinned with the
constants the paper prints: latencies generated from them must give them back, with L(n,B) from
Eq. 5, and the merge-depth term must stay identifiable next to the quadratic one."""
import os

import numpy as np

import bench
from oracle.scan import merge_depth

GOLD = os.path.join(os.path.dirname(__file__), "golden", "scaling_fit_constants.txt")


def _constants():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    a, b, c, B = rows[0]
    return float(a), float(b), float(c), int(B)


def test_fit_recovers_the_printed_constants():
    a, b, c, B = _constants()
    ns = [1 << lg for lg in range(10, 16)]
    ts = [a * merge_depth(n, B) + b * float(n) * n + c for n in ns]
    fit = bench.fit_scaling_law(ns, ts, block=B)
    assert fit["L"] == [merge_depth(n, B) for n in ns] == [16, 18, 20, 22, 24, 26]
    assert abs(fit["a"] - a) < 1e-9 and abs(fit["b"] - b) < 1e-15 and abs(fit["c"] - c) < 1e-7
    assert fit["r2"] > 1 - 1e-12


def test_fit_with_noise_and_without_a_depth_term():
    a, b, c, B = _constants()
    ns = [1 << lg for lg in range(10, 16)]
    rng = np.random.default_rng(5)
    ts = [(a * merge_depth(n, B) + b * float(n) * n + c) * (1 + 1e-3 * rng.standard_normal()) for n in ns]
    fit = bench.fit_scaling_law(ns, ts, block=B)
    assert abs(fit["b"] / b - 1) < 5e-3 and fit["r2"] > 0.9999
    flat = bench.fit_scaling_law(ns, [b * float(n) * n for n in ns], block=B)
    assert abs(flat["a"]) < 1e-9 and abs(flat["c"]) < 1e-7
