"""Monoid laws of the merge operator, block composition (Prop. 1) and the paper's two-level scan."""
import math
import os

import numpy as np
import pytest

import oracle
from oracle import scan
from paper_2604_23798_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _state(seed, d, m=None):
    u = inputs.uniform01(seed, 0, 0, d + 2)
    mm = (u[0] * 12.0 - 6.0) if m is None else m
    return (mm, 0.1 + 5.0 * u[1], (u[2:] * 4.0 - 2.0))


def _same(a, b, tol=1e-13):
    assert a[0] == b[0] or abs(a[0] - b[0]) <= tol
    assert abs(a[1] - b[1]) <= tol * (1 + abs(b[1]))
    assert np.all(np.abs(a[2] - b[2]) <= tol * (1 + np.abs(b[2])))


def _canon(u):
    """State -> (log of the unnormalised sum, weighted mean): unique for equivalent states."""
    m, S, W = u
    return m + math.log(S), W / S


# ---- Fig. 1(a): the scan harness on the sum monoid ------------------------------------------

def _fig1a():
    with open(os.path.join(GOLDEN, "fig1a_prefix_sum.txt")) as f:
        lines = [l for l in f if not l.startswith("#")]
    x = [int(t) for t in lines[0].split()]
    p = [int(t) for t in lines[1].split()]
    lo, hi, tot = (int(t) for t in lines[2].split())
    return x, p, lo, hi, tot


def test_fig1a_prefix_sums_all_scan_shapes():
    x, p, lo, hi, tot = _fig1a()
    add = lambda a, b: a + b
    assert scan.sequential_scan(x, add, 0) == p
    assert scan.hillis_steele_scan(x, add) == p
    ex, total = scan.blelloch_exclusive_scan(x, add, 0)
    assert ex == [0] + p[:-1] and total == p[-1]
    for block in (1, 2, 3, 4, 8, 128):
        out, total = scan.two_level_scan(x, add, 0, block)
        assert out == p and total == p[-1]
    assert p[hi - 1] - p[lo - 2] == tot == sum(x[lo - 1:hi])


def test_scan_order_preserved_for_noncommutative_op():
    # string concatenation is associative but not commutative: catches operand swaps in the sweeps
    items = [chr(ord("a") + i) for i in range(13)]
    cat = lambda a, b: a + b
    ref = scan.sequential_scan(items, cat, "")
    assert scan.hillis_steele_scan(items, cat) == ref
    ex, total = scan.blelloch_exclusive_scan(items, cat, "")
    assert [e + x for e, x in zip(ex, items)] == ref and total == ref[-1]
    for block in (2, 4, 5):
        assert scan.two_level_scan(items, cat, "", block)[0] == ref


def test_merge_depth_formula():
    # L(n,B) = ceil(log2 B) + 2 ceil(log2(n/B)) + 3 <= 2 ceil(log2 n) + 3   (Eq. 5), B = 128
    for n, L in ((197, 12), (512, 14), (4096, 20), (16384, 24), (32768, 26), (65536, 28)):
        assert scan.merge_depth(n, 128) == L
        assert L <= 2 * math.ceil(math.log2(n)) + 3


# ---- monoid laws ----------------------------------------------------------------------------

@pytest.mark.parametrize("merge", [oracle.merge_case, oracle.merge_unsum])
def test_identity_is_two_sided(merge):
    e = oracle.identity(5)
    a = _state(1, 5)
    _same(merge(a, e), a, 0)
    _same(merge(e, a), a, 0)
    ee = merge(e, e)
    assert ee[0] == -np.inf and ee[1] == 0.0 and np.all(ee[2] == 0.0)


def test_case_form_equals_compact_form():
    for s in range(40):
        a, b = _state(2 * s, 6), _state(2 * s + 1, 6)
        _same(oracle.merge_case(a, b), oracle.merge_unsum(a, b))
    a, b = _state(7, 6, m=1.5), _state(8, 6, m=1.5)       # equal maxima: either branch
    _same(oracle.merge_case(a, b), oracle.merge_unsum(a, b))
    _same(oracle.merge_case(a, b), oracle.merge_case(b, a))


def test_merge_against_hand_values():
    # a = (0, 1, [2]), b = (ln 2, 3, [-1]): m = ln 2, S = 3 + 1*e^{0-ln2} = 3.5, W = -1 + 2*0.5 = 0
    a = (0.0, 1.0, np.array([2.0]))
    b = (math.log(2.0), 3.0, np.array([-1.0]))
    for merge in (oracle.merge_case, oracle.merge_unsum):
        for x, y in ((a, b), (b, a)):
            m, S, W = merge(x, y)
            assert abs(m - math.log(2.0)) < 1e-15 and abs(S - 3.5) < 1e-14 and abs(W[0]) < 1e-14


def test_associativity_and_closure():
    e = oracle.identity(4)
    for s in range(60):
        a, b, c = _state(3 * s, 4), _state(3 * s + 1, 4), _state(3 * s + 2, 4)
        if s % 7 == 0:
            b = e
        if s % 11 == 0:
            c = (a[0], c[1], c[2])                       # equal maxima
        l = oracle.merge_case(oracle.merge_case(a, b), c)
        r = oracle.merge_case(a, oracle.merge_case(b, c))
        _same(l, r)
        assert l[1] >= 0.0 and np.all(np.isfinite(l[2]))


def test_merge_factors_never_exceed_one():
    # Lemma 1: with max re-anchoring every scaling exponent is <= 0, so S of a merge of unit states <= count
    states = [(float(m), 1.0, np.array([1.0])) for m in (3.0, -2.0, 700.0, 0.5, -900.0)]
    acc = oracle.identity(1)
    for u in states:
        acc = oracle.merge_case(acc, u)
        assert acc[1] <= len(states) and np.isfinite(acc[1])
    assert acc[0] == 700.0 and abs(acc[1] - 1.0) < 1e-12


# ---- Prop. 1: block composition and merge trees ---------------------------------------------

def _problem(n=300, d=8, seed=5):
    cnt = n * d
    q = inputs.normal(seed, 0, 0, cnt).reshape(1, 1, n, d)
    k = inputs.normal(seed, 1, 0, cnt).reshape(1, 1, n, d)
    v = inputs.normal(seed, 2, 0, cnt).reshape(1, 1, n, d)
    return q, k, v


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("C", [1, 2, 3, 7, 300])
def test_partials_combine_to_single_pass(C, causal):
    q, k, v = _problem()
    ref = oracle.attn_rows(q, k, v, 0.35, causal=causal)
    pm, pS, pW = oracle.partials_rows(q, k, v, 0.35, C, causal=causal)
    out = oracle.combine_rows(pm, pS, pW)
    assert np.all(np.abs(out - ref) <= 1e-13 * (1 + np.abs(ref)))
    if causal and C > 1:
        assert np.isneginf(pm[0, 1]) and pS[0, 1] == 0 and np.all(pW[0, 1] == 0)  # masked chunk = identity


def test_block_128_composition_and_two_level_scan():
    # per-key unit states u_j = (s_j, 1, v_j); blocks of 128 reduced by (+) equal the global result,
    # and the two-level scan's prefixes equal the causal outputs.
    n, d = 300, 8
    q, k, v = _problem(n, d)
    scale, i = 0.35, 123
    s = scale * (k[0, 0].astype(np.float64) @ q[0, 0, i].astype(np.float64))
    units = [(float(s[j]), 1.0, v[0, 0, j].astype(np.float64)) for j in range(n)]
    ref = oracle.attn_rows(q, k, v, scale, rows=np.array([i]))[0]
    blocks = [units[a:a + 128] for a in range(0, n, 128)]
    tot = oracle.identity(d)
    for b in blocks:
        bt = oracle.identity(d)
        for u in b:
            bt = oracle.merge_case(bt, u)
        tot = oracle.merge_case(tot, bt)
    assert np.all(np.abs(tot[2] / tot[1] - ref) <= 1e-13 * (1 + np.abs(ref)))
    # chunk states from the C routine agree (in canonical form) with the unit-state reduction
    pm, pS, pW = oracle.partials_rows(q, k, v, scale, 3, rows=np.array([i]))
    bt = oracle.identity(d)
    for u in units[:100]:
        bt = oracle.merge_case(bt, u)
    l0, y0 = _canon(bt)
    l1, y1 = _canon((pm[0, 0], pS[0, 0], pW[0, 0]))
    assert abs(l0 - l1) < 1e-12 and np.all(np.abs(y0 - y1) < 1e-12)
    assert abs(pm[0, 0] - max(s[:100])) < 1e-14          # the chunk maximum itself, natural-log units
    # full two-level scan: prefix j of the scan for query row j's own scores is the causal output
    pref, total = scan.two_level_scan(units, oracle.merge_case, oracle.identity(d), block=128)
    assert np.all(np.abs(total[2] / total[1] - ref) <= 1e-13 * (1 + np.abs(ref)))
    seq = scan.sequential_scan(units, oracle.merge_case, oracle.identity(d))
    for j in (0, 1, 127, 128, 129, 255, 256, 299):
        a, b = _canon(pref[j]), _canon(seq[j])
        assert abs(a[0] - b[0]) < 1e-12 and np.all(np.abs(a[1] - b[1]) < 1e-12)


def test_random_merge_trees_agree():
    n, d = 64, 4
    q, k, v = _problem(n, d, seed=9)
    s = 0.5 * (k[0, 0].astype(np.float64) @ q[0, 0, 0].astype(np.float64))
    ref = oracle.attn_rows(q, k, v, 0.5, rows=np.array([0]))[0]
    for t in range(8):
        nodes = [(float(s[j]), 1.0, v[0, 0, j].astype(np.float64)) for j in range(n)]
        picks = inputs.uniform01(100 + t, 0, 0, n)
        step = 0
        while len(nodes) > 1:                             # merge a random adjacent pair (keeps key order)
            p = int(picks[step % n] * (len(nodes) - 1))
            nodes[p:p + 2] = [oracle.merge_case(nodes[p], nodes[p + 1])]
            step += 1
        m, S, W = nodes[0]
        assert np.all(np.abs(W / S - ref) <= 1e-13 * (1 + np.abs(ref)))
