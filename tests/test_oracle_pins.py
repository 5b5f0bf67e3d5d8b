"""Pins of the FP64 oracle against things other than itself.

Each test is chosen so that a plausible mistake in the oracle (dropped scale,
wrong sign in the exponent, transposed operand, wrong mask edge, wrong chunk
bounds) fails at least one of them.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2604_23798_amd import inputs

RT = 1e-13  # FP64 agreement level between two exact formulations


def _rand(B, H, n, d, seed, sigma=1.0):
    cnt = B * H * n * d
    sh = (B, H, n, d)
    return (inputs.normal(seed, 0, 0, cnt, sigma).reshape(sh),
            inputs.normal(seed, 1, 0, cnt, sigma).reshape(sh),
            inputs.normal(seed, 2, 0, cnt).reshape(sh))


def _close(a, b, tol=RT):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    assert a.shape == b.shape
    assert np.all(np.abs(a - b) <= tol * (1.0 + np.abs(b))), float(np.max(np.abs(a - b)))


# ---- hand-computed closed forms -------------------------------------------------------------

def test_single_key_returns_value():
    q, k, v = _rand(1, 2, 1, 4, 11)
    _close(oracle.attn_rows(q, k, v, 0.5), v.reshape(2, 4))
    _close(oracle.fold_rows(q, k, v, 0.5), v.reshape(2, 4))


def test_two_keys_sigmoid_mixture():
    # n = 2: y = sigma(s1 - s2) v1 + sigma(s2 - s1) v2 with s_j = scale <q, k_j>, typed by hand.
    q = np.array([[[[1.0, -2.0], [0.5, 0.25]]]], np.float32)      # [1,1,2,2]
    k = np.array([[[[3.0, 1.0], [-1.0, 2.0]]]], np.float32)
    v = np.array([[[[10.0, -4.0], [2.0, 8.0]]]], np.float32)
    scale = 0.7
    # row 0: q=(1,-2): s1 = .7*(3-2) = .7 ; s2 = .7*(-1-4) = -3.5
    # row 1: q=(.5,.25): s1 = .7*(1.5+.25) = 1.225 ; s2 = .7*(-.5+.5) = 0
    exp = []
    for s1, s2 in ((0.7, -3.5), (1.225, 0.0)):
        w1 = 1.0 / (1.0 + math.exp(s2 - s1))
        exp.append([w1 * 10.0 + (1 - w1) * 2.0, w1 * -4.0 + (1 - w1) * 8.0])
    _close(oracle.attn_rows(q, k, v, scale), np.array(exp))
    _close(oracle.fold_rows(q, k, v, scale), np.array(exp))
    # causal: row 0 sees only key 0
    out = oracle.attn_rows(q, k, v, scale, causal=True)
    _close(out[0], [10.0, -4.0])
    _close(out[1], exp[1])


def test_three_keys_brute_force_unshifted():
    # Eq. 1 literally, without max subtraction, in Python floats.
    q, k, v = _rand(1, 1, 3, 2, 5)
    scale = 1.0 / math.sqrt(2)
    out = oracle.attn_rows(q, k, v, scale)
    for i in range(3):
        s = [scale * sum(float(q[0, 0, i, t]) * float(k[0, 0, j, t]) for t in range(2)) for j in range(3)]
        den = sum(math.exp(x) for x in s)
        y = [sum(math.exp(s[j]) * float(v[0, 0, j, t]) for j in range(3)) / den for t in range(2)]
        _close(out[i], y)


def test_zero_query_gives_column_mean():
    q, k, v = _rand(2, 2, 37, 8, 3)
    q[:] = 0
    out = oracle.attn_rows(q, k, v, 0.3).reshape(2, 2, 37, 8)
    mean = v.astype(np.float64).mean(axis=2, keepdims=True)
    _close(out, np.broadcast_to(mean, out.shape))
    # causal: row i = mean of v[0..i]
    outc = oracle.attn_rows(q, k, v, 0.3, causal=True).reshape(2, 2, 37, 8)
    cm = np.cumsum(v.astype(np.float64), axis=2) / np.arange(1, 38).reshape(1, 1, 37, 1)
    _close(outc, cm)


# ---- library routine as a black box ---------------------------------------------------------

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 2, 33, 8), (2, 3, 130, 16), (1, 1, 257, 64)])
def test_against_torch_float64_softmax(shape, causal):
    B, H, n, d = shape
    q, k, v = _rand(B, H, n, d, 17 + n)
    scale = 1.0 / math.sqrt(d)
    tq, tk, tv = (torch.from_numpy(t).double() for t in (q, k, v))
    s = (tq @ tk.transpose(-1, -2)) * scale
    if causal:
        s = s.masked_fill(torch.ones(n, n).triu(1).bool(), float("-inf"))
    ref = (torch.softmax(s, dim=-1) @ tv).numpy().reshape(-1, d)
    _close(oracle.attn_rows(q, k, v, scale, causal=causal), ref, 1e-12)
    _close(oracle.fold_rows(q, k, v, scale, causal=causal), ref, 1e-12)


def test_against_torch_sdpa_with_key_padding():
    B, H, n, d = 3, 2, 50, 16
    q, k, v = _rand(B, H, n, d, 23)
    kv_len = np.array([50, 1, 29], np.int32)
    scale = 0.25
    tq, tk, tv = (torch.from_numpy(t).double() for t in (q, k, v))
    mask = (torch.arange(n)[None, :] < torch.from_numpy(kv_len)[:, None])[:, None, None, :]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    _close(oracle.attn_rows(q, k, v, scale, kv_len=kv_len), ref.numpy().reshape(-1, d), 1e-12)
    # kv_len = 1 => every row of that batch returns v_0 (padded query rows are still computed)
    out = oracle.attn_rows(q, k, v, scale, kv_len=kv_len).reshape(B, H, n, d)
    _close(out[1], np.broadcast_to(v[1, :, :1, :].astype(np.float64), (H, n, d)))
    # kv_len = n equals no mask
    _close(oracle.attn_rows(q, k, v, scale, kv_len=np.full(B, n, np.int32)), oracle.attn_rows(q, k, v, scale))


# ---- invariants ------------------------------------------------------------------------------

def test_fold_equals_definition():
    q, k, v = _rand(1, 2, 300, 32, 41)
    for causal in (False, True):
        _close(oracle.fold_rows(q, k, v, 0.2, causal=causal), oracle.attn_rows(q, k, v, 0.2, causal=causal))


def test_causal_row_equals_prefix_problem():
    q, k, v = _rand(1, 1, 40, 8, 9)
    full = oracle.attn_rows(q, k, v, 0.4, causal=True)
    _close(full[0], v[0, 0, 0])                       # the first row sees only itself
    for i in (0, 1, 7, 39):
        # non-causal problem restricted to keys 0..i, evaluated for query i
        qq = np.repeat(q[:, :, i:i + 1], i + 1, axis=2)
        ref = oracle.attn_rows(qq, k[:, :, :i + 1], v[:, :, :i + 1], 0.4)[0]
        _close(full[i], ref)


def test_shift_invariance_through_the_inputs():
    # Reserve coordinate 0: q[..., 0] = 1 and k[..., 0] += c / scale shifts every score by c.
    q, k, v = _rand(1, 2, 64, 8, 77)
    scale = 0.5
    q[..., 0] = 1.0
    k[..., 0] = np.round(k[..., 0] * 4) / 4          # keep k0 + c/scale exactly representable
    base = oracle.attn_rows(q, k, v, scale)
    for c in (-1000.0, 40.0, 10000.0):
        k2 = k.copy()
        k2[..., 0] += np.float32(c / scale)
        _close(oracle.attn_rows(q, k2, v, scale), base, 1e-10)
        _close(oracle.fold_rows(q, k2, v, scale), base, 1e-10)


def test_one_hot_when_one_score_dominates():
    B, H, n, d = 1, 1, 50, 8
    q, k, v = _rand(B, H, n, d, 31)
    j = 17
    k[0, 0, j] = q[0, 0, 3] * 60.0                    # score gap of hundreds for query 3
    out = oracle.attn_rows(q, k, v, 1.0, rows=np.array([3]))
    _close(out[0], v[0, 0, j], 1e-15)


def test_key_permutation_invariance():
    q, k, v = _rand(1, 2, 90, 16, 55)
    perm = np.argsort(inputs.uniform01(3, 0, 0, 90))
    _close(oracle.attn_rows(q, k[:, :, perm], v[:, :, perm], 0.25), oracle.attn_rows(q, k, v, 0.25), 1e-12)


def test_no_visible_key_outputs_zero():
    q, k, v = _rand(2, 1, 5, 4, 2)
    out = oracle.attn_rows(q, k, v, 1.0, kv_len=np.array([0, 5], np.int32)).reshape(2, 5, 4)
    assert np.all(out[0] == 0.0) and np.all(np.isfinite(out))
    assert np.all(oracle.fold_rows(q, k, v, 1.0, kv_len=np.array([0, 5], np.int32)).reshape(2, 5, 4)[0] == 0)


def test_wide_scores_stay_finite():
    # config-5-like: scores with sigma ~ 64; every exponent argument is <= 0 so nothing overflows.
    q, k, v = _rand(1, 1, 512, 64, 99, sigma=8.0)
    out = oracle.attn_rows(q, k, v, 0.125)
    assert np.all(np.isfinite(out))
    _close(oracle.fold_rows(q, k, v, 0.125), out, 1e-12)


def test_row_subset_matches_full():
    q, k, v = _rand(2, 2, 31, 8, 8)
    full = oracle.attn_rows(q, k, v, 0.3, causal=True)
    rows = np.array([0, 5, 30, 31, 61, 123], np.int64)
    assert np.array_equal(oracle.attn_rows(q, k, v, 0.3, causal=True, rows=rows), full[rows])


def test_ladder_f32_is_close_but_not_exact():
    q, k, v = _rand(1, 1, 256, 64, 4)
    ref = oracle.attn_rows(q, k, v, 0.125)
    lad = oracle.ladder_f32_fold_rows(q, k, v, 0.125).astype(np.float64)
    err = np.linalg.norm(lad - ref, axis=1) / np.linalg.norm(ref, axis=1)
    assert 0 < err.max() < 1e-5


def test_round_to_binary16_against_the_library_cast():
    """The oracle's own rounding to IEEE half against numpy's float16 cast (a black box): random values over
    the whole exponent range, exact ties (to even), the denormal range, the overflow threshold."""
    rng = np.random.default_rng(5)
    xs = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-9, 5, 2000),
                         [0.0, 1.0, -1.0, 65504.0, 65519.99, 65520.0, -65520.0, 1e-8, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -24,
                          2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -30,
                          1.0 / 3.0, 0.1, 2049.0, 2051.0, 4098.0]])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).astype(np.float64)
    got = np.array([oracle.round_f16(x) for x in xs])
    assert np.array_equal(got, want), [(x, g, w) for x, g, w in zip(xs, got, want) if g != w][:5]


def test_ladder_f16_rounds_the_weights_and_the_output_and_nothing_else():
    # one key: the value row itself, rounded to half
    q, k, v = _rand(1, 1, 1, 8, 41)
    assert np.array_equal(oracle.ladder_f16_rows(q, k, v, 0.3)[0], v[0, 0, 0].astype(np.float16).astype(np.float64))
    # q = 0: every weight is exactly 1 (representable), so only the output is rounded: half(column mean)
    q, k, v = _rand(1, 2, 37, 8, 42)
    q[:] = 0
    mean = v.astype(np.float64).mean(axis=2)                                       # [1, 2, 8]
    got = oracle.ladder_f16_rows(q, k, v, 0.3).reshape(1, 2, 37, 8)
    assert np.array_equal(got[0, :, 5], mean[0].astype(np.float16).astype(np.float64))
    # two keys, s1 - s2 = ln 3 by construction: weights 1 and 1/3; half(1/3) = 1365 / 4096 multiplies v2,
    # the normaliser keeps 1 + 1/3
    q = np.array([[[[1.0]]]], np.float32).repeat(2, axis=2)
    k = np.array([[[[2.0], [0.0]]]], np.float32)
    v = np.array([[[[3.0], [2.0]]]], np.float32)
    scale = float(np.log(3.0) / 2.0)
    got = oracle.ladder_f16_rows(q, k, v, scale)[0, 0]
    exact = oracle.attn_rows(q, k, v, scale)[0, 0]
    w = np.exp(0.0 - 2.0 * scale)                                                  # 1/3 up to the rounding of scale
    want = float(np.float16((3.0 + float(np.float16(w)) * 2.0) / (1.0 + w)))
    assert got == want and abs(got - exact) < 2e-3
    # in general: within half-precision roundoff of the definition, row by row
    q, k, v = _rand(2, 2, 300, 32, 43)
    for causal in (False, True):
        ref = oracle.attn_rows(q, k, v, 0.2, causal=causal)
        lad = oracle.ladder_f16_rows(q, k, v, 0.2, causal=causal)
        err = np.linalg.norm(lad - ref, axis=1) / np.linalg.norm(ref, axis=1)
        assert 0 < err.max() < 2.0 ** -10
        assert np.array_equal(lad, lad.astype(np.float16).astype(np.float64))        # outputs are halves
        # error model: rounding the output alone leaves a row error of about 0.7 * 2^-11 / sqrt(3); the rounded
        # weights add an independent error of about the same size, so the ladder sits a factor ~1.4 above it
        only_out = ref.astype(np.float16).astype(np.float64)
        mean_err = lambda a: float(np.mean(np.linalg.norm(a - ref, axis=1) / np.linalg.norm(ref, axis=1)))
        assert 1.2 < mean_err(lad) / mean_err(only_out) < 1.7


def test_varlen_reduces_to_dense_problems():
    # equal-length packed sequences are a dense batch in another layout; unequal ones are independent
    B, H, n, d = 3, 2, 17, 8
    q, k, v = _rand(B, H, n, d, 61)
    pk = lambda t: np.ascontiguousarray(t.transpose(0, 2, 1, 3)).reshape(B * n, H, d)      # [B,n,H,d] packed
    cu = np.arange(B + 1) * n
    for causal in (False, True):
        dense = oracle.attn_rows(q, k, v, 0.3, causal=causal).reshape(B, H, n, d)
        _close(oracle.attn_varlen(pk(q), pk(k), pk(v), cu, 0.3, causal=causal).reshape(B, n, H, d),
               dense.transpose(0, 2, 1, 3))
    q2, k2, v2, cu2 = inputs.make_varlen(5, lengths=[4, 0, 1, 9], H=2, d=8)
    out = oracle.attn_varlen(q2, k2, v2, cu2, 0.5)
    _close(out[4], v2[4])                                    # the one-token sequence returns its value
    _close(out[5:], oracle.attn_varlen(q2[5:], k2[5:], v2[5:], [0, 9], 0.5))
    _close(out[:4], oracle.attn_varlen(q2[:4], k2[:4], v2[:4], [0, 4], 0.5))


def test_lse_closed_forms_and_library():
    q, k, v = _rand(2, 2, 40, 8, 71)
    lse = oracle.lse_rows(q, k, 0.3).reshape(2, 2, 40)
    s = torch.from_numpy(q).double() @ torch.from_numpy(k).double().transpose(-1, -2) * 0.3
    _close(lse, torch.logsumexp(s, dim=-1).numpy(), 1e-12)
    m = torch.ones(40, 40).triu(1).bool()
    _close(oracle.lse_rows(q, k, 0.3, causal=True).reshape(2, 2, 40),
           torch.logsumexp(s.masked_fill(m, float("-inf")), dim=-1).numpy(), 1e-12)
    q0 = np.zeros_like(q)
    _close(oracle.lse_rows(q0, k, 0.3), np.full(2 * 2 * 40, math.log(40.0)))      # uniform scores: ln n
    _close(oracle.lse_rows(q, k, 0.3, causal=True).reshape(2, 2, 40)[..., 0],
           0.3 * np.einsum("bhd,bhd->bh", q[:, :, 0].astype(np.float64), k[:, :, 0].astype(np.float64)))  # n = 1: s itself
    assert np.all(np.isneginf(oracle.lse_rows(q, k, 0.3, kv_len=np.array([0, 40], np.int32)).reshape(2, 80)[0]))
    # consistency with the state form: lse = m_c + ln S_c for a single chunk
    pm, pS, _ = oracle.partials_rows(q, k, v, 0.3, 1)
    _close(oracle.lse_rows(q, k, 0.3), pm[:, 0] + np.log(pS[:, 0]), 1e-12)


# ---- rectangular attention (n_q != n_k): cross-attention, chunked prefill, decoding -----------
def _rect(B, H, nq, nk, d, seed):
    q = inputs.normal(seed, 0, 0, B * H * nq * d).reshape(B, H, nq, d)
    k = inputs.normal(seed, 1, 0, B * H * nk * d).reshape(B, H, nk, d)
    v = inputs.normal(seed, 2, 0, B * H * nk * d).reshape(B, H, nk, d)
    return q, k, v


def test_cross_single_query_two_keys_by_hand():
    q = np.array([[[[2.0, 1.0]]]], np.float32)
    k = np.array([[[[1.0, 0.0], [0.0, 3.0]]]], np.float32)
    v = np.array([[[[4.0, -2.0], [-6.0, 10.0]]]], np.float32)
    s1, s2 = 0.5 * 2.0, 0.5 * 3.0
    w1 = 1.0 / (1.0 + math.exp(s2 - s1))
    out, lse = oracle.cross_rows(q, k, v, 0.5)
    _close(out[0], [w1 * 4.0 + (1 - w1) * -6.0, w1 * -2.0 + (1 - w1) * 10.0])
    _close(lse[0], math.log(math.exp(s1) + math.exp(s2)))
    # causal with one query and two keys: the query is the LAST position, so it sees both keys
    out_c, _ = oracle.cross_rows(q, k, v, 0.5, causal=True)
    _close(out_c, out)


@pytest.mark.parametrize("nq,nk", [(5, 23), (23, 5), (1, 40), (17, 17)])
@pytest.mark.parametrize("causal", [False, True])
def test_cross_against_library_softmax(nq, nk, causal):
    B, H, d = 2, 3, 8
    q, k, v = _rect(B, H, nq, nk, d, 31 + nq)
    tq, tk, tv = (torch.from_numpy(t).double() for t in (q, k, v))
    s = (tq @ tk.transpose(-1, -2)) * 0.4
    if causal:
        i = torch.arange(nq)[:, None]
        j = torch.arange(nk)[None, :]
        s = s.masked_fill(j > i + (nk - nq), float("-inf"))
    p = torch.softmax(s, -1)
    p = torch.nan_to_num(p, nan=0.0)                     # rows with no visible key
    out, lse = oracle.cross_rows(q, k, v, 0.4, causal=causal)
    _close(out, (p @ tv).numpy().reshape(-1, d))
    ref_lse = torch.logsumexp(s, -1).numpy().reshape(-1)
    vis = np.isfinite(ref_lse)
    _close(lse[vis], ref_lse[vis])
    assert np.all(np.isneginf(lse[~vis])) and np.all(out[~vis] == 0)
    if causal and nk < nq:
        assert (~vis).reshape(B * H, nq)[:, : nq - nk].all() and vis.reshape(B * H, nq)[:, nq - nk:].all()


def test_cross_square_case_is_the_square_routine():
    q, k, v = _rand(2, 2, 29, 8, 41)
    kv_len = np.array([29, 9], np.int32)
    for causal in (False, True):
        out, lse = oracle.cross_rows(q, k, v, 0.3, causal=causal, kv_len=kv_len)
        _close(out, oracle.attn_rows(q, k, v, 0.3, causal=causal, kv_len=kv_len))
        _close(lse, oracle.lse_rows(q, k, 0.3, causal=causal, kv_len=kv_len))


def test_cross_tail_queries_of_a_causal_problem():
    """Chunked prefill / decoding: the last n_q queries of a causal square problem, given alone."""
    B, H, n, d = 1, 2, 45, 8
    q, k, v = _rand(B, H, n, d, 43)
    full = oracle.attn_rows(q, k, v, 0.25, causal=True).reshape(B, H, n, d)
    for nq in (1, 7, 32):
        out, _ = oracle.cross_rows(q[:, :, n - nq:], k, v, 0.25, causal=True)
        _close(out.reshape(B, H, nq, d), full[:, :, n - nq:])


def test_cross_key_padding_and_row_subset():
    B, H, nq, nk, d = 2, 2, 6, 19, 4
    q, k, v = _rect(B, H, nq, nk, d, 47)
    kv_len = np.array([19, 4], np.int32)
    out, _ = oracle.cross_rows(q, k, v, 0.7, kv_len=kv_len)
    trunc, _ = oracle.cross_rows(q[1:], k[1:, :, :4], v[1:, :, :4], 0.7)
    _close(out.reshape(B, H * nq, d)[1], trunc)
    rows = np.array([3, 23, 0], np.int64)
    sub, _ = oracle.cross_rows(q, k, v, 0.7, kv_len=kv_len, rows=rows)
    _close(sub, out[rows])


# ---- values of their own width d_v != d (V in R^{n x d_v}, W in R^{d_v}) ---------------------------
def _rect_dv(B, H, nq, nk, d, dv, seed):
    q = inputs.normal(seed, 0, 0, B * H * nq * d).reshape(B, H, nq, d)
    k = inputs.normal(seed, 1, 0, B * H * nk * d).reshape(B, H, nk, d)
    v = inputs.normal(seed, 2, 0, B * H * nk * dv).reshape(B, H, nk, dv)
    return q, k, v


def test_dv_two_keys_three_value_columns_by_hand():
    q = np.array([[[[2.0, 1.0]]]], np.float32)
    k = np.array([[[[1.0, 0.0], [0.0, 3.0]]]], np.float32)
    v = np.array([[[[4.0, -2.0, 1.0], [-6.0, 10.0, 5.0]]]], np.float32)
    s1, s2 = 0.5 * 2.0, 0.5 * 3.0
    w1 = 1.0 / (1.0 + math.exp(s2 - s1))
    out, lse = oracle.dv_rows(q, k, v, 0.5)
    assert out.shape == (1, 3)
    _close(out[0], [w1 * 4.0 + (1 - w1) * -6.0, w1 * -2.0 + (1 - w1) * 10.0, w1 * 1.0 + (1 - w1) * 5.0])
    _close(lse[0], math.log(math.exp(s1) + math.exp(s2)))
    # one value column, d = 2: the output is the softmax-weighted mean of that column
    out1, _ = oracle.dv_rows(q, k, v[..., 2:], 0.5)
    _close(out1[0], [w1 * 1.0 + (1 - w1) * 5.0])


def test_dv_brute_force_in_python_floats():
    B, H, nq, nk, d, dv = 1, 2, 3, 5, 2, 3
    q, k, v = _rect_dv(B, H, nq, nk, d, dv, 61)
    for causal in (False, True):
        out, lse = oracle.dv_rows(q, k, v, 0.9, causal=causal)
        for h in range(H):
            for i in range(nq):
                vis = [j for j in range(nk) if not causal or j <= i + nk - nq]
                s = [0.9 * sum(float(q[0, h, i, t]) * float(k[0, h, j, t]) for t in range(d)) for j in vis]
                z = sum(math.exp(x) for x in s)
                for c in range(dv):
                    y = sum(math.exp(x) * float(v[0, h, j, c]) for x, j in zip(s, vis)) / z
                    assert abs(out[h * nq + i, c] - y) < 1e-12 * (1 + abs(y))
                assert abs(lse[h * nq + i] - math.log(z)) < 1e-12


@pytest.mark.parametrize("nq,nk,d,dv", [(5, 23, 8, 3), (23, 5, 4, 16), (1, 40, 16, 8), (17, 17, 8, 24)])
@pytest.mark.parametrize("causal", [False, True])
def test_dv_against_library_softmax(nq, nk, d, dv, causal):
    B, H = 2, 3
    q, k, v = _rect_dv(B, H, nq, nk, d, dv, 67 + nq)
    tq, tk, tv = (torch.from_numpy(t).double() for t in (q, k, v))
    s = (tq @ tk.transpose(-1, -2)) * 0.4
    if causal:
        i = torch.arange(nq)[:, None]
        j = torch.arange(nk)[None, :]
        s = s.masked_fill(j > i + (nk - nq), float("-inf"))
    p = torch.nan_to_num(torch.softmax(s, -1), nan=0.0)
    out, lse = oracle.dv_rows(q, k, v, 0.4, causal=causal)
    _close(out, (p @ tv).numpy().reshape(-1, dv))
    ref_lse = torch.logsumexp(s, -1).numpy().reshape(-1)
    vis = np.isfinite(ref_lse)
    _close(lse[vis], ref_lse[vis])
    assert np.all(np.isneginf(lse[~vis])) and np.all(out[~vis] == 0)


def test_dv_columns_are_independent_and_equal_width_is_the_rectangular_routine():
    """out(V = [V1 | V2]) = [out(V1) | out(V2)]: each block through the equal-width routine."""
    B, H, nq, nk, d = 2, 2, 9, 21, 8
    q, k, v = _rect_dv(B, H, nq, nk, d, 2 * d, 71)
    kv_len = np.array([21, 6], np.int32)
    for causal in (False, True):
        out, lse = oracle.dv_rows(q, k, v, 0.3, causal=causal, kv_len=kv_len)
        for blk in range(2):
            vb = np.ascontiguousarray(v[..., blk * d:(blk + 1) * d])
            ref, ref_lse = oracle.cross_rows(q, k, vb, 0.3, causal=causal, kv_len=kv_len)
            _close(out[:, blk * d:(blk + 1) * d], ref)
            _close(lse, ref_lse)
    # constant value rows come back unchanged whatever the scores are
    vc = np.broadcast_to(np.arange(5, dtype=np.float32), (B, H, nk, 5)).copy()
    out, _ = oracle.dv_rows(q, k, vc, 1.7)
    _close(out, np.broadcast_to(np.arange(5.0), out.shape))
    rows = np.array([7, 0, 30], np.int64)
    sub, _ = oracle.dv_rows(q, k, v, 0.3, kv_len=kv_len, rows=rows)
    _close(sub, oracle.dv_rows(q, k, v, 0.3, kv_len=kv_len)[0][rows])
