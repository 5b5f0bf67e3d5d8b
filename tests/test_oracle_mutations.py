"""Do the pins bite?  Plant one plausible mistake at a time in a COPY of the oracle's C source
(dropped scale, wrong sign, off-by-one mask, ignored padding, misindexed values, dropped rescale,
wrong chunk bound, missing normalisation, ...), build it, run the battery of pins against it and
require that the battery fails.  The battery passes on the untouched oracle.  CPU only."""
import math
import os
import subprocess
import tempfile

import numpy as np
import pytest
import torch

import oracle
from paper_2604_23798_amd import inputs

SRC = os.path.join(os.path.dirname(oracle.__file__), "elsa_oracle.c")


def _rand(B, H, n, d, seed):
    cnt, sh = B * H * n * d, (B, H, n, d)
    return (inputs.normal(seed, 0, 0, cnt).reshape(sh), inputs.normal(seed, 1, 0, cnt).reshape(sh),
            inputs.normal(seed, 2, 0, cnt).reshape(sh))


def _close(a, b, tol=1e-11):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    assert a.shape == b.shape and np.all(np.abs(a - b) <= tol * (1.0 + np.abs(b)))


def battery():
    """A condensed run of the pins: closed forms, the library softmax, masks, states, merges."""
    # two keys by hand: y = sigma(s1 - s2) v1 + sigma(s2 - s1) v2
    q = np.array([[[[1.0, -2.0], [0.5, 0.25]]]], np.float32)
    k = np.array([[[[3.0, 1.0], [-1.0, 2.0]]]], np.float32)
    v = np.array([[[[10.0, -4.0], [2.0, 8.0]]]], np.float32)
    exp = []
    for s1, s2 in ((0.7, -3.5), (1.225, 0.0)):
        w1 = 1.0 / (1.0 + math.exp(s2 - s1))
        exp.append([w1 * 10.0 + (1 - w1) * 2.0, w1 * -4.0 + (1 - w1) * 8.0])
    _close(oracle.attn_rows(q, k, v, 0.7), np.array(exp))
    _close(oracle.fold_rows(q, k, v, 0.7), np.array(exp))
    _close(oracle.attn_rows(q, k, v, 0.7, causal=True)[0], [10.0, -4.0])
    # library float64 softmax, causal and padded
    B, H, n, d = 2, 2, 37, 8
    q, k, v = _rand(B, H, n, d, 7)
    tq, tk, tv = (torch.from_numpy(t).double() for t in (q, k, v))
    s = (tq @ tk.transpose(-1, -2)) * 0.3
    _close(oracle.attn_rows(q, k, v, 0.3), (torch.softmax(s, -1) @ tv).numpy().reshape(-1, d))
    sc = s.masked_fill(torch.ones(n, n).triu(1).bool(), float("-inf"))
    refc = (torch.softmax(sc, -1) @ tv).numpy().reshape(-1, d)
    _close(oracle.attn_rows(q, k, v, 0.3, causal=True), refc)
    _close(oracle.fold_rows(q, k, v, 0.3, causal=True), refc)
    kv_len = np.array([37, 11], np.int32)
    mask = (torch.arange(n)[None, :] < torch.from_numpy(kv_len)[:, None])[:, None, None, :]
    refp = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=0.3)
    _close(oracle.attn_rows(q, k, v, 0.3, kv_len=kv_len), refp.numpy().reshape(-1, d))
    _close(oracle.lse_rows(q, k, 0.3).reshape(B, H, n), torch.logsumexp(s, -1).numpy())
    # states of Prop. 1: the chunk maximum, identity chunks, and their merge
    pm, pS, pW = oracle.partials_rows(q, k, v, 0.3, 3, causal=True)
    sfull = s.numpy().reshape(-1, n)
    assert abs(pm[n - 1, 0] - sfull[n - 1, :13].max()) < 1e-12 and abs(pm[n - 1, 1] - sfull[n - 1, 13:26].max()) < 1e-12
    assert np.isneginf(pm[0, 1]) and pS[0, 1] == 0
    _close(oracle.combine_rows(pm, pS, pW), refc)
    a = (0.0, 1.0, np.array([2.0]))
    b = (math.log(2.0), 3.0, np.array([-1.0]))
    for x, y in ((a, b), (b, a)):
        for merge in (oracle.merge_case, oracle.merge_unsum):
            m, S, W = merge(x, y)
            assert abs(m - math.log(2.0)) < 1e-15 and abs(S - 3.5) < 1e-14 and abs(W[0]) < 1e-14
    # rectangular attention against the library softmax, both aspect ratios, causal and padded
    for nq, nk in ((5, 23), (23, 5)):
        qq = inputs.normal(9, 0, 0, 2 * 2 * nq * 8).reshape(2, 2, nq, 8)
        kk = inputs.normal(9, 1, 0, 2 * 2 * nk * 8).reshape(2, 2, nk, 8)
        vv = inputs.normal(9, 2, 0, 2 * 2 * nk * 8).reshape(2, 2, nk, 8)
        a, b_, c = (torch.from_numpy(x).double() for x in (qq, kk, vv))
        sx = (a @ b_.transpose(-1, -2)) * 0.4
        o, l = oracle.cross_rows(qq, kk, vv, 0.4)
        _close(o, (torch.softmax(sx, -1) @ c).numpy().reshape(-1, 8))
        _close(l, torch.logsumexp(sx, -1).numpy().reshape(-1))
        i, j = torch.arange(nq)[:, None], torch.arange(nk)[None, :]
        sm = sx.masked_fill(j > i + (nk - nq), float("-inf"))
        o, _ = oracle.cross_rows(qq, kk, vv, 0.4, causal=True)
        _close(o, (torch.nan_to_num(torch.softmax(sm, -1), nan=0.0) @ c).numpy().reshape(-1, 8))
        kl = np.array([nk, 3], np.int32)
        sp = sx.masked_fill((j >= torch.from_numpy(kl).long()[:, None, None, None]), float("-inf"))
        o, _ = oracle.cross_rows(qq, kk, vv, 0.4, kv_len=kl)
        _close(o, (torch.softmax(sp, -1) @ c).numpy().reshape(-1, 8))
    # values of their own width: library softmax, both masks, and the log-normaliser
    for nq, nk, dd, dv in ((23, 5, 4, 16), (5, 23, 8, 3)):      # the first case keeps every planted index inside v
        qq = inputs.normal(13, 0, 0, 2 * 2 * nq * dd).reshape(2, 2, nq, dd)
        kk = inputs.normal(13, 1, 0, 2 * 2 * nk * dd).reshape(2, 2, nk, dd)
        vv = inputs.normal(13, 2, 0, 2 * 2 * nk * dv).reshape(2, 2, nk, dv)
        a, b_, c = (torch.from_numpy(x).double() for x in (qq, kk, vv))
        sx = (a @ b_.transpose(-1, -2)) * 0.4
        o, l = oracle.dv_rows(qq, kk, vv, 0.4)
        _close(o, (torch.softmax(sx, -1) @ c).numpy().reshape(-1, dv))
        _close(l, torch.logsumexp(sx, -1).numpy().reshape(-1))
        i, j = torch.arange(nq)[:, None], torch.arange(nk)[None, :]
        sm = sx.masked_fill(j > i + (nk - nq), float("-inf"))
        o, _ = oracle.dv_rows(qq, kk, vv, 0.4, causal=True)
        _close(o, (torch.nan_to_num(torch.softmax(sm, -1), nan=0.0) @ c).numpy().reshape(-1, dv))
        kl = np.array([nk, 3], np.int32)
        sp = sx.masked_fill((j >= torch.from_numpy(kl).long()[:, None, None, None]), float("-inf"))
        o, _ = oracle.dv_rows(qq, kk, vv, 0.4, kv_len=kl)
        _close(o, (torch.softmax(sp, -1) @ c).numpy().reshape(-1, dv))
    lad = oracle.ladder_f32_fold_rows(q, k, v, 0.3).astype(np.float64)
    ref = oracle.attn_rows(q, k, v, 0.3)
    assert np.max(np.linalg.norm(lad - ref, axis=1) / np.linalg.norm(ref, axis=1)) < 1e-5
    # binary16 rounding against the library cast; the half-precision ladder on equal weights (q = 0)
    xs = [1.0 / 3.0, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -25, 1.5 * 2.0 ** -24, 70000.0, -0.1, 2051.0, 3e-6]
    with np.errstate(over="ignore"):
        assert [oracle.round_f16(x) for x in xs] == [float(np.float16(x)) for x in xs]
    l16 = oracle.ladder_f16_rows(np.zeros_like(q), k, v, 0.3)
    assert np.array_equal(l16.reshape(B, H, n, d)[:, :, 3], v.astype(np.float64).mean(axis=2).astype(np.float16).astype(np.float64))
    l16 = oracle.ladder_f16_rows(q, k, v, 0.3)
    assert np.max(np.linalg.norm(l16 - ref, axis=1) / np.linalg.norm(ref, axis=1)) < 2.0 ** -10
    mean_err = lambda a: float(np.mean(np.linalg.norm(a - ref, axis=1) / np.linalg.norm(ref, axis=1)))
    assert 1.2 < mean_err(l16) / mean_err(ref.astype(np.float16).astype(np.float64)) < 1.7      # rounded weights add their share


MUTATIONS = [
    ("dropped scale", "return scale * acc;", "return acc;"),
    ("wrong sign in the exponent", "double e = exp(s[j] - m);", "double e = exp(m - s[j]);"),
    ("causal mask off by one", "if (causal && i + 1 < lim) lim = i + 1;", "if (causal && i < lim) lim = i;"),
    ("padding ignored", "int64_t lim = kv_len ? (int64_t)kv_len[b] : n;", "int64_t lim = n;"),
    ("values read from the wrong key", "            const float *vj = vb + (size_t)j * d;\n            for (int t = 0; t < d; ++t) o[t] += e",
     "            const float *vj = vb + (size_t)(L - 1 - j) * d;\n            for (int t = 0; t < d; ++t) o[t] += e"),
    ("fold: running maximum not carried", "m_run = m_next; S_run = S_next;", "S_run = S_next;"),
    ("fold: key lifted with weight 0", "d, scale), 1.0, Wkey, d,", "d, scale), 0.0, Wkey, d,"),
    ("fold: key lifted with the wrong value row", "Wkey[t] = (double)vals[(size_t)j * d + t];", "Wkey[t] = (double)vals[(size_t)i * d + t];"),
    ("merge: past not rescaled when the maximum moves", "*mo = mb; *So = Sb + Sa * f;", "*mo = mb; *So = Sb + Sa;"),
    ("merge: factor inverted", "double f = exp(mb - ma);", "double f = exp(ma - mb);"),
    ("merge: un-sum without renorm", "*So = (Sa * ea + Sb * eb) * em;", "*So = (Sa * ea + Sb * eb);"),
    ("chunk bound shifted", "int64_t lo = (int64_t)c * chunk, hi = lo + chunk;", "int64_t lo = (int64_t)c * chunk + 1, hi = lo + chunk;"),
    ("chunk maximum not recorded", "part_m[(size_t)r * C + c] = m;", "part_m[(size_t)r * C + c] = 0.0;"),
    ("combine without normalisation", "out[(size_t)r * d + t] = (S > 0.0) ? Wa[t] / S : 0.0;", "out[(size_t)r * d + t] = Wa[t];"),
    ("log-normaliser without its maximum", "lse[r] = (L > 0) ? m + log(S) : -INFINITY;", "lse[r] = (L > 0) ? log(S) : -INFINITY;"),
    ("transposed operand in the score", "acc += (double)qi[t] * (double)kj[t];", "acc += (double)qi[t] * (double)kj[d - 1 - t];"),
    ("rectangular: diagonal aligned with the first key", "int64_t last = i + ((int64_t)nk - (int64_t)nq);", "int64_t last = i;"),
    ("rectangular: diagonal shifted the wrong way", "int64_t last = i + ((int64_t)nk - (int64_t)nq);", "int64_t last = i + ((int64_t)nq - (int64_t)nk);"),
    ("rectangular: keys strided by the query count", "const float *kb = k + (size_t)bh * nk * d;", "const float *kb = k + (size_t)bh * nq * d;"),
    ("rectangular: padding ignored", "int64_t L = kv_len ? (int64_t)kv_len[b] : nk;", "int64_t L = nk;"),
    ("rectangular: log-normaliser without its maximum", "if (lse) lse[r] = m + log(S);", "if (lse) lse[r] = log(S);"),
    ("own value width: values strided by the key width", "const float *vals = v + (size_t)bh * nk * dv;", "const float *vals = v + (size_t)bh * nk * d;"),
    ("own value width: value rows strided by the key width", "acc += w[j] * (double)vals[(size_t)j * dv + c];", "acc += w[j] * (double)vals[(size_t)j * d + c];"),
    ("own value width: not normalised", "y[c] = acc / Z;", "y[c] = acc;"),
    ("own value width: diagonal off by one", "int64_t diag = i + ((int64_t)nk - (int64_t)nq) + 1;", "int64_t diag = i + ((int64_t)nk - (int64_t)nq);"),
    ("own value width: padding ignored", "int64_t vis = kv_len ? (int64_t)kv_len[b] : nk;", "int64_t vis = nk;"),
    ("own value width: weights without their maximum in the log-normaliser", "if (lse) lse[r] = top + log(Z);", "if (lse) lse[r] = log(Z);"),
    ("half rounding: ties away from even", "nearbyint(ldexp(x, -ulp_exp))", "floor(ldexp(x, -ulp_exp) + 0.5)"),
    ("half rounding: no gradual underflow", "if (ulp_exp < -24) ulp_exp = -24;", ""),
    ("half-precision ladder: weights not rounded", "double wh = elsa_oracle_round_f16(w);", "double wh = w;"),
    ("half-precision ladder: output not rounded", "y[t] = elsa_oracle_round_f16(y[t] / Z);", "y[t] = y[t] / Z;"),
    ("single-precision ladder: past not rescaled", "*S = f32_add(Sk, f32_mul(*S, f));", "*S = f32_add(Sk, *S);"),
]


def _build(src_text, tmpdir, name):
    c = os.path.join(tmpdir, name + ".c")
    so = os.path.join(tmpdir, name + ".so")
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off", "-o", so, c, "-lm"])
    return so


@pytest.fixture()
def swap_oracle_lib():
    good = oracle._load()
    yield
    oracle._lib = good


def test_battery_passes_on_the_real_oracle():
    battery()


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(what, old, new, swap_oracle_lib):
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation target not found: " + what
    with tempfile.TemporaryDirectory() as tmp:
        so = _build(text.replace(old, new, 1), tmp, "mutant")
        oracle._lib = None
        real_build = oracle.build
        oracle.build = lambda force=False: so
        try:
            oracle._load()                      # binds argtypes on the mutant
        finally:
            oracle.build = real_build
        with pytest.raises(AssertionError):
            battery()
