"""ELSA oracle -- TEST INFRASTRUCTURE, not a product path.

ctypes front end of ``elsa_oracle.c`` (plain single-threaded FP64 C).  Only
``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package.  It does not import, link or call the HIP library.

All tensors are numpy arrays, contiguous row-major ``[B, H, n, d]`` float32
(FP16 experiments pass FP16-representable float32 values).  A *row* is the flat
query index ``(b*H + h)*n + i``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "elsa_oracle.c")
_LIB = os.path.join(_HERE, "_elsa_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
             "-fno-fast-math", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lp = ctypes.POINTER(ctypes.c_int64)
        I, D, L = ctypes.c_int, ctypes.c_double, ctypes.c_int64
        rows_sig = [fp, fp, fp, I, I, I, I, D, I, ip, lp, L, dp]
        lib.elsa_oracle_attn_rows.argtypes = rows_sig
        lib.elsa_oracle_fold_rows.argtypes = rows_sig
        lib.elsa_oracle_lse_rows.argtypes = [fp, fp, I, I, I, I, D, I, ip, lp, L, dp]
        lib.elsa_oracle_partials_rows.argtypes = [fp, fp, fp, I, I, I, I, D, I, ip, I, lp, L, dp, dp, dp]
        mrg = [D, D, dp, D, D, dp, I, dp, dp, dp]
        lib.elsa_oracle_merge_case.argtypes = mrg
        lib.elsa_oracle_merge_case.restype = None
        lib.elsa_oracle_merge_unsum.argtypes = mrg
        lib.elsa_oracle_merge_unsum.restype = None
        lib.elsa_oracle_combine_rows.argtypes = [dp, dp, dp, L, I, I, dp]
        lib.elsa_oracle_cross_rows.argtypes = [fp, fp, fp, I, I, I, I, I, D, I, ip, lp, L, dp, dp]
        lib.elsa_oracle_dv_rows.argtypes = [fp, fp, fp, I, I, I, I, I, I, D, I, ip, lp, L, dp, dp]
        lib.elsa_ladder_f32_fold_rows.argtypes = [fp, fp, fp, I, I, I, I, ctypes.c_float, I, ip, lp, L, fp]
        lib.elsa_ladder_f16_rows.argtypes = rows_sig
        lib.elsa_oracle_round_f16.argtypes = [D]
        lib.elsa_oracle_round_f16.restype = D
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _prep(q, k, v, kv_len, rows):
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    assert q.ndim == 4 and q.shape == k.shape == v.shape, "expect [B,H,n,d] with d_v == d"
    B, H, n, d = q.shape
    if kv_len is None:
        kl, klp = None, None
    else:
        kl = np.ascontiguousarray(kv_len, dtype=np.int32)
        assert kl.shape == (B,)
        klp = kl.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    if rows is None:
        rows = np.arange(B * H * n, dtype=np.int64)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows.size == 0 or (rows.min() >= 0 and rows.max() < B * H * n))
    rp = rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    return (q, k, v, kl, rows), (qp, kp, vp, B, H, n, d), klp, rp


def attn_rows(q, k, v, scale, causal=False, kv_len=None, rows=None):
    """Softmax attention by its definition (Eq. 1, max-subtracted as in Eq. 12).

    Returns float64 ``[len(rows), d]`` (all rows when ``rows`` is None)."""
    keep, (qp, kp, vp, B, H, n, d), klp, rp = _prep(q, k, v, kv_len, rows)
    rows = keep[4]
    out = np.empty((rows.size, d), dtype=np.float64)
    rc = _load().elsa_oracle_attn_rows(qp, kp, vp, B, H, n, d, float(scale), int(bool(causal)), klp,
                                       rp, rows.size, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    assert rc == 0
    return out


def fold_rows(q, k, v, scale, causal=False, kv_len=None, rows=None):
    """Per-query sequential fold (Alg. 1) in FP64.  Same return as ``attn_rows``."""
    keep, (qp, kp, vp, B, H, n, d), klp, rp = _prep(q, k, v, kv_len, rows)
    rows = keep[4]
    out = np.empty((rows.size, d), dtype=np.float64)
    rc = _load().elsa_oracle_fold_rows(qp, kp, vp, B, H, n, d, float(scale), int(bool(causal)), klp,
                                       rp, rows.size, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    assert rc == 0
    return out


def lse_rows(q, k, scale, causal=False, kv_len=None, rows=None):
    """ln sum_j e^{s_ij} per row (float64 ``[len(rows)]``); ``-inf`` where no key is visible."""
    keep, (qp, kp, _, B, H, n, d), klp, rp = _prep(q, k, k, kv_len, rows)
    rows = keep[4]
    out = np.empty(rows.size, dtype=np.float64)
    rc = _load().elsa_oracle_lse_rows(qp, kp, B, H, n, d, float(scale), int(bool(causal)), klp, rp, rows.size,
                                      out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    assert rc == 0
    return out


def partials_rows(q, k, v, scale, num_splits, causal=False, kv_len=None, rows=None):
    """Chunk states (m_c, S_c, W_c) of Prop. 1 for ``num_splits`` contiguous key chunks.

    Returns ``(m [R,C], S [R,C], W [R,C,d])`` float64; fully masked chunks hold
    the identity ``(-inf, 0, 0)``."""
    keep, (qp, kp, vp, B, H, n, d), klp, rp = _prep(q, k, v, kv_len, rows)
    rows = keep[4]
    C = int(num_splits)
    assert 1 <= C
    pm = np.empty((rows.size, C), dtype=np.float64)
    pS = np.empty((rows.size, C), dtype=np.float64)
    pW = np.empty((rows.size, C, d), dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().elsa_oracle_partials_rows(qp, kp, vp, B, H, n, d, float(scale), int(bool(causal)), klp, C,
                                           rp, rows.size, pm.ctypes.data_as(dp), pS.ctypes.data_as(dp),
                                           pW.ctypes.data_as(dp))
    assert rc == 0
    return pm, pS, pW


def attn_varlen(q, k, v, cu_seqlens, scale, causal=False):
    """Packed sequences ``[total_tokens, H, d]``: the definition applied to every sequence on its
    own (pure slicing around ``attn_rows``).  Returns float64 ``[total_tokens, H, d]``."""
    q = np.asarray(q, dtype=np.float32)
    k = np.asarray(k, dtype=np.float32)
    v = np.asarray(v, dtype=np.float32)
    T, H, d = q.shape
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    assert cu[0] == 0 and cu[-1] == T and np.all(np.diff(cu) >= 0)
    out = np.zeros((T, H, d), dtype=np.float64)
    for s in range(cu.size - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b == a:
            continue
        dense = lambda t: np.ascontiguousarray(t[a:b].transpose(1, 0, 2))[None]      # [1, H, len, d]
        o = attn_rows(dense(q), dense(k), dense(v), scale, causal=causal)
        out[a:b] = o.reshape(H, b - a, d).transpose(1, 0, 2)
    return out


def cross_rows(q, k, v, scale, causal=False, kv_len=None, rows=None):
    """Rectangular attention by its definition: ``q [B,H,n_q,d]`` against ``k, v [B,H,n_k,d]``.

    Causal reading: key j is visible to query i iff ``j <= i + (n_k - n_q)`` (last query aligned
    with last key).  Returns ``(out [R,d], lse [R])`` float64; a row is ``(b*H + h)*n_q + i``."""
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    assert q.ndim == 4 and k.ndim == 4 and k.shape == v.shape
    B, H, nq, d = q.shape
    nk = k.shape[2]
    assert k.shape == (B, H, nk, d)
    klp = None
    if kv_len is not None:
        kl = np.ascontiguousarray(kv_len, dtype=np.int32)
        assert kl.shape == (B,)
        klp = kl.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    if rows is None:
        rows = np.arange(B * H * nq, dtype=np.int64)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows.size == 0 or (rows.min() >= 0 and rows.max() < B * H * nq))
    out = np.empty((rows.size, d), dtype=np.float64)
    lse = np.empty(rows.size, dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().elsa_oracle_cross_rows(qp, kp, vp, B, H, nq, nk, d, float(scale), int(bool(causal)), klp,
                                        rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), rows.size,
                                        out.ctypes.data_as(dp), lse.ctypes.data_as(dp))
    assert rc == 0
    return out, lse


def dv_rows(q, k, v, scale, causal=False, kv_len=None, rows=None):
    """Attention whose values have their own width: ``q [B,H,n_q,d]``, ``k [B,H,n_k,d]``,
    ``v [B,H,n_k,d_v]`` (the paper's V in R^{n x d_v}, W in R^{d_v}).  Masks as in ``cross_rows``.
    Returns ``(out [R,d_v], lse [R])`` float64; a row is ``(b*H + h)*n_q + i``."""
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    assert q.ndim == 4 and k.ndim == 4 and v.ndim == 4
    B, H, nq, d = q.shape
    nk, dv = v.shape[2], v.shape[3]
    assert k.shape == (B, H, nk, d) and v.shape == (B, H, nk, dv)
    klp = None
    if kv_len is not None:
        kl = np.ascontiguousarray(kv_len, dtype=np.int32)
        assert kl.shape == (B,)
        klp = kl.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    if rows is None:
        rows = np.arange(B * H * nq, dtype=np.int64)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows.size == 0 or (rows.min() >= 0 and rows.max() < B * H * nq))
    out = np.empty((rows.size, dv), dtype=np.float64)
    lse = np.empty(rows.size, dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().elsa_oracle_dv_rows(qp, kp, vp, B, H, nq, nk, d, dv, float(scale), int(bool(causal)), klp,
                                     rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), rows.size,
                                     out.ctypes.data_as(dp), lse.ctypes.data_as(dp))
    assert rc == 0
    return out, lse


def _merge(fn, a, b):
    ma, Sa, Wa = a
    mb, Sb, Wb = b
    Wa, Wap = _f64(Wa)
    Wb, Wbp = _f64(Wb)
    d = Wa.size
    assert Wb.size == d
    Wo = np.empty(d, dtype=np.float64)
    mo, So = ctypes.c_double(), ctypes.c_double()
    fn(float(ma), float(Sa), Wap, float(mb), float(Sb), Wbp, d, ctypes.byref(mo), ctypes.byref(So),
       Wo.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return mo.value, So.value, Wo


def merge_case(a, b):
    """a (+) b in the case form of Eq. 3; a, b are ``(m, S, W[d])``."""
    return _merge(_load().elsa_oracle_merge_case, a, b)


def merge_unsum(a, b):
    """a (+) b as un-sum-renorm (Eq. 4)."""
    return _merge(_load().elsa_oracle_merge_unsum, a, b)


def identity(d):
    """The identity element e = (-inf, 0, 0)."""
    return (-np.inf, 0.0, np.zeros(d, dtype=np.float64))


def combine_rows(part_m, part_S, part_W):
    """Left-to-right (+) over the chunk axis, then W/S.  Shapes [R,C], [R,C], [R,C,d]."""
    pm, pmp = _f64(part_m)
    pS, pSp = _f64(part_S)
    pW, pWp = _f64(part_W)
    R, C = pm.shape
    d = pW.shape[-1]
    assert pS.shape == (R, C) and pW.shape == (R, C, d)
    out = np.empty((R, d), dtype=np.float64)
    rc = _load().elsa_oracle_combine_rows(pmp, pSp, pWp, R, C, d,
                                          out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    assert rc == 0
    return out


def ladder_f32_fold_rows(q, k, v, scale, causal=False, kv_len=None, rows=None):
    """Alg. 1 carried out entirely in IEEE single precision (diagnostic ladder)."""
    keep, (qp, kp, vp, B, H, n, d), klp, rp = _prep(q, k, v, kv_len, rows)
    rows = keep[4]
    out = np.empty((rows.size, d), dtype=np.float32)
    rc = _load().elsa_ladder_f32_fold_rows(qp, kp, vp, B, H, n, d, float(scale), int(bool(causal)), klp,
                                           rp, rows.size, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    assert rc == 0
    return out


def round_f16(x: float) -> float:
    """``x`` rounded to the nearest IEEE binary16 value (ties to even), as a Python float."""
    return float(_load().elsa_oracle_round_f16(float(x)))


def ladder_f16_rows(q, k, v, scale, causal=False, kv_len=None, rows=None):
    """The definition in FP64 with the two roundings the FP16 variant makes by design: each weight to
    binary16 where it multiplies a value row, and the output to binary16 (diagnostic ladder)."""
    keep, (qp, kp, vp, B, H, n, d), klp, rp = _prep(q, k, v, kv_len, rows)
    rows = keep[4]
    out = np.empty((rows.size, d), dtype=np.float64)
    rc = _load().elsa_ladder_f16_rows(qp, kp, vp, B, H, n, d, float(scale), int(bool(causal)), klp,
                                      rp, rows.size, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    assert rc == 0
    return out
