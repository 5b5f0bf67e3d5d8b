"""Host-side checks of the C-ABI library: it loads, exports what the header declares, and
rejects bad arguments before touching the GPU.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2604_23798_amd", "libelsa.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libelsa.so not built (run __graft_entry__.build())")


def _declared():
    txt = open(os.path.join(ROOT, "include", "elsa.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(elsa_[a-z0-9_]+)\s*\(", txt)))


def test_every_declared_symbol_is_exported():
    lib = ctypes.CDLL(LIB)
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    from paper_2604_23798_amd import elsa
    assert sorted(elsa.EXPORTS) == names


def test_status_strings_and_options():
    from paper_2604_23798_amd import elsa
    assert elsa.status_string(0) == "ok"
    assert "invalid" in elsa.status_string(1) and "unknown" in elsa.status_string(99)
    for opt in range(6):
        assert elsa.elsa_get_option(opt) == 0
    elsa.elsa_set_option(elsa.OPT_PATH, 1)
    assert elsa.elsa_get_option(elsa.OPT_PATH) == 1
    elsa.elsa_set_option(elsa.OPT_PATH, 0)
    with pytest.raises(elsa.ElsaError):
        elsa.elsa_set_option(elsa.OPT_PATH, 4)
    with pytest.raises(elsa.ElsaError):
        elsa.elsa_set_option(9, 0)
    assert elsa.elsa_variant_name(2, 1).startswith("mfma") and elsa.elsa_variant_name(1, 1).startswith("fma")
    assert elsa.elsa_variant_name(2, 99) is None
    assert elsa.elsa_variant_name(3, 1).startswith("mfma16") and elsa.elsa_variant_name(3, 6) == "mfma16_q256_w8" and elsa.elsa_variant_name(3, 7) is None


def test_workspace_bytes():
    from paper_2604_23798_amd import elsa
    B, H, n, d, C = 1, 12, 197, 64, 4
    rows = B * H * C * n
    a = lambda x: (x + 255) // 256 * 256
    assert elsa.elsa_split_kv_workspace_bytes(B, H, n, d, C) == 2 * a(rows * 4) + a(rows * d * 4)
    assert elsa.elsa_split_kv_workspace_bytes(B, H, n, 48, C) == 0
    assert elsa.elsa_split_kv_workspace_bytes(B, H, n, 32, C) == 2 * a(rows * 4) + a(rows * 32 * 4)
    assert elsa.elsa_split_kv_workspace_bytes(B, H, 0, d, C) == 0


def test_bad_arguments_are_rejected_before_any_launch():
    from paper_2604_23798_amd import elsa
    lib = elsa.raw()
    p = ctypes.c_void_p(256)            # never dereferenced: every call below fails validation first
    ok = dict(B=1, H=1, n=8, d=64)
    INV, UNS = 1, 2
    f = lambda **kw: lib.elsa_attn_fwd(kw.get("q", p), p, p, kw.get("out", p), kw.get("B", 1), kw.get("H", 1),
                                       kw.get("n", 8), kw.get("d", 64), kw.get("scale", 0.125), 0,
                                       kw.get("dtype", 0), None)
    assert f(q=None) == INV and f(out=None) == INV
    assert f(B=0) == INV and f(H=-1) == INV and f(n=0) == INV
    assert f(d=48) == UNS and f(d=192) == UNS and f(dtype=2) == UNS
    assert f(scale=float("nan")) == INV and f(scale=float("inf")) == INV
    assert f(n=1 << 24, d=128) == UNS          # one K slice of 8 GiB: beyond the 2 GiB buffer range
    s = lambda C, **kw: lib.elsa_attn_fwd_split_kv(p, p, p, kw.get("pm", p), p, p, 1, 1, 8, 64, 0.125, 0, None, C, 0, None)
    assert s(0) == INV and s(9) == INV and s(2, pm=None) == INV
    c = lambda C, **kw: lib.elsa_combine(p, p, p, kw.get("out", p), 1, 1, 8, kw.get("d", 64), C, 0, None)
    assert c(0) == INV and c(9) == INV and c(2, out=None) == INV and c(2, d=48) == UNS
    assert lib.elsa_set_workspace(p, 0) == INV and lib.elsa_set_workspace(None, 16) == INV
    assert lib.elsa_set_workspace(ctypes.c_void_p(8), 1024) == 3
    assert lib.elsa_set_workspace(None, 0) == 0
    assert lib.elsa_debug_layout_probe(None, None) == INV
    vl = lambda **kw: lib.elsa_attn_fwd_varlen(p, p, p, p, kw.get("cu", p), kw.get("ns", 2), kw.get("T", 64),
                                               kw.get("mx", 40), 2, kw.get("d", 64), 0.125, 0, 0, None)
    assert vl(cu=None) == INV and vl(ns=0) == INV and vl(ns=5000) == INV and vl(T=0) == INV
    assert vl(mx=0) == INV and vl(mx=65) == INV and vl(d=80) == UNS
    x = lambda **kw: lib.elsa_attn_fwd_cross(kw.get("q", p), p, p, p, None, 1, 1, kw.get("nq", 4), kw.get("nk", 8),
                                             kw.get("d", 64), 0.125, 0, None, 0, None)
    assert x(q=None) == INV and x(nq=0) == INV and x(nk=0) == INV and x(nk=-3) == INV and x(d=80) == UNS
    assert x(nq=1, nk=1 << 24, d=128) == UNS   # the key slice, not the query count, sets the limit
    dv = lambda **kw: lib.elsa_attn_fwd_dv(kw.get("q", p), p, p, kw.get("out", p), None, 1, 1, kw.get("nq", 4), kw.get("nk", 8),
                                           kw.get("d", 64), kw.get("dv", 128), kw.get("scale", 0.125), 0, None,
                                           kw.get("dtype", 0), None)
    assert dv(q=None) == INV and dv(out=None) == INV and dv(nq=0) == INV and dv(nk=0) == INV
    assert dv(scale=float("nan")) == INV and dv(dtype=2) == UNS
    for d_, dv_ in ((64, 96), (96, 64), (192, 64), (64, 192), (256, 128), (48, 64), (64, 0)):
        assert dv(d=d_, dv=dv_) == UNS
    assert dv(d=80, dv=80) == UNS               # equal widths: the rules of the rectangular entry point
    assert dv(nq=1, nk=1 << 23, d=32, dv=128) == UNS   # the wider of the K and V slices sets the 2 GiB limit
    st = lambda **kw: lib.elsa_attn_stream_step(kw.get("q", p), p, p, kw.get("state", p), 1, 1, kw.get("nq", 4),
                                                kw.get("nc", 8), kw.get("d", 64), 0.125, 0, 0, None, 1, 0, None)
    assert st(q=None) == INV and st(state=None) == INV and st(nq=0) == INV and st(nc=0) == INV and st(d=80) == UNS
    assert st(state=ctypes.c_void_p(8)) == 3
    fin = lambda **kw: lib.elsa_attn_stream_finish(kw.get("state", p), kw.get("out", p), None, 1, 1, 4, kw.get("d", 64), 0, None)
    assert fin(state=None) == INV and fin(out=None) == INV and fin(d=5) == UNS and fin(state=ctypes.c_void_p(8)) == 3
    assert elsa.elsa_stream_state_bytes(2, 3, 5, 64) == elsa.elsa_split_kv_workspace_bytes(2, 3, 5, 64, 1)
