"""GPU parity at the full workload sizes, in the launch configuration the benchmark times
(library defaults), on seeded row samples the oracle computes one by one (first/last row, the
neighbours of 32-, 64-, 128- and 256-row boundaries, the edges of causal tiles, random rows per
head).  Rows are independent, so a sampled row is a complete check of that row; the rows outside the
sample are covered by two checks that need no oracle: the whole NaN-prefilled output must come back
finite, and two tilings with different query-tile heights must agree on every row.

Tolerances.  Binding on every sampled row: e_row, e_mix and -- on the well-conditioned elements
(|ref| >= rms of the row) -- the literal form |d| / (|ref| + 1e-6), all within the stated tolerance.
On the remaining elements the literal form is not attainable by any evaluation in the stated precision;
there the test requires that the GPU violates it no more than a plain CPU evaluation in that precision
does on the same rows (the single-precision fold of Alg. 1 for FP32 I/O; the definition with
half-rounded weights and outputs for FP16 I/O): fraction of violating elements within 1.25x, worst
element within 4x."""
import numpy as np
import pytest

import oracle
from paper_2604_23798_amd import inputs
from tests import gpu_util as G
from tests.parity import assert_parity, ladder_check, metrics, tolerance

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not G.have_gpu():
        pytest.skip("no GPU")
    from paper_2604_23798_amd import elsa  # noqa: F401


def _check(w, per_head, ladder=True, **opts):
    q, k, v, kv_len = inputs.make(w)
    rows = inputs.sample_rows(w, per_head=per_head)
    f32 = lambda t: t.astype(np.float32)
    ref = oracle.attn_rows(f32(q), f32(k), f32(v), w.scale, causal=w.causal, kv_len=kv_len, rows=rows)
    with G.Options(**opts):
        out = G.fwd(q, k, v, w.scale, causal=w.causal, kv_len=kv_len, rows=rows)     # also: whole output finite
    tol = tolerance(w.n, w.fp16)
    m = assert_parity(out, ref, tol, "%s %s" % (w.name, opts or "default"))
    if ladder:
        if w.fp16:
            lad = oracle.ladder_f16_rows(f32(q), f32(k), f32(v), w.scale, causal=w.causal, kv_len=kv_len, rows=rows)
        else:
            lad = oracle.ladder_f32_fold_rows(f32(q), f32(k), f32(v), w.scale, causal=w.causal, kv_len=kv_len, rows=rows)
        ml = metrics(lad.astype(np.float64), ref, tol)
        msg = "%s literal form: GPU e_elem %.3g (%.3g%% above tol), CPU ladder e_elem %.3g (%.3g%%)" % (
            w.name, m["e_elem"], 100 * m["frac_elem_viol"], ml["e_elem"], 100 * ml["frac_elem_viol"])
        print(msg)
        assert ladder_check(m, ml), msg
    return m


def test_vit_b16_224_all_rows():
    w = inputs.WORKLOADS["vit_b16_224"]
    _check(w, per_head=w.n)


@pytest.mark.parametrize("name", ["bert_base", "bert_base_padded"])
def test_bert_base(name):
    _check(inputs.WORKLOADS[name], per_head=12)


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("n", [1024, 2048, 4096, 8192, 16384])
def test_long_sequence_sweep(n, fp16):
    _check(inputs.sweep(n, fp16), per_head=40 if n >= 8192 else 24)


@pytest.mark.parametrize("n", [1024, 4096, 16384])
def test_row_error_within_a_small_multiple_of_the_merge_depth_bound(n):
    """Thm 1: ||y_hat - y|| / ||y|| <= u * L(n, B) + O(u^2) per row for the scan with exact scores.
    The kernel also rounds the scores (FP32 dot products), so the check allows a factor 8 on top of
    u * L(n, 128): N(0,1) inputs keep the score rounding at the same order as the bound."""
    from oracle.scan import merge_depth
    w = inputs.sweep(n)
    m = _check(w, per_head=24, ladder=False)
    u = 2.0 ** -24
    assert m["e_row"] <= 8 * u * merge_depth(n, 128), (m["e_row"], u * merge_depth(n, 128))


def test_sweep_16k_vector_fma_path():
    _check(inputs.sweep(16384), per_head=8, ladder=False, path=1)


@pytest.mark.parametrize("name", ["llama13b_32k", "llama13b_32k_fp16"])
def test_llama13b_causal_32k(name):
    _check(inputs.WORKLOADS[name], per_head=32)


def test_hires_vit_64k_wide_scores():
    m = _check(inputs.WORKLOADS["hires_vit_64k"], per_head=32)
    assert m["max_abs"] < 1e-3


def test_early_causal_rows_first_row_exact_and_literal_form_as_the_cpu_ladder():
    """The first 256 rows of every head of the causal 32K workload, every element.  Row 0 sees one key: the
    output is that value row bit for bit.  The literal elementwise form is not attainable on all elements even
    here (measured: 13 of 40960 elements of rows 0..7 exceed 1e-4 -- two or three weighted values that cancel),
    so it is bound the same way as at full length: no worse than the single-precision CPU fold on these rows."""
    w = inputs.WORKLOADS["llama13b_32k"]
    q, k, v, _ = inputs.make(w)
    rows = (np.arange(w.B * w.H)[:, None] * w.n + np.arange(256)[None, :]).reshape(-1).astype(np.int64)
    f32 = lambda t: t.astype(np.float32)
    ref = oracle.attn_rows(f32(q), f32(k), f32(v), w.scale, causal=True, rows=rows)
    out = G.fwd(q, k, v, w.scale, causal=True, rows=rows)
    m = assert_parity(out, ref, 1e-4, "llama13b_32k, rows 0..255 of every head")
    assert np.array_equal(out.reshape(w.H, 256, w.d)[:, 0], v[0, :, 0].astype(np.float64))
    lad = oracle.ladder_f32_fold_rows(f32(q), f32(k), f32(v), w.scale, causal=True, rows=rows).astype(np.float64)
    ml = metrics(lad, ref, 1e-4)
    print("rows 0..255: GPU %.4g%% of elements above 1e-4 (worst %.3g), CPU ladder %.4g%% (worst %.3g)" % (
        100 * m["frac_elem_viol"], m["e_elem"], 100 * ml["frac_elem_viol"], ml["e_elem"]))
    assert ladder_check(m, ml), (m, ml)


@pytest.mark.parametrize("name,a,b", [("sweep_n16384", dict(), dict(path=2, variant=11)),
                                      ("sweep_n16384_fp16", dict(), dict(path=3, variant=1)),
                                      ("llama13b_32k", dict(), dict(path=2, variant=11)),
                                      ("llama13b_32k_fp16", dict(), dict(path=3, variant=4)),
                                      ("hires_vit_64k", dict(), dict(path=2, variant=2))])
def test_two_tilings_agree_on_every_row(name, a, b):
    """Every row, not a sample: the default launch and a forced tiling with another query-tile height (so
    that no block boundary, work order or key range coincides) must agree within twice the tolerance in the
    mixed elementwise form, and neither may leave a row of the NaN-prefilled output unwritten.  A complement
    to the oracle sample above, not a substitute for it."""
    import torch
    from paper_2604_23798_amd import elsa
    w = inputs.WORKLOADS[name]
    q, k, v, _ = inputs.make(w)
    tq, tk, tv = G.to_dev(q), G.to_dev(k), G.to_dev(v)
    outs, names = [], []
    for opts in (a, b):
        out = torch.full_like(tq, float("nan"))
        with G.Options(**opts):
            elsa.elsa_attn_fwd(tq, tk, tv, out, w.scale, w.causal)
            names.append(elsa.elsa_last_kernel())
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all()), (name, opts)
        outs.append(out.float())
    assert names[0] != names[1], names
    x, y = outs
    rms = y.pow(2).mean(dim=-1, keepdim=True).sqrt()
    e_mix = ((x - y).abs() / (y.abs() + rms)).max().item()
    e_row = ((x - y).norm(dim=-1) / y.norm(dim=-1)).max().item()
    tol = tolerance(w.n, w.fp16)
    print("%s: %s vs %s on all %d rows: e_mix %.3g e_row %.3g" % (name, names[0], names[1], w.B * w.H * w.n, e_mix, e_row))
    assert e_mix <= 2 * tol and e_row <= 2 * tol, (names, e_mix, e_row)


@pytest.mark.parametrize("name", ["swin_w7", "swin_w8", "swin_w14", "swin_w16"])
def test_window_attention_shapes(name):
    """Many small independent windows (d = 32): batched tiny problems, every row checked."""
    w = inputs.WORKLOADS[name]
    _check(w, per_head=w.n)
    _check(w.with_(fp16=True, name=name + "_fp16"), per_head=w.n)


@pytest.mark.parametrize("fp16", [False, True])
def test_one_head_at_416400_tokens(fp16):
    """Far beyond the stated sizes (n is no multiple of any tile): same tolerance as at 64K."""
    w = inputs.WORKLOADS["frames_416k"]
    if fp16:
        w = w.with_(fp16=True, name="frames_416k_fp16")
    q, k, v, kv_len = inputs.make(w)
    rows = inputs.sample_rows(w, per_head=64)
    f32 = lambda t: t.astype(np.float32)
    ref = oracle.attn_rows(f32(q), f32(k), f32(v), w.scale, rows=rows)
    out = G.fwd(q, k, v, w.scale, rows=rows)
    assert_parity(out, ref, 2e-3 if fp16 else 1e-4, w.name)


def test_small_workloads_with_workspace_split():
    """The two short workloads again with a lent workspace, so the library splits the key range."""
    import torch
    from paper_2604_23798_amd import elsa
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)
    try:
        _check(inputs.WORKLOADS["vit_b16_224"], per_head=197, splits=2)
        _check(inputs.sweep(1024), per_head=24)
        _check(inputs.sweep(2048), per_head=24)
    finally:
        elsa.elsa_set_workspace(None)


@pytest.mark.parametrize("fp16", [False, True])
def test_decode_against_32k_keys_with_the_workspace_the_benchmark_lends(fp16):
    """The decode workload of bench.py (B 2, H 40, one query, 32768 keys, d 128, 16 key chunks + combine):
    every row checked (a row is one (batch, head))."""
    import torch
    from paper_2604_23798_amd import elsa
    B, H, d, nq, nk = 2, 40, 128, 1, 32768
    q = inputs.normal(1007, 0, 0, B * H * nq * d).reshape(B, H, nq, d)
    k = inputs.normal(1007, 1, 0, B * H * nk * d).reshape(B, H, nk, d)
    v = inputs.normal(1007, 2, 0, B * H * nk * d).reshape(B, H, nk, d)
    if fp16:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    scale = float(np.float32(d ** -0.5))
    f32 = lambda t: t.astype(np.float32)
    ref, ref_lse = oracle.cross_rows(f32(q), f32(k), f32(v), scale, causal=True)
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)
    try:
        out, lse = G.fwd_cross(q, k, v, scale, causal=True, want_lse=True)
        assert elsa.elsa_last_kernel() == "fma_decode_q1" and elsa.elsa_last_splits() == 16
    finally:
        elsa.elsa_set_workspace(None)
    assert_parity(out, ref, tolerance(nk, fp16), "decode_32k fp16=%d" % fp16)
    assert np.max(np.abs(lse - ref_lse)) < (5e-3 if fp16 else 2e-5)


@pytest.mark.parametrize("name", ["dv_192_128_8192", "dv_192_128_8192_causal_fp16", "dv_64_128_16384", "dv_128_64_16384_fp16"])
def test_value_width_workloads_of_the_benchmark(name):
    """bench.py's dv_<d>_<d_v>_<n> workloads (B 1, H 16) on sampled rows: first and last rows, the
    neighbours of a tile boundary, and evenly spaced ones."""
    parts = name.split("_")
    d, dv, n = int(parts[1]), int(parts[2]), int(parts[3])
    fp16, causal = "fp16" in parts[4:], "causal" in parts[4:]
    B, H = 1, 16
    q = inputs.normal(1012, 0, 0, B * H * n * d).reshape(B, H, n, d)
    k = inputs.normal(1012, 1, 0, B * H * n * d).reshape(B, H, n, d)
    v = inputs.normal(1012, 2, 0, B * H * n * dv).reshape(B, H, n, dv)
    if fp16:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    scale = float(np.float32(d ** -0.5))
    per_head = np.unique(np.concatenate([[0, 1, 127, 128, 129, n - 2, n - 1], np.linspace(0, n - 1, 25).astype(np.int64)]))
    rows = (np.arange(B * H)[:, None] * n + per_head[None, :]).reshape(-1).astype(np.int64)
    f32 = lambda t: t.astype(np.float32)
    ref, _ = oracle.dv_rows(f32(q), f32(k), f32(v), scale, causal=causal, rows=rows)
    out = G.fwd_dv(q, k, v, scale, causal=causal)[rows]
    assert_parity(out, ref, tolerance(n, fp16), name)
