"""GPU parity: the HIP path (through the C ABI) against the FP64 oracle, element by element,
on seeded inputs small enough for the full oracle yet spanning several tiles and ragged tails."""
import math

import numpy as np
import pytest

import oracle
from paper_2604_23798_amd import inputs
from tests import gpu_util as G
from tests.parity import assert_parity, tolerance

pytestmark = pytest.mark.gpu

MFMA, FMA, MFMA16 = 2, 1, 3
ALL_KERNELS = [(MFMA, 1), (MFMA, 2), (MFMA, 3), (MFMA, 4), (MFMA, 5), (MFMA, 6), (MFMA, 7), (MFMA, 8),
               (MFMA, 9), (MFMA, 10), (MFMA, 11), (FMA, 1), (FMA, 2)]


def _rand(B, H, n, d, seed, sigma=1.0, fp16=False):
    cnt = B * H * n * d
    sh = (B, H, n, d)
    q = inputs.normal(seed, 0, 0, cnt, sigma).reshape(sh)
    k = inputs.normal(seed, 1, 0, cnt, sigma).reshape(sh)
    v = inputs.normal(seed, 2, 0, cnt).reshape(sh)
    if fp16:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    return q, k, v


def _f32(*ts):
    return tuple(t.astype(np.float32) for t in ts)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not G.have_gpu():
        pytest.skip("no GPU")
    from paper_2604_23798_amd import elsa  # noqa: F401  (fails loudly if the library is missing)


def test_mfma_layout_and_half_wave_exchange():
    """The operand maps the forward kernel is built on, read back from the hardware."""
    import torch
    from paper_2604_23798_amd import elsa
    out = torch.zeros(5 * 16 * 64, device="cuda")
    elsa.elsa_debug_layout_probe(out)
    torch.cuda.synchronize()
    r = out.cpu().numpy().reshape(5, 16, 64)
    lane = np.arange(64)
    for i in range(16):
        assert np.array_equal(r[0, i], 8 * (i // 4) + 4 * (lane // 32) + (i % 4) + 1), ("row map", i)
        assert np.array_equal(r[1, i], lane % 32 + 1), ("column map", i)
        assert np.all(r[2, i] == 1.0), ("k index = lane / 32", i)
    assert np.array_equal(r[3, 0], lane % 32 + 32)
    assert np.array_equal(r[3, 1], 2 * (lane % 32) + 32)
    ex = 2.0 ** (-lane / 8.0)
    assert np.all(np.abs(r[4, 0] - ex) <= 4 * 2.0 ** -24 * ex)


def test_issue_probe_hook_runs_and_orders_the_instruction_kinds():
    """The measurement hook behind ``bench.py --issue-rates``: every kind runs, rejects bad arguments, and the two
    facts the kernels' design rests on hold -- an exponential costs more issue time than an add, and a wave's adds
    are barely slowed by FP16 MFMAs of the other wave of its SIMD while FP32 MFMAs stop them."""
    import torch
    from paper_2604_23798_amd import elsa
    out = torch.zeros(8 + 256 * 512, device="cuda")
    t = {}
    for ka, kb, waves in [(0, 0, 1), (2, 2, 1), (2, 7, 2), (6, 2, 2), (5, 2, 2), (1, 1, 2), (3, 3, 1), (4, 4, 1)]:
        elsa.elsa_debug_issue_probe(out, ka, kb, waves, 2000)
        elsa.elsa_debug_issue_probe(out, ka, kb, waves, 2000)
        torch.cuda.synchronize()
        r = out[:8].cpu().numpy()
        assert np.all(r[:4 * waves] > 0)
        t[(ka, kb, waves)] = (r[:4].mean(), r[4:8].mean())
    assert t[(0, 0, 1)][0] > 1.2 * t[(2, 2, 1)][0]                 # exp vs add
    add_alone = t[(2, 7, 2)][0]
    assert t[(6, 2, 2)][1] < 1.5 * add_alone                       # adds beside FP16 MFMAs: nearly unhindered
    assert t[(5, 2, 2)][1] > 2.0 * add_alone                       # adds beside FP32 MFMAs: they wait
    for bad in [(-1, 0, 1, 10), (0, 11, 1, 10), (0, 0, 3, 10), (0, 0, 1, 0), (10, 1, 2, 10), (0, 9, 2, 10)]:
        with pytest.raises(elsa.ElsaError):
            elsa.elsa_debug_issue_probe(out, *bad)
    # the register-only model of one FP16 fold step (kinds 8 = its MFMAs, 9 = its fold, 10 = the whole step): the
    # whole step takes at least its longer part and no more than both parts one after the other (plus 15 %)
    m = {}
    for k in (8, 9, 10):
        for _ in range(2):
            elsa.elsa_debug_issue_probe(out, k, k, 2, 1000)
        torch.cuda.synchronize()
        r = out[:8].cpu().numpy()
        assert np.all(r > 0)
        m[k] = float(r.max())
    assert max(m[8], m[9]) <= m[10] <= 1.15 * (m[8] + m[9]), m


@pytest.mark.parametrize("path,variant", ALL_KERNELS)
@pytest.mark.parametrize("shape", [(1, 2, 197, 64), (2, 2, 330, 64), (1, 2, 300, 128), (2, 3, 200, 32)])
@pytest.mark.parametrize("causal", [False, True])
def test_small_problems_every_kernel(path, variant, shape, causal):
    B, H, n, d = shape
    q, k, v = _rand(B, H, n, d, 100 + n)
    scale = 1.0 / math.sqrt(d)
    ref = oracle.attn_rows(q, k, v, scale, causal=causal)
    with G.Options(path=path, variant=variant):
        out = G.fwd(q, k, v, scale, causal=causal)
    assert_parity(out, ref, tolerance(n), "path%d v%d %s causal=%d" % (path, variant, shape, causal))


@pytest.mark.parametrize("path,variant", [(MFMA, 1), (MFMA, 3), (FMA, 1), (MFMA16, 1), (MFMA16, 2), (MFMA16, 3), (MFMA16, 4)])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_fp16_io(path, variant, d):
    B, H, n = 1, 3, 450
    q, k, v = _rand(B, H, n, d, 7, fp16=True)
    scale = 1.0 / math.sqrt(d)
    for causal in (False, True):
        ref = oracle.attn_rows(*_f32(q, k, v), scale, causal=causal)
        with G.Options(path=path, variant=variant):
            out = G.fwd(q, k, v, scale, causal=causal)
        assert_parity(out, ref, tolerance(n, fp16=True), "fp16 path%d v%d d%d causal=%d" % (path, variant, d, causal))


@pytest.mark.parametrize("variant", [1, 2, 3, 4])
def test_fp16_matrix_core_path_masks_splits_and_edges(variant):
    """The FP16-MFMA kernel through every feature: padding, causal, split-KV states, combine,
    ragged sizes, negative and zero scale (zero falls back to the FP32-MFMA kernel)."""
    import torch
    from paper_2604_23798_amd import elsa
    tol = 2e-3
    B, H, n, d = 3, 2, 333, 64
    q, k, v = _rand(B, H, n, d, 91, fp16=True)
    qf, kf, vf = _f32(q, k, v)
    kv_len = np.array([333, 0, 77], np.int32)
    for causal in (False, True):
        with G.Options(path=MFMA16, variant=variant):
            out = G.fwd(q, k, v, 0.125, causal=causal, kv_len=kv_len)
        assert_parity(out, oracle.attn_rows(qf, kf, vf, 0.125, causal=causal, kv_len=kv_len), tol, "fp16 masks")
        assert np.all(out.reshape(B, H, n, d)[1] == 0.0)
    with G.Options(path=MFMA16, variant=variant):
        out = G.fwd(q, k, v, -0.3)
        name = elsa.elsa_last_kernel()
    assert name.startswith("mfma16")
    assert_parity(out, oracle.attn_rows(qf, kf, vf, -0.3), tol, "fp16 negative scale")
    out = G.fwd(q, k, v, 0.0)                                   # auto path: FP32-MFMA fallback
    assert not elsa.elsa_last_kernel().startswith("mfma16")
    assert_parity(out, oracle.attn_rows(qf, kf, vf, 0.0), tol, "fp16 zero scale")
    for nn in (1, 31, 33, 65):
        q2, k2, v2 = _rand(1, 1, nn, 128, 92 + nn, fp16=True)
        with G.Options(path=MFMA16, variant=variant):
            o2 = G.fwd(q2, k2, v2, 0.09, causal=True)
        assert_parity(o2, oracle.attn_rows(*_f32(q2, k2, v2), 0.09, causal=True), tol, "fp16 n=%d" % nn)
    C = 3
    with G.Options(path=MFMA16, variant=variant):
        pm, pS, pW = G.split_kv(q, k, v, 0.125, C, causal=True)
    gm, gS, gW = G.parts_to_rows(pm, pS, pW)
    om, oS, oW = oracle.partials_rows(qf, kf, vf, 0.125, C, causal=True)
    ident = np.isneginf(om)
    assert np.array_equal(np.isneginf(gm), ident) and np.all(gS[ident] == 0) and np.all(gW[ident] == 0)
    live = ~ident
    assert np.all(np.abs(gm[live] - om[live]) <= 4e-6 * (1 + np.abs(om[live])))
    assert np.all(np.abs(gm[live] + np.log(gS[live]) - om[live] - np.log(oS[live])) <= 1e-3)
    out16 = torch.full((B, H, n, d), float("nan"), device="cuda", dtype=torch.float16)
    elsa.elsa_combine(pm, pS, pW, out16)
    torch.cuda.synchronize()
    assert_parity(out16.reshape(-1, d).double().cpu().numpy(), oracle.attn_rows(qf, kf, vf, 0.125, causal=True), tol,
                  "fp16 split + combine")


@pytest.mark.parametrize("d", [96, 128, 256])
def test_fp16_wide_tile_of_eight_query_waves(d):
    """FP16 tile 6 (d >= 96): 256 query rows per block, eight query waves of one group each on shared K/V tiles.
    Ragged sizes around its tile edges, causal mask, key padding with NaN beyond kv_len, log-normaliser, and the
    states it writes (through the exact-maximum instantiation) against the FP64 oracle; unsupported below d = 96."""
    import torch
    from paper_2604_23798_amd import elsa
    tol = 2e-3
    scale = 1.0 / math.sqrt(d)
    for n in (700, 257, 255, 33):
        q, k, v = _rand(2, 2, n, d, 300 + n + d, fp16=True)
        qf, kf, vf = _f32(q, k, v)
        for causal in (False, True):
            with G.Options(path=MFMA16, variant=6):
                out, lse = G.fwd_cross(q, k, v, scale, causal=causal, want_lse=True)
                assert elsa.elsa_last_kernel() == "mfma16_q256_w8"
            assert_parity(out, oracle.attn_rows(qf, kf, vf, scale, causal=causal), tol, "w8 d%d n%d causal=%d" % (d, n, causal))
            assert np.all(np.abs(lse - oracle.lse_rows(qf, kf, scale, causal=causal)) <= tol)
    B, H, n = 3, 2, 600
    q, k, v = _rand(B, H, n, d, 310 + d, fp16=True)
    kv_len = np.array([600, 0, 301], np.int32)
    for b in range(B):
        k[b, :, kv_len[b]:] = np.nan
        v[b, :, kv_len[b]:] = np.inf
    qf, kf, vf = _f32(q, k, v)
    for causal in (False, True):
        with G.Options(path=MFMA16, variant=6):
            out = G.fwd(q, k, v, scale, causal=causal, kv_len=kv_len)
        assert np.all(np.isfinite(out))
        assert_parity(out, oracle.attn_rows(qf, kf, vf, scale, causal=causal, kv_len=kv_len), tol, "w8 padded d%d" % d)
    q, k, v = _rand(1, 2, 520, d, 320 + d, fp16=True)
    qf, kf, vf = _f32(q, k, v)
    with G.Options(path=MFMA16, variant=6):
        pm, pS, pW = G.split_kv(q, k, v, scale, 2, causal=True)
    gm, gS, gW = G.parts_to_rows(pm, pS, pW)
    om, oS, oW = oracle.partials_rows(qf, kf, vf, scale, 2, causal=True)
    live = ~np.isneginf(om)
    assert np.array_equal(np.isneginf(gm), ~live)
    assert np.all(np.abs(gm[live] - om[live]) <= 4e-6 * (1 + np.abs(om[live])))             # the exact chunk maximum
    assert np.all(np.abs(gm[live] + np.log(gS[live]) - om[live] - np.log(oS[live])) <= 1e-3)
    q, k, v = _rand(1, 1, 300, 64, 330, fp16=True)
    with G.Options(path=MFMA16, variant=6):
        with pytest.raises(elsa.ElsaError):
            G.fwd(q, k, v, 0.125)


@pytest.mark.parametrize("path,variant", [(MFMA16, 1), (MFMA16, 2), (MFMA16, 3), (MFMA16, 4), (MFMA16, 6), (MFMA, 1), (MFMA, 3), (MFMA, 7), (MFMA, 11)])
@pytest.mark.parametrize("d", [64, 128])
def test_reference_that_lags_the_maximum(path, variant, d):
    if path == MFMA16 and variant == 6 and d < 96:
        pytest.skip("tile 6 serves d >= 96 only")
    """The matrix-core tiles let the m of the running state lag the true maximum and redo a step the exact way when
    a partial row sum passes their limit (2^10 with FP16 weights, 2^16 with FP32 ones) or a row meets its first
    key.  Score profiles along the keys that exercise both sides of that test: a slow creep (no single step jumps,
    the lag accumulates past the limit), jumps far above the limit, one early spike that stays the maximum, a
    descent, a creep that stays below the limit for good, and rows whose every score is far below zero (a first
    reference of 0 would lose them).  Output and log-normaliser against the FP64 oracle, with and without a
    causal mask."""
    fp16 = path == MFMA16
    B, H, n = 1, 2, 700
    scale = 0.125
    j = np.arange(n)
    profiles = {                                   # added to every score of key j, in natural units
        "creep": 0.75 * (j // 32),                 # +0.75 per 32 keys: 15.75 in all (22.7 in log2 units)
        "jumps": 12.0 * (j // 100),                # +12 every 100 keys: e^12 > 2^16 at once
        "spike": np.where(j == 5, 40.0, 0.0),      # one early key dominates
        "descent": -0.25 * (j // 16),
        "small creep": 0.125 * (j // 64),          # 1.25 in all: the reference is never renewed after the first step
        "far below zero": np.full(n, -200.0) + 0.25 * (j % 7),
    }
    for name, prof in profiles.items():
        # FP32 dot products of magnitude |c| are rounded at ulp(|c|) per accumulation step: the same allowance as in
        # the shift test (32 u |c|) on top of the ordinary tolerance; the FP16 path's 2e-3 covers it
        tol = 2e-3 if fp16 else 2e-5 + 32 * 2.0 ** -24 * float(np.abs(prof).max())
        q, k, v = _rand(B, H, n, d, 77 + d, fp16=fp16)
        q[..., 0] = 1.0
        k[..., 0] = (prof / scale)[None, None, :].astype(k.dtype)          # multiples of 1 / 8 up to 2^11: exact in FP16
        qf, kf, vf = _f32(q, k, v)
        for causal in (False, True):
            ref = oracle.attn_rows(qf, kf, vf, scale, causal=causal)
            with G.Options(path=path, variant=variant):
                out, lse = G.fwd_cross(q, k, v, scale, causal=causal, want_lse=True)
            assert np.all(np.isfinite(out)), name
            assert_parity(out, ref, tol, "path%d v%d d%d %s causal=%d" % (path, variant, d, name, causal))
            ref_lse = oracle.lse_rows(qf, kf, scale, causal=causal)
            assert np.all(np.abs(lse - ref_lse) <= tol * (1 + np.abs(ref_lse))), (name, float(np.abs(lse - ref_lse).max()))


@pytest.mark.parametrize("path,variant", ALL_KERNELS)
def test_key_padding_mask(path, variant):
    B, H, n, d = 5, 2, 200, 64
    q, k, v = _rand(B, H, n, d, 21)
    kv_len = np.array([200, 1, 0, 129, 64], np.int32)
    for causal in (False, True):
        ref = oracle.attn_rows(q, k, v, 0.125, causal=causal, kv_len=kv_len)
        with G.Options(path=path, variant=variant):
            out = G.fwd(q, k, v, 0.125, causal=causal, kv_len=kv_len)
        assert_parity(out, ref, tolerance(n), "padding path%d v%d causal=%d" % (path, variant, causal))
        o = out.reshape(B, H, n, d)
        assert np.all(o[2] == 0.0)                                   # no visible key -> zeros
        if not causal:
            assert np.all(np.abs(o[1] - v[1, :, :1].astype(np.float64)) <= 1e-6)   # kv_len = 1 -> v_0
    # kv_len = n through the masked entry point equals the unmasked call bit for bit
    with G.Options(path=path, variant=variant):
        a = G.fwd(q, k, v, 0.125, kv_len=np.full(B, n, np.int32))
        b = G.fwd(q, k, v, 0.125)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("path,variant", [(MFMA, 1), (MFMA, 3), (FMA, 1), (FMA, 2)])
@pytest.mark.parametrize("C", [1, 2, 3, 7])
@pytest.mark.parametrize("causal", [False, True])
def test_split_kv_states_and_combine(path, variant, C, causal):
    import torch
    from paper_2604_23798_amd import elsa
    B, H, n, d = 1, 2, 300, 64
    q, k, v = _rand(B, H, n, d, 33)
    scale = 0.125
    tol = tolerance(n)
    om, oS, oW = oracle.partials_rows(q, k, v, scale, C, causal=causal)
    with G.Options(path=path, variant=variant):
        pm, pS, pW = G.split_kv(q, k, v, scale, C, causal=causal)
    gm, gS, gW = G.parts_to_rows(pm, pS, pW)
    ident = np.isneginf(om)
    # masked chunks are the identity exactly
    assert np.array_equal(np.isneginf(gm), ident)
    assert np.all(gS[ident] == 0.0) and np.all(gW[ident] == 0.0)
    live = ~ident
    # the chunk maximum in natural-log units
    assert np.all(np.abs(gm[live] - om[live]) <= 4e-6 * (1 + np.abs(om[live])))
    # canonical form: log of the unnormalised mass, and the chunk's own weighted mean
    lse_g = gm[live] + np.log(gS[live])
    lse_o = om[live] + np.log(oS[live])
    assert np.all(np.abs(lse_g - lse_o) <= 1e-5)
    assert_parity((gW[live] / gS[live][:, None]), (oW[live] / oS[live][:, None]), tol, "chunk means C=%d" % C)
    # second pass on the device states
    out = torch.full((B, H, n, d), float("nan"), device="cuda")
    elsa.elsa_combine(pm, pS, pW, out)
    torch.cuda.synchronize()
    ref = oracle.attn_rows(q, k, v, scale, causal=causal)
    assert_parity(out.reshape(-1, d).double().cpu().numpy(), ref, tol, "combine C=%d causal=%d" % (C, causal))


@pytest.mark.parametrize("d,fp16_out", [(64, False), (128, False), (64, True), (32, False)])
def test_combine_alone_on_oracle_states(d, fp16_out):
    """elsa_combine fed with block states written by the oracle (incl. identities)."""
    import torch
    from paper_2604_23798_amd import elsa
    B, H, n, C = 1, 2, 150, 5
    q, k, v = _rand(B, H, n, d, 44)
    om, oS, oW = oracle.partials_rows(q, k, v, 0.2, C, causal=True)
    pm = torch.from_numpy(om.reshape(B, H, n, C).transpose(0, 1, 3, 2).astype(np.float32).copy()).cuda()
    pS = torch.from_numpy(oS.reshape(B, H, n, C).transpose(0, 1, 3, 2).astype(np.float32).copy()).cuda()
    pW = torch.from_numpy(oW.reshape(B, H, n, C, d).transpose(0, 1, 3, 2, 4).astype(np.float32).copy()).cuda()
    out = torch.full((B, H, n, d), float("nan"), device="cuda", dtype=torch.float16 if fp16_out else torch.float32)
    elsa.elsa_combine(pm, pS, pW, out)
    torch.cuda.synchronize()
    ref = oracle.attn_rows(q, k, v, 0.2, causal=True)
    assert_parity(out.reshape(-1, d).double().cpu().numpy(), ref, tolerance(n, fp16_out), "combine alone d=%d" % d)
    # all-identity rows give zeros
    pm[:] = float("-inf")
    pS[:] = 0
    pW[:] = 0
    elsa.elsa_combine(pm, pS, pW, out)
    torch.cuda.synchronize()
    assert torch.all(out == 0)


@pytest.mark.parametrize("path", [MFMA, FMA])
def test_internal_split_through_workspace(path):
    import torch
    from paper_2604_23798_amd import elsa
    B, H, n, d = 1, 2, 1100, 64
    q, k, v = _rand(B, H, n, d, 55)
    ref = oracle.attn_rows(q, k, v, 0.125)
    refc = oracle.attn_rows(q, k, v, 0.125, causal=True)
    ws = torch.empty(elsa.elsa_split_kv_workspace_bytes(B, H, n, d, 4), dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)
    try:
        with G.Options(path=path, splits=4):
            out = G.fwd(q, k, v, 0.125)
            outc = G.fwd(q, k, v, 0.125, causal=True)
        with G.Options(path=path):           # auto: small problem + workspace -> splits on its own
            outa = G.fwd(q, k, v, 0.125)
    finally:
        elsa.elsa_set_workspace(None)
    assert_parity(out, ref, tolerance(n), "workspace split")
    assert_parity(outc, refc, tolerance(n), "workspace split causal")
    assert_parity(outa, ref, tolerance(n), "workspace auto split")


@pytest.mark.parametrize("path,variant", ALL_KERNELS)
def test_degenerate_sizes(path, variant):
    for n in (1, 2, 31, 32, 33, 64, 65):
        q, k, v = _rand(1, 1, n, 64, 60 + n)
        with G.Options(path=path, variant=variant):
            out = G.fwd(q, k, v, 0.125)
            outc = G.fwd(q, k, v, 0.125, causal=True)
        assert_parity(out, oracle.attn_rows(q, k, v, 0.125), 2e-5, "n=%d" % n)
        assert_parity(outc, oracle.attn_rows(q, k, v, 0.125, causal=True), 2e-5, "n=%d causal" % n)
        assert np.all(np.abs(outc[0] - v[0, 0, 0]) <= 1e-6)              # causal row 0 sees only itself


@pytest.mark.parametrize("path,variant", [(MFMA, 1), (MFMA, 3), (FMA, 1)])
def test_wide_scores_one_hot_and_shift(path, variant):
    # scores with sigma ~ 64 (the high-resolution ViT recipe): rescaling path, no inf/nan
    q, k, v = _rand(1, 2, 700, 64, 71, sigma=8.0)
    with G.Options(path=path, variant=variant):
        out = G.fwd(q, k, v, 0.125)
    assert_parity(out, oracle.attn_rows(q, k, v, 0.125), 1e-4, "wide scores")
    # one dominant key per row -> its value row, to FP32 roundoff
    q, k, v = _rand(1, 1, 256, 64, 72)
    k[0, 0, 100] = 0
    q[..., 0] = 1.0
    k[..., 0] = 0
    k[0, 0, 100, 0] = 2000.0                 # scaled gap 250 >> 104: every other weight underflows to 0
    with G.Options(path=path, variant=variant):
        out = G.fwd(q, k, v, 0.125)
    assert np.all(out == v[0, 0, 100].astype(np.float64)[None, :])
    # Shifting every score of a row by a constant c leaves the output unchanged in real arithmetic.
    # In FP32 the shifted dot products are rounded at ulp(|c|), so the weights move by about
    # u*|c| per accumulation step: the bound below is 32*u*|c| (plus the ordinary tolerance).
    q, k, v = _rand(1, 2, 300, 64, 73)
    q[..., 0] = 1.0
    k[..., 0] = np.round(k[..., 0] * 4) / 4
    ref = oracle.attn_rows(q, k, v, 0.125)
    for c in (-30.0, 50.0, -400.0, 1000.0):
        k2 = k.copy()
        k2[..., 0] += np.float32(c / 0.125)
        with G.Options(path=path, variant=variant):
            out = G.fwd(q, k2, v, 0.125)
        assert_parity(out, ref, 2e-5 + 32 * 2.0 ** -24 * abs(c), "shift %g" % c)


@pytest.mark.parametrize("path,variant", [(MFMA, 1), (MFMA, 2), (MFMA, 3), (FMA, 1), (FMA, 2)])
def test_varlen_packed_sequences(path, variant):
    lens = [197, 0, 1, 130, 64, 33, 300]
    q, k, v, cu = inputs.make_varlen(17, lengths=lens, H=3, d=64)
    T = q.shape[0]
    for causal in (False, True):
        ref = oracle.attn_varlen(q, k, v, cu, 0.125, causal=causal).reshape(T * 3, 64)
        with G.Options(path=path, variant=variant):
            out = G.fwd_varlen(q, k, v, cu, max(lens), 0.125, causal=causal).reshape(T * 3, 64)
        assert_parity(out, ref, tolerance(max(lens)), "varlen path%d v%d causal=%d" % (path, variant, causal))
    # a single packed sequence with one head is the dense problem: same kernel, same bits
    q1, k1, v1, cu1 = inputs.make_varlen(18, lengths=[257], H=1, d=64)
    with G.Options(path=path, variant=variant):
        a = G.fwd_varlen(q1, k1, v1, cu1, 257, 0.125).reshape(257, 64)
        b = G.fwd(q1.reshape(1, 1, 257, 64), k1.reshape(1, 1, 257, 64), v1.reshape(1, 1, 257, 64), 0.125)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("d", [32, 64, 128])
def test_varlen_fp16_and_paper_recipe(d):
    # 8 sequences with lengths uniform on [256, 1792] (the padding-free workload), default kernels
    for fp16 in (False, True):
        q, k, v, cu = inputs.make_varlen(19, 8, 256, 1792, H=2, d=d, fp16=fp16)
        T = q.shape[0]
        ref = oracle.attn_varlen(q, k, v, cu, d ** -0.5, causal=False).reshape(T * 2, d)
        out = G.fwd_varlen(q, k, v, cu, int(np.diff(cu).max()), d ** -0.5).reshape(T * 2, d)
        assert_parity(out, ref, tolerance(1792, fp16), "varlen recipe d=%d fp16=%d" % (d, fp16))


@pytest.mark.parametrize("path,variant,splits", [(MFMA, 1, 0), (MFMA, 3, 0), (FMA, 1, 0), (MFMA, 1, 3), (MFMA16, 1, 0)])
def test_log_normaliser_and_drift_metrics(path, variant, splits):
    """elsa_attn_fwd_lse: the row log-normaliser, and through it the paper's six drift metrics
    (probabilities P_ij = e^{s_ij - lse_i}) on a short, a long-ish and a wide-score problem."""
    import torch
    from paper_2604_23798_amd import elsa
    from tests.parity import drift_metrics
    fp16 = path == MFMA16
    for (n, sigma, causal) in ((197, 1.0, False), (1500, 1.0, True), (700, 8.0, False)):
        B, H, d = 1, 2, 64
        q, k, v = _rand(B, H, n, d, 300 + n, sigma=sigma, fp16=fp16)
        qf, kf, vf = _f32(q, k, v)
        tq, tk, tv = G.to_dev(q), G.to_dev(k), G.to_dev(v)
        out = torch.full_like(tq, float("nan"))
        lse = torch.full((B, H, n), float("nan"), device="cuda")
        ws = torch.empty(elsa.elsa_split_kv_workspace_bytes(B, H, n, d, max(splits, 1)), dtype=torch.uint8, device="cuda")
        if splits:
            elsa.elsa_set_workspace(ws)
        try:
            with G.Options(path=path, variant=variant, splits=splits):
                elsa.elsa_attn_fwd_lse(tq, tk, tv, out, lse, 0.125, causal)
            torch.cuda.synchronize()
        finally:
            elsa.elsa_set_workspace(None)
        ref_lse = oracle.lse_rows(qf, kf, 0.125, causal=causal)
        got_lse = lse.reshape(-1).double().cpu().numpy()
        # |s| reaches ~300 on the wide problem: an FP32 score carries ~1e-4 of rounding there
        assert np.all(np.abs(got_lse - ref_lse) <= (2e-3 if fp16 else 2e-5 * max(1.0, sigma ** 2))), \
            float(np.abs(got_lse - ref_lse).max())
        ref_y = oracle.attn_rows(qf, kf, vf, 0.125, causal=causal)
        got_y = out.reshape(-1, d).double().cpu().numpy()
        s = 0.125 * np.einsum("bhid,bhjd->bhij", qf.astype(np.float64), kf.astype(np.float64)).reshape(-1, n)
        if causal:
            s = np.where(np.tile(np.tril(np.ones((n, n), bool)), (B * H, 1)), s, -np.inf)
        m = drift_metrics(np.exp(s - got_lse[:, None]), np.exp(s - ref_lse[:, None]), got_y, ref_y)
        print("drift path%d n=%d sigma=%g:" % (path, n, sigma), m)
        tol = tolerance(n, fp16) if sigma == 1.0 else (2e-3 if fp16 else 1e-4)
        assert m["arg_rate"] == 0.0
        assert m["dP_inf"][2] <= 10 * tol and m["dP_l2_rel"][2] <= 10 * tol and m["js"][2] <= tol
        assert m["dY_l2_rel"][2] <= tol


def test_deterministic_and_option_reporting():
    from paper_2604_23798_amd import elsa
    q, k, v = _rand(1, 4, 777, 64, 81)
    for path, variant in ALL_KERNELS:
        with G.Options(path=path, variant=variant):
            a = G.fwd(q, k, v, 0.125)
            name = elsa.elsa_last_kernel()
            b = G.fwd(q, k, v, 0.125)
        assert np.array_equal(a, b)
        assert name == elsa.elsa_variant_name(path, variant)
    with G.Options(path=MFMA, variant=1, xcd_map=2):
        c = G.fwd(q, k, v, 0.125)
    with G.Options(path=MFMA, variant=1, xcd_map=1):
        d_ = G.fwd(q, k, v, 0.125)
    assert np.array_equal(c, d_)            # the block-to-work mapping does not change any result


def test_causal_work_orders_give_identical_results():
    """Block -> work item maps are permutations: every order must produce the same bits."""
    # 320 blocks: the reversed run is partial; 960 blocks: the whole second half is reversed
    for w, paths in ((inputs.sweep(2048).with_(causal=True, H=20, name="order"), (0, 1)),
                     (inputs.sweep(8192).with_(causal=True, H=15, name="order4"), (0,))):
        q, k, v, _ = inputs.make(w)
        rows = inputs.sample_rows(w, per_head=16)
        ref = oracle.attn_rows(q, k, v, w.scale, causal=True, rows=rows)
        for path in paths:
            outs = []
            for opts in (dict(snake=1), dict(snake=0), dict(xcd_map=1), dict(xcd_map=2)):
                with G.Options(path=path, **opts):
                    outs.append(G.fwd(q, k, v, w.scale, causal=True))
                assert np.array_equal(outs[-1], outs[0]), (w.name, path, opts)
            assert_parity(outs[0][rows], ref, tolerance(w.n), "order parity %s path %d" % (w.name, path))


def test_padded_batches_sorted_by_length_give_identical_results():
    """Key padding: batch entries are served longest first (ranks recomputed on the device); the order
    is a permutation of the work items, so the bits cannot change.  Ties and zero lengths included."""
    B, H, n, d = 9, 3, 300, 64
    q, k, v = _rand(B, H, n, d, 4242)
    kv_len = np.array([300, 17, 300, 0, 128, 129, 17, 299, 1], np.int32)
    ref = oracle.attn_rows(q, k, v, 0.125, kv_len=kv_len)
    for path in (0, 1):
        outs = []
        for opts in (dict(snake=1), dict(snake=0)):
            with G.Options(path=path, **opts):
                outs.append(G.fwd(q, k, v, 0.125, kv_len=kv_len))
        assert np.array_equal(outs[0], outs[1]), path
        assert_parity(outs[1], ref, tolerance(n), "sorted padded batches path %d" % path)


@pytest.mark.parametrize("causal", [False, True])
def test_packed_sequences_sorted_by_length_give_identical_results(causal):
    """Up to 64 packed sequences are served longest first; more than 64 in list order.  Either way
    the bits are those of the plain order."""
    for lengths in ([700, 3, 512, 0, 129, 700, 64, 1], list(range(1, 71))):
        q, k, v, cu = inputs.make_varlen(4343, H=3, d=64, lengths=lengths)
        ref = oracle.attn_varlen(q, k, v, cu, 0.125, causal=causal)
        outs = []
        for opts in (dict(snake=1), dict(snake=0)):
            with G.Options(**opts):
                outs.append(G.fwd_varlen(q, k, v, cu, max(lengths), 0.125, causal=causal))
        assert np.array_equal(outs[0], outs[1]), len(lengths)
        assert_parity(outs[1].reshape(-1, 64), ref.reshape(-1, 64), tolerance(max(lengths)), "sorted packed sequences")
