"""GPU parity for the head dimensions beyond 32 / 64 / 128: d = 96 and d = 256 on the matrix-core
tiles (FP32 and FP16), the decode kernel, split-KV + combine, packed sequences, rectangular
attention and the streamed evaluation."""
import numpy as np
import pytest

import oracle
from paper_2604_23798_amd import inputs
from tests import gpu_util as G
from tests.parity import assert_parity, tolerance

pytestmark = pytest.mark.gpu
DIMS = [96, 256]


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not G.have_gpu():
        pytest.skip("no GPU")
    from paper_2604_23798_amd import elsa  # noqa: F401


def _qkv(B, H, nq, nk, d, seed, fp16=False, sigma=1.0):
    q = inputs.normal(seed, 0, 0, B * H * nq * d, sigma).reshape(B, H, nq, d)
    k = inputs.normal(seed, 1, 0, B * H * nk * d, sigma).reshape(B, H, nk, d)
    v = inputs.normal(seed, 2, 0, B * H * nk * d).reshape(B, H, nk, d)
    if fp16:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    return q, k, v


f32 = lambda t: t.astype(np.float32)


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("d", DIMS)
def test_square_problems_masks_and_forced_tiles(d, fp16):
    for n in (1, 33, 197, 520):
        q, k, v = _qkv(2, 2, n, n, d, 1100 + n + d, fp16)
        kv_len = np.array([n, max(1, n // 2)], np.int32)
        for causal in (False, True):
            for kl in (None, kv_len):
                ref = oracle.attn_rows(f32(q), f32(k), f32(v), d ** -0.5, causal=causal, kv_len=kl)
                for opts in ({}, dict(path=2, variant=1), dict(path=2, variant=3)) + (
                        (dict(path=3, variant=1), dict(path=3, variant=3)) if fp16 else ()):
                    with G.Options(**opts):
                        out = G.fwd(q, k, v, d ** -0.5, causal=causal, kv_len=kl, masked_entry=True)
                    assert_parity(out, ref, tolerance(n, fp16), "d%d n%d c%d pad%d %s" % (d, n, causal, kl is not None, opts))


@pytest.mark.parametrize("d", DIMS)
def test_wide_scores(d):
    q, k, v = _qkv(1, 2, 300, 300, d, 1200 + d, sigma=4.0)
    ref = oracle.attn_rows(q, k, v, d ** -0.5)
    out = G.fwd(q, k, v, d ** -0.5)
    assert_parity(out, ref, 1e-4, "wide d%d" % d)


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("d", DIMS)
def test_split_kv_states_and_combine(d, fp16):
    import torch
    from paper_2604_23798_amd import elsa
    B, H, n, C = 1, 3, 333, 4
    q, k, v = _qkv(B, H, n, n, d, 1300 + d, fp16)
    pm, pS, pW = G.split_kv(q, k, v, d ** -0.5, C, causal=True)
    m, S, W = G.parts_to_rows(pm, pS, pW)
    rm, rS, rW = oracle.partials_rows(f32(q), f32(k), f32(v), d ** -0.5, C, causal=True)
    live = rS > 0
    assert np.array_equal(live, S > 0)
    tol = tolerance(n, fp16)
    assert np.max(np.abs((m[live] + np.log(S[live])) - (rm[live] + np.log(rS[live])))) < (5e-3 if fp16 else 2e-5)
    assert_parity((W / np.where(live, S, 1)[..., None])[live], (rW / np.where(live, rS, 1)[..., None])[live], tol, "states d%d" % d)
    out = torch.full((B, H, n, d), float("nan"), device="cuda", dtype=torch.float16 if fp16 else torch.float32)
    elsa.elsa_combine(pm, pS, pW, out)
    torch.cuda.synchronize()
    ref = oracle.attn_rows(f32(q), f32(k), f32(v), d ** -0.5, causal=True)
    assert_parity(out.reshape(-1, d).double().cpu().numpy(), ref, tol, "combine d%d" % d)
    # the library's own split with a lent workspace
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)
    try:
        with G.Options(splits=3):
            got = G.fwd(q, k, v, d ** -0.5, causal=True)
    finally:
        elsa.elsa_set_workspace(None)
    assert_parity(got, ref, tol, "internal split d%d" % d)


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("d", DIMS)
def test_rectangular_and_decode(d, fp16):
    import torch
    from paper_2604_23798_amd import elsa
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    for nq, nk in [(1, 2500), (3, 700), (40, 900), (200, 64)]:
        q, k, v = _qkv(2, 2, nq, nk, d, 1400 + nq + d, fp16)
        kv_len = np.array([nk, nk // 3], np.int32)
        ref, ref_lse = oracle.cross_rows(f32(q), f32(k), f32(v), d ** -0.5, causal=True, kv_len=kv_len)
        for lend in (False, True):
            elsa.elsa_set_workspace(ws if lend else None)
            try:
                out, lse = G.fwd_cross(q, k, v, d ** -0.5, causal=True, kv_len=kv_len, want_lse=True)
                if nq <= 4:
                    assert elsa.elsa_last_kernel() == "fma_decode_q1"
            finally:
                elsa.elsa_set_workspace(None)
            assert_parity(out, ref, tolerance(nk, fp16), "cross d%d %dx%d ws%d" % (d, nq, nk, lend))
            vis = np.isfinite(ref_lse)
            assert np.max(np.abs(lse[vis] - ref_lse[vis])) < (5e-3 if fp16 else 2e-5)


@pytest.mark.parametrize("d", DIMS)
def test_packed_sequences(d):
    lengths = [130, 1, 77, 300]
    for fp16 in (False, True):
        q, k, v, cu = inputs.make_varlen(1500 + d, H=2, d=d, fp16=fp16, lengths=lengths)
        ref = oracle.attn_varlen(f32(q), f32(k), f32(v), cu, d ** -0.5, causal=True)
        out = G.fwd_varlen(q, k, v, cu, max(lengths), d ** -0.5, causal=True)
        assert_parity(out.reshape(-1, d), ref.reshape(-1, d), tolerance(300, fp16), "varlen d%d" % d)


@pytest.mark.parametrize("d", DIMS)
def test_streamed_chunks(d):
    import torch
    from paper_2604_23798_amd import elsa
    for fp16 in (False, True):
        for nq in (1, 150):
            B, H, nk = 1, 2, 640
            q, k, v = _qkv(B, H, nq, nk, d, 1600 + nq + d, fp16)
            tq = G.to_dev(q)
            state = torch.empty(elsa.elsa_stream_state_bytes(B, H, nq, d), dtype=torch.uint8, device="cuda")
            k0 = 0
            for ci, nc in enumerate((200, 200, 240)):
                kc = G.to_dev(np.ascontiguousarray(k[:, :, k0:k0 + nc]))
                vc = G.to_dev(np.ascontiguousarray(v[:, :, k0:k0 + nc]))
                elsa.elsa_attn_stream_step(tq, kc, vc, state, d ** -0.5, first=(ci == 0), causal=True,
                                           causal_shift=(nk - nq) - k0)
                k0 += nc
            out = torch.full_like(tq, float("nan"))
            elsa.elsa_attn_stream_finish(state, out)
            torch.cuda.synchronize()
            ref, _ = oracle.cross_rows(f32(q), f32(k), f32(v), d ** -0.5, causal=True)
            assert_parity(out.reshape(-1, d).double().cpu().numpy(), ref, tolerance(nk, fp16), "stream d%d nq%d" % (d, nq))


@pytest.mark.parametrize("d", DIMS)
def test_paths_without_these_head_dimensions_say_so(d):
    q, k, v = _qkv(1, 1, 64, 64, d, 1700)
    for opts in (dict(path=1, variant=1), dict(path=1, variant=4), dict(path=2, variant=10)):
        with G.Options(**opts):
            with pytest.raises(RuntimeError):
                G.fwd(q, k, v, 0.1)
