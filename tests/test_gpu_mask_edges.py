"""A masked key is the identity element of the monoid -- whatever its K and V rows hold.

Padded batches keep garbage in the rows at or beyond ``kv_len[b]``.  The oracle skips those keys; the
kernels must behave as if they did: for every kernel family and entry point the output with NaN and
+-Inf planted in the padded rows must equal, bit for bit, the output with zeros there, and match the
oracle.  Also pinned here: scaling V by a power of two scales the output by the same power of two bit
for bit (the weights never depend on V), and the treatment of FP32-denormal value entries."""
import numpy as np
import pytest

import oracle
from paper_2604_23798_amd import inputs
from tests import gpu_util as G
from tests.parity import assert_parity, tolerance

pytestmark = pytest.mark.gpu

MFMA, FMA, MFMA16 = 2, 1, 3


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not G.have_gpu():
        pytest.skip("no GPU")
    from paper_2604_23798_amd import elsa  # noqa: F401


def _qkv(B, H, nq, nk, d, dv, seed, fp16=False):
    q = inputs.normal(seed, 0, 0, B * H * nq * d).reshape(B, H, nq, d)
    k = inputs.normal(seed, 1, 0, B * H * nk * d).reshape(B, H, nk, d)
    v = inputs.normal(seed, 2, 0, B * H * nk * dv).reshape(B, H, nk, dv)
    if fp16:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    return q, k, v


# what the padded rows hold: (K filler, V filler); zeros are the reference
POISONS = [("nan", np.nan, np.nan), ("+inf", np.inf, np.inf), ("-inf", -np.inf, -np.inf), ("mixed", np.inf, np.nan)]


def _filled(k, v, kv_len, kfill, vfill):
    k2, v2 = k.copy(), v.copy()
    for b, L in enumerate(kv_len):
        L = max(0, min(int(L), k.shape[2]))
        k2[b, :, L:] = kfill
        v2[b, :, L:] = vfill
    return k2, v2


def _f32(*ts):
    return tuple(t.astype(np.float32) for t in ts)


def _check_masked(q, k, v, kv_len, scale, causal, tol, what, run):
    """``run(k, v)`` -> float64 [R, dv] through the HIP path; compares poisoned runs with the zero-filled one."""
    kz, vz = _filled(k, v, kv_len, 0.0, 0.0)
    base = run(kz, vz)
    assert np.all(np.isfinite(base)), what
    for name, kf, vf in POISONS:
        kp, vp = _filled(k, v, kv_len, kf, vf)
        got = run(kp, vp)
        assert np.array_equal(got, base), "%s: padded rows holding %s change the output" % (what, name)
    return base


SQUARE_KERNELS = ([(MFMA, i, 64, False) for i in range(1, 12)] + [(MFMA, i, 128, False) for i in (1, 3, 11, 12, 13)] +
                  [(MFMA, 1, 32, False), (MFMA, 10, 32, False), (MFMA, 1, 96, False), (MFMA, 3, 96, False), (MFMA, 1, 256, False)] +
                  [(MFMA, 1, 64, True), (MFMA, 3, 64, True)] +
                  [(FMA, 1, 64, False), (FMA, 2, 64, False), (FMA, 1, 128, False), (FMA, 1, 64, True)] +
                  [(MFMA16, i, 64, True) for i in (1, 2, 3, 4)] + [(MFMA16, i, 128, True) for i in (1, 3, 4)] +
                  [(MFMA16, 1, 96, True), (MFMA16, 1, 256, True), (MFMA16, 1, 32, True)])


@pytest.mark.parametrize("path,variant,d,fp16", SQUARE_KERNELS)
def test_padded_rows_may_hold_anything_square(path, variant, d, fp16):
    """elsa_attn_fwd_masked, every tile configuration: lengths that end inside a 32-key step, on a step
    boundary, at one key and at none."""
    B, H, n = 5, 2, 333
    q, k, v = _qkv(B, H, n, n, d, d, 500 + d, fp16)
    kv_len = np.array([n, 77, 1, 0, 256], np.int32)
    scale = d ** -0.5
    for causal in (False, True):
        def run(kk, vv):
            with G.Options(path=path, variant=variant):
                return G.fwd(q, kk, vv, scale, causal=causal, kv_len=kv_len)
        what = "path%d v%d d%d fp16=%d causal=%d" % (path, variant, d, fp16, causal)
        base = _check_masked(q, k, v, kv_len, scale, causal, tolerance(n, fp16), what, run)
        ref = oracle.attn_rows(*_f32(q, k, v), scale, causal=causal, kv_len=kv_len)
        assert_parity(base, ref, tolerance(n, fp16), what)
        assert np.all(base.reshape(B, H, n, d)[3] == 0.0)


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("nq,d", [(1, 64), (1, 128), (3, 64), (4, 128), (7, 128), (1, 96), (1, 256), (16, 64), (24, 128), (40, 64)])
def test_padded_rows_may_hold_anything_decoding(nq, d, fp16):
    """elsa_attn_fwd_cross with few queries against many keys: the streaming vector kernels (one, four,
    eight queries per block) and the key-splitting matrix-core tiles, with and without an internal key split."""
    import torch
    from paper_2604_23798_amd import elsa
    B, H, nk = 3, 2, 1500
    q, k, v = _qkv(B, H, nq, nk, d, d, 600 + nq + d, fp16)
    kv_len = np.array([nk, 701, 5], np.int32)
    scale = d ** -0.5
    ref, _ = oracle.cross_rows(*_f32(q, k, v), scale, causal=False, kv_len=kv_len)
    for lend in (False, True):
        ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda") if lend else None
        elsa.elsa_set_workspace(ws)
        try:
            names = []

            def run(kk, vv):
                o = G.fwd_cross(q, kk, vv, scale, kv_len=kv_len)
                names.append((elsa.elsa_last_kernel(), elsa.elsa_last_splits()))
                return o
            what = "decode nq=%d d=%d fp16=%d workspace=%d" % (nq, d, fp16, lend)
            base = _check_masked(q, k, v, kv_len, scale, False, tolerance(nk, fp16), what, run)
        finally:
            elsa.elsa_set_workspace(None)
        print(what, names[0])
        assert_parity(base, ref, tolerance(nk, fp16), what)


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("d,dv", [(64, 128), (128, 64), (32, 64), (192, 128)])
def test_padded_rows_may_hold_anything_value_width(d, dv, fp16):
    B, H, nq, nk = 3, 2, 150, 290
    q, k, v = _qkv(B, H, nq, nk, d, dv, 700 + d + dv, fp16)
    kv_len = np.array([nk, 100, 33], np.int32)
    scale = d ** -0.5
    for causal in (False, True):
        for variant in (1, 3):
            if variant == 3 and d == 192 and not fp16:
                continue                      # no key-splitting FP32 tile at this width
            def run(kk, vv):
                with G.Options(variant=variant):
                    return G.fwd_dv(q, kk, vv, scale, causal=causal, kv_len=kv_len)
            what = "dv d=%d dv=%d fp16=%d causal=%d variant=%d" % (d, dv, fp16, causal, variant)
            base = _check_masked(q, k, v, kv_len, scale, causal, tolerance(nk, fp16), what, run)
            ref, _ = oracle.dv_rows(*_f32(q, k, v), scale, causal=causal, kv_len=kv_len)
            assert_parity(base, ref, tolerance(nk, fp16), what)


@pytest.mark.parametrize("path,variant,fp16", [(MFMA, 1, False), (MFMA, 3, False), (MFMA, 7, False), (FMA, 1, False), (FMA, 2, False),
                                               (MFMA16, 1, True), (MFMA16, 3, True)])
def test_padded_rows_may_hold_anything_chunk_states(path, variant, fp16):
    """elsa_attn_fwd_split_kv: the states of chunks that a length cuts short or empties."""
    B, H, n, d, C = 3, 2, 300, 64, 4
    q, k, v = _qkv(B, H, n, n, d, d, 800, fp16)
    kv_len = np.array([n, 80, 151], np.int32)

    def states(kk, vv):
        with G.Options(path=path, variant=variant):
            pm, pS, pW = G.split_kv(q, kk, vv, 0.125, C, kv_len=kv_len)
        return [t.cpu().numpy() for t in (pm, pS, pW)]
    kz, vz = _filled(k, v, kv_len, 0.0, 0.0)
    base = states(kz, vz)
    for name, kf, vf in POISONS:
        got = states(*_filled(k, v, kv_len, kf, vf))
        for a, b in zip(got, base):
            assert np.array_equal(a, b), (name, path, variant)
    om, oS, oW = oracle.partials_rows(*_f32(q, k, v), 0.125, C, kv_len=kv_len)
    gm = base[0].transpose(0, 1, 3, 2).reshape(-1, C)
    assert np.array_equal(np.isneginf(gm), np.isneginf(om))


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("nq,d", [(200, 64), (2, 128), (160, 128)])
def test_padded_rows_may_hold_anything_streamed_chunks(nq, d, fp16):
    """elsa_attn_stream_step with a kv_len per chunk: the padded rows of every chunk are poisoned."""
    import torch
    from paper_2604_23798_amd import elsa
    B, H, chunks, nc = 2, 2, 3, 130
    nk = chunks * nc
    q, k, v = _qkv(B, H, nq, nk, d, d, 900 + nq, fp16)
    lens = np.array([[nc, 57], [100, 0], [1, nc]], np.int32)      # [chunk][batch]
    scale = d ** -0.5

    def run(fill_k, fill_v):
        tq = G.to_dev(q)
        state = torch.empty(elsa.elsa_stream_state_bytes(B, H, nq, d), dtype=torch.uint8, device="cuda")
        for c in range(chunks):
            kc, vc = k[:, :, c * nc:(c + 1) * nc].copy(), v[:, :, c * nc:(c + 1) * nc].copy()
            kc, vc = _filled(kc, vc, lens[c], fill_k, fill_v)
            elsa.elsa_attn_stream_step(tq, G.to_dev(kc), G.to_dev(vc), state, scale, first=(c == 0), kv_len=G.to_dev(lens[c]))
        out = torch.full_like(tq, float("nan"))
        elsa.elsa_attn_stream_finish(state, out)
        torch.cuda.synchronize()
        return out.reshape(-1, d).double().cpu().numpy()
    base = run(0.0, 0.0)
    for name, kf, vf in POISONS:
        assert np.array_equal(run(kf, vf), base), (name, nq, d, fp16)
    # the oracle on the visible keys of every chunk, gathered into one dense problem per batch entry
    qf, kf_, vf_ = _f32(q, k, v)
    for b in range(B):
        keep = np.concatenate([np.arange(c * nc, c * nc + lens[c][b]) for c in range(chunks)])
        ref, _ = oracle.cross_rows(qf[b:b + 1], kf_[b:b + 1][:, :, keep], vf_[b:b + 1][:, :, keep], scale)
        assert_parity(base.reshape(B, H * nq, d)[b], ref, tolerance(nk, fp16), "streamed chunks b=%d" % b)


def test_padded_rows_may_hold_anything_internal_split():
    """elsa_attn_fwd_masked with a lent workspace (the library cuts the keys itself), FP32 and FP16."""
    import torch
    from paper_2604_23798_amd import elsa
    B, H, n, d = 2, 4, 1100, 64
    kv_len = np.array([n, 515], np.int32)
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)
    try:
        for fp16 in (False, True):
            q, k, v = _qkv(B, H, n, n, d, d, 1000, fp16)
            for splits in (0, 3):
                def run(kk, vv):
                    with G.Options(splits=splits):
                        return G.fwd(q, kk, vv, 0.125, kv_len=kv_len)
                base = _check_masked(q, k, v, kv_len, 0.125, False, tolerance(n, fp16), "internal split %d fp16=%d" % (splits, fp16), run)
                assert_parity(base, oracle.attn_rows(*_f32(q, k, v), 0.125, kv_len=kv_len), tolerance(n, fp16), "internal split")
    finally:
        elsa.elsa_set_workspace(None)


SCALE_KERNELS = [(MFMA, 1), (MFMA, 2), (MFMA, 3), (MFMA, 4), (MFMA, 7), (MFMA, 9), (MFMA, 10), (MFMA, 11), (FMA, 1), (FMA, 2)]


@pytest.mark.parametrize("path,variant", SCALE_KERNELS)
def test_value_scale_equivariance_fp32(path, variant):
    """out(2^k V) = 2^k out(V), bit for bit: the weights do not depend on V and every operation applied
    to V (products with weights, sums, the final division) commutes with an exact power-of-two scaling
    as long as nothing leaves the FP32 normal range."""
    B, H, n, d = 1, 3, 333, 64
    q, k, v = _qkv(B, H, n, n, d, d, 1100)
    for causal in (False, True):
        with G.Options(path=path, variant=variant):
            base = G.fwd(q, k, v, 0.125, causal=causal)
            for e in (20, -20):
                got = G.fwd(q, k, (v * np.float32(2.0 ** e)).astype(np.float32), 0.125, causal=causal)
                assert np.array_equal(got, base * 2.0 ** e), (path, variant, e, causal)


def test_value_scale_equivariance_few_queries_and_chunks():
    import torch
    from paper_2604_23798_amd import elsa
    B, H, nk, d = 2, 2, 2000, 128
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)
    try:
        for nq in (1, 4, 8, 16):
            q, k, v = _qkv(B, H, nq, nk, d, d, 1200 + nq)
            base = G.fwd_cross(q, k, v, 0.09, causal=True)
            got = G.fwd_cross(q, k, (v * np.float32(2.0 ** 20)).astype(np.float32), 0.09, causal=True)
            assert elsa.elsa_last_splits() > 1
            assert np.array_equal(got, base * 2.0 ** 20), nq
    finally:
        elsa.elsa_set_workspace(None)


@pytest.mark.parametrize("variant", [1, 2, 3, 4])
def test_value_scale_equivariance_fp16(variant):
    """FP16 I/O: V * 8 stays exact in FP16; the output scales exactly wherever both results are FP16 normals."""
    B, H, n, d = 1, 3, 333, 64
    q, k, v = _qkv(B, H, n, n, d, d, 1300, fp16=True)
    with G.Options(path=MFMA16, variant=variant):
        base = G.fwd(q, k, v, 0.125)
        got = G.fwd(q, k, (v.astype(np.float32) * 8).astype(np.float16), 0.125)
    ok = (np.abs(base) >= 2.0 ** -14) & (np.abs(got) < 65504)
    assert ok.mean() > 0.99
    assert np.array_equal(got[ok], base[ok] * 8.0)


DENORMAL_KERNELS = [(MFMA, 1), (MFMA, 3), (MFMA, 7), (MFMA, 9), (MFMA, 10), (MFMA, 11), (FMA, 1), (FMA, 2)]


@pytest.mark.parametrize("path,variant", DENORMAL_KERNELS)
def test_fp32_denormal_values_are_preserved(path, variant):
    """Policy for value entries below the FP32 normal range (1.18e-38): they are NOT flushed.  The FP32
    matrix-core and vector instructions that touch V (products with weights, sums, the final scaling)
    keep denormals; only the exponentials flush (a weight below the normal range becomes 0, which drops
    at most n * 1.2e-38 of mass).  A value column that is constant at a denormal c must therefore come
    out as c, not as 0 -- to within the roundings of some hundred products and sums that themselves fall
    into the denormal range (spacing 1.4e-45)."""
    B, H, n, d = 1, 2, 200, 64
    q, k, v = _qkv(B, H, n, n, d, d, 1500)
    tiny = np.float32(1.401298464324817e-45)
    v[..., 0] = np.float32(1e-40)
    v[..., 1] = np.float32(-3e-39)
    v[..., 2] = np.float32(1.5e-38)              # just inside the normal range
    with G.Options(path=path, variant=variant):
        out = G.fwd(q, k, v, 0.125)
    for col in range(3):
        c = float(v[0, 0, 0, col])
        assert np.all(np.abs(out[:, col] - c) <= 64 * float(tiny)), (path, variant, col, out[:2, col])


def test_fp32_denormal_values_are_preserved_when_decoding_and_combining():
    import torch
    from paper_2604_23798_amd import elsa
    B, H, nk, d = 1, 2, 900, 64
    tiny = 1.401298464324817e-45
    for nq in (1, 4):
        q, k, v = _qkv(B, H, nq, nk, d, d, 1600 + nq)
        v[..., 0] = np.float32(1e-40)
        ws = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")
        elsa.elsa_set_workspace(ws)
        try:
            out = G.fwd_cross(q, k, v, 0.125)
            assert elsa.elsa_last_splits() > 1 and elsa.elsa_last_kernel().startswith("fma_decode")
        finally:
            elsa.elsa_set_workspace(None)
        assert np.all(np.abs(out[:, 0] - float(np.float32(1e-40))) <= 64 * tiny), out[:, 0]
