"""GPU parity of attention whose values have their own width (d_v != d) through the C ABI, against
the FP64 oracle: every (d, d_v) pair served, both tiles, both I/O types, masks, key split."""
import numpy as np
import pytest

import oracle
from paper_2604_23798_amd import inputs
from tests import gpu_util as G
from tests.parity import assert_parity, tolerance

pytestmark = pytest.mark.gpu

PAIRS = [(32, 64), (32, 128), (64, 32), (64, 128), (128, 32), (128, 64), (192, 128)]


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not G.have_gpu():
        pytest.skip("no GPU")
    from paper_2604_23798_amd import elsa  # noqa: F401


def _rect(B, H, nq, nk, d, dv, seed, fp16=False, sigma=1.0):
    q = inputs.normal(seed, 0, 0, B * H * nq * d, sigma).reshape(B, H, nq, d)
    k = inputs.normal(seed, 1, 0, B * H * nk * d, sigma).reshape(B, H, nk, d)
    v = inputs.normal(seed, 2, 0, B * H * nk * dv).reshape(B, H, nk, dv)
    if fp16:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    return q, k, v


def _ref(q, k, v, scale, **kw):
    f32 = lambda t: t.astype(np.float32)
    return oracle.dv_rows(f32(q), f32(k), f32(v), scale, **kw)


# several tiles and a ragged tail in both directions, one query, more queries than keys
SHAPES = [(1, 777), (37, 2000), (200, 64), (129, 131), (300, 333), (515, 515)]


@pytest.mark.parametrize("d,dv", PAIRS)
@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("variant", [1, 3, 6])
def test_every_pair_on_both_tiles(d, dv, fp16, variant):
    from paper_2604_23798_amd import elsa
    if variant == 6 and not (fp16 and max(d, dv) >= 128):
        # the 256-row tile of eight query waves exists for FP16 tiles with a 128-wide (or wider) operand only
        q, k, v = _rect(1, 1, 8, 8, d, dv, 1, fp16=fp16)
        with G.Options(variant=6), pytest.raises(elsa.ElsaError) as e:
            G.fwd_dv(q, k, v, 0.1)
        assert e.value.code == elsa.ERR_UNSUPPORTED
        return
    if variant == 3 and d == 192 and not fp16:
        q, k, v = _rect(1, 1, 8, 8, d, dv, 1)
        with G.Options(variant=3), pytest.raises(elsa.ElsaError) as e:
            G.fwd_dv(q, k, v, 0.1)
        assert e.value.code == elsa.ERR_UNSUPPORTED
        return
    for (nq, nk) in SHAPES:
        for causal in (False, True):
            print("dv case d=%d dv=%d fp16=%d variant=%d nq=%d nk=%d causal=%d" % (d, dv, fp16, variant, nq, nk, causal), flush=True)
            q, k, v = _rect(2, 3, nq, nk, d, dv, 400 + nq + d, fp16=fp16)
            ref, ref_lse = _ref(q, k, v, d ** -0.5, causal=causal)
            with G.Options(variant=variant):
                out, lse = G.fwd_dv(q, k, v, d ** -0.5, causal=causal, want_lse=True)
                name = elsa.elsa_last_kernel()
            assert name == ("mfma16_dv_" if fp16 else "mfma_dv_") + {1: "q128", 3: "xwave", 6: "q256_w8"}[variant]
            assert out.shape == ref.shape
            assert_parity(out, ref, tolerance(max(nq, nk), fp16), "dv %s %dx%d d%d dv%d c%d" % (name, nq, nk, d, dv, causal))
            vis = np.isfinite(ref_lse)
            assert np.all(np.isneginf(lse[~vis])) and np.all(out[~vis] == 0)
            assert np.max(np.abs(lse[vis] - ref_lse[vis]), initial=0.0) < (5e-3 if fp16 else 2e-5)


@pytest.mark.parametrize("fp16", [False, True])
def test_fp16_io_on_the_fp32_tiles_and_zero_scale(fp16):
    """ELSA_OPT_PATH = 2 keeps FP16 I/O on the FP32 matrix-core tiles; scale = 0 (uniform weights:
    the output is the mean of the visible value rows) takes the same tiles by itself."""
    from paper_2604_23798_amd import elsa
    d, dv = 64, 128
    q, k, v = _rect(1, 2, 150, 260, d, dv, 431, fp16=fp16)
    ref, _ = _ref(q, k, v, 0.125, causal=True)
    with G.Options(path=2):
        out = G.fwd_dv(q, k, v, 0.125, causal=True)
        assert elsa.elsa_last_kernel().startswith("mfma_dv_")
    assert_parity(out, ref, tolerance(260, fp16), "dv path 2")
    out0 = G.fwd_dv(q, k, v, 0.0)
    assert elsa.elsa_last_kernel().startswith("mfma_dv_")
    mean = v.astype(np.float64).mean(axis=2, keepdims=True).repeat(150, axis=2).reshape(-1, dv)
    assert_parity(out0, mean, tolerance(260, fp16), "dv scale 0")


@pytest.mark.parametrize("fp16", [False, True])
def test_key_padding_sorted_batches_and_empty_entries(fp16):
    B, H, nq, nk, d, dv = 5, 2, 140, 600, 128, 64
    q, k, v = _rect(B, H, nq, nk, d, dv, 433, fp16=fp16)
    kv_len = np.array([600, 33, 0, 412, 1], np.int32)
    for causal in (False, True):
        ref, ref_lse = _ref(q, k, v, 0.2, causal=causal, kv_len=kv_len)
        out, lse = G.fwd_dv(q, k, v, 0.2, causal=causal, kv_len=kv_len, want_lse=True)
        assert_parity(out, ref, tolerance(nk, fp16), "dv padded")
        vis = np.isfinite(ref_lse)
        assert np.all(np.isneginf(lse[~vis])) and np.all(out[~vis] == 0)
        with G.Options(snake=1):
            plain = G.fwd_dv(q, k, v, 0.2, causal=causal, kv_len=kv_len)
        assert np.array_equal(plain, out)        # the work order is a permutation: bit-identical


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("d,dv,nq", [(192, 128, 1), (64, 128, 4), (128, 64, 48), (32, 64, 300)])
def test_lent_workspace_splits_the_key_range(d, dv, nq, fp16):
    """With a workspace the key range is cut into chunks whose states (W of width d_v) are merged
    by the combine kernel (Prop. 1): same result as the single pass."""
    import torch
    from paper_2604_23798_amd import elsa
    B, H, nk = 2, 3, 5000
    q, k, v = _rect(B, H, nq, nk, d, dv, 435 + nq, fp16=fp16)
    kv_len = np.array([5000, 2049], np.int32)
    ref, ref_lse = _ref(q, k, v, d ** -0.5, causal=True, kv_len=kv_len)
    single = G.fwd_dv(q, k, v, d ** -0.5, causal=True, kv_len=kv_len)
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)
    try:
        out, lse = G.fwd_dv(q, k, v, d ** -0.5, causal=True, kv_len=kv_len, want_lse=True)
        with G.Options(splits=5):
            forced = G.fwd_dv(q, k, v, d ** -0.5, causal=True, kv_len=kv_len)
    finally:
        elsa.elsa_set_workspace(None)
    tol = tolerance(nk, fp16)
    assert_parity(single, ref, tol, "dv single pass")
    assert_parity(out, ref, tol, "dv split")
    assert_parity(forced, ref, tol, "dv 5 chunks")
    assert np.max(np.abs(lse - ref_lse)) < (5e-3 if fp16 else 2e-5)


def test_equal_widths_are_the_rectangular_entry_point_bitwise():
    q, k, v = _rect(1, 4, 130, 500, 64, 64, 437)
    a = G.fwd_dv(q, k, v, 0.125, causal=True)
    b = G.fwd_cross(q, k, v, 0.125, causal=True)
    assert np.array_equal(a, b)


def test_value_blocks_are_independent():
    """out(V = [V1 | V2]) = [out(V1) | out(V2)] -- against the d_v = d entry point on each block."""
    d = 64
    q, k, v = _rect(2, 2, 200, 700, d, 2 * d, 439)
    wide = G.fwd_dv(q, k, v, 0.125, causal=True)
    for blk in range(2):
        part = G.fwd_cross(q, k, np.ascontiguousarray(v[..., blk * d:(blk + 1) * d]), 0.125, causal=True)
        assert np.max(np.abs(wide[:, blk * d:(blk + 1) * d] - part)) < 2e-6


def test_rejected_arguments():
    from paper_2604_23798_amd import elsa
    for d, dv in ((64, 96), (96, 64), (192, 64), (256, 128), (64, 192), (48, 64)):
        q, k, v = _rect(1, 1, 8, 8, d, dv, 3)
        with pytest.raises(elsa.ElsaError) as e:
            G.fwd_dv(q, k, v, 0.1)
        assert e.value.code == elsa.ERR_UNSUPPORTED
    q, k, v = _rect(1, 1, 8, 8, 64, 128, 3)
    for opts in (dict(path=1), dict(variant=2), dict(variant=7)):
        with G.Options(**opts), pytest.raises(elsa.ElsaError) as e:
            G.fwd_dv(q, k, v, 0.1)
        assert e.value.code == elsa.ERR_UNSUPPORTED
    with pytest.raises(elsa.ElsaError) as e:
        G.fwd_dv(q, k, v, float("nan"))
    assert e.value.code == elsa.ERR_INVALID_ARG
