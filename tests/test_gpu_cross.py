"""GPU parity of rectangular attention (n_q != n_k: cross-attention, chunked prefill, decoding)
through the C ABI, against the FP64 oracle, for every kernel family and both I/O types."""
import numpy as np
import pytest

import oracle
from paper_2604_23798_amd import inputs
from tests import gpu_util as G
from tests.parity import assert_parity, tolerance

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not G.have_gpu():
        pytest.skip("no GPU")
    from paper_2604_23798_amd import elsa  # noqa: F401


def _rect(B, H, nq, nk, d, seed, fp16=False, sigma=1.0):
    q = inputs.normal(seed, 0, 0, B * H * nq * d, sigma).reshape(B, H, nq, d)
    k = inputs.normal(seed, 1, 0, B * H * nk * d, sigma).reshape(B, H, nk, d)
    v = inputs.normal(seed, 2, 0, B * H * nk * d).reshape(B, H, nk, d)
    if fp16:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    return q, k, v


def _ref(q, k, v, scale, **kw):
    f32 = lambda t: t.astype(np.float32)
    return oracle.cross_rows(f32(q), f32(k), f32(v), scale, **kw)


SHAPES = [(1, 777), (5, 300), (37, 2000), (200, 64), (129, 131), (64, 1100), (300, 333)]
KERNELS = [(2, v) for v in range(1, 9)] + [(2, 11), (1, 1), (1, 2)]


@pytest.mark.parametrize("path,variant", KERNELS)
@pytest.mark.parametrize("causal", [False, True])
def test_fp32_kernels_on_rectangular_problems(path, variant, causal):
    for (nq, nk) in SHAPES:
        for d in (64, 128) if (nq + nk) % 2 else (64,):
            q, k, v = _rect(2, 3, nq, nk, d, 100 + nq)
            ref, _ = _ref(q, k, v, d ** -0.5, causal=causal)
            with G.Options(path=path, variant=variant):
                out = G.fwd_cross(q, k, v, d ** -0.5, causal=causal)
            assert_parity(out, ref, tolerance(max(nq, nk), False), "cross p%d v%d %dx%d d%d c%d" % (path, variant, nq, nk, d, causal))


@pytest.mark.parametrize("variant", [1, 2, 3, 4])
@pytest.mark.parametrize("causal", [False, True])
def test_fp16_matrix_core_kernels_on_rectangular_problems(variant, causal):
    for (nq, nk) in SHAPES:
        for d in (32, 64, 128):
            q, k, v = _rect(1, 4, nq, nk, d, 200 + nk, fp16=True)
            ref, _ = _ref(q, k, v, d ** -0.5, causal=causal)
            with G.Options(path=3, variant=variant):
                out = G.fwd_cross(q, k, v, d ** -0.5, causal=causal)
            assert_parity(out, ref, tolerance(max(nq, nk), True), "cross f16 v%d %dx%d d%d c%d" % (variant, nq, nk, d, causal))


@pytest.mark.parametrize("fp16", [False, True])
def test_default_configuration_with_padding_and_lse(fp16):
    B, H, nq, nk, d = 3, 2, 70, 500, 32
    q, k, v = _rect(B, H, nq, nk, d, 301, fp16=fp16)
    kv_len = np.array([500, 33, 0], np.int32)
    for causal in (False, True):
        ref, ref_lse = _ref(q, k, v, 0.2, causal=causal, kv_len=kv_len)
        out, lse = G.fwd_cross(q, k, v, 0.2, causal=causal, kv_len=kv_len, want_lse=True)
        assert_parity(out, ref, tolerance(nk, fp16), "cross padded")
        vis = np.isfinite(ref_lse)
        assert np.all(np.isneginf(lse[~vis])) and np.all(out[~vis] == 0)
        assert np.max(np.abs(lse[vis] - ref_lse[vis])) < (5e-3 if fp16 else 2e-5)


def test_more_queries_than_keys_under_the_causal_mask():
    """n_k < n_q: the first n_q - n_k queries see no key -> zeros, lse = -inf (identity state)."""
    B, H, nq, nk, d = 1, 2, 150, 40, 64
    q, k, v = _rect(B, H, nq, nk, d, 302)
    ref, ref_lse = _ref(q, k, v, 0.125, causal=True)
    for opts in (dict(), dict(path=2, variant=3), dict(path=1, variant=1)):
        with G.Options(**opts):
            out, lse = G.fwd_cross(q, k, v, 0.125, causal=True, want_lse=True)
        assert_parity(out, ref, tolerance(nq, False), "nk<nq")
        blind = np.isneginf(ref_lse)
        assert blind.reshape(B * H, nq)[:, : nq - nk].all() and np.all(out[blind] == 0) and np.all(np.isneginf(lse[blind]))


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("nq", [1, 4, 48])
def test_decoding_with_a_lent_workspace_splits_the_key_range(nq, fp16):
    """Few queries against a long cache: with a workspace the library cuts the keys into chunks,
    emits one state per chunk and merges them (Prop. 1); the result is that of the single pass."""
    import torch
    from paper_2604_23798_amd import elsa
    B, H, nk, d = 2, 4, 9000, 128
    q, k, v = _rect(B, H, nq, nk, d, 303 + nq, fp16=fp16)
    kv_len = np.array([9000, 4097], np.int32)
    ref, ref_lse = _ref(q, k, v, d ** -0.5, causal=True, kv_len=kv_len)
    single = G.fwd_cross(q, k, v, d ** -0.5, causal=True, kv_len=kv_len)
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)
    try:
        out, lse = G.fwd_cross(q, k, v, d ** -0.5, causal=True, kv_len=kv_len, want_lse=True)
        with G.Options(splits=7):
            forced = G.fwd_cross(q, k, v, d ** -0.5, causal=True, kv_len=kv_len)
    finally:
        elsa.elsa_set_workspace(None)
    tol = tolerance(nk, fp16)
    assert_parity(single, ref, tol, "decode single pass")
    assert_parity(out, ref, tol, "decode split")
    assert_parity(forced, ref, tol, "decode 7 chunks")
    assert np.max(np.abs(lse - ref_lse)) < (5e-3 if fp16 else 2e-5)


def test_square_call_through_the_rectangular_entry_point_is_bitwise_the_square_entry_point():
    w = inputs.WORKLOADS["vit_b16_224"]
    q, k, v, _ = inputs.make(w)
    a = G.fwd(q, k, v, w.scale, causal=True)
    b = G.fwd_cross(q, k, v, w.scale, causal=True)
    assert np.array_equal(a, b)


# ---- the vector kernel for one to four queries (decoding) --------------------------------------
@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_decode_kernel_shapes_masks_and_chunks(d, fp16):
    import torch
    from paper_2604_23798_amd import elsa
    ws = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    for nq, nk in [(1, 1), (1, 5), (2, 64), (1, 777), (3, 1000), (4, 4100), (7, 130), (4, 3)]:
        B, H = 2, 3
        q, k, v = _rect(B, H, nq, nk, d, 400 + nq + nk, fp16=fp16)
        kv_len = np.array([nk, max(0, nk // 3)], np.int32)
        for causal in (False, True):
            for kl in (None, kv_len):
                ref, ref_lse = _ref(q, k, v, d ** -0.5, causal=causal, kv_len=kl)
                vis = np.isfinite(ref_lse)
                for variant in (3, 4):
                    for splits in (0, 3):
                        if splits > nk:
                            continue
                        elsa.elsa_set_workspace(ws if splits else None)
                        try:
                            with G.Options(path=1, variant=variant, splits=splits):
                                out, lse = G.fwd_cross(q, k, v, d ** -0.5, causal=causal, kv_len=kl, want_lse=True)
                                assert elsa.elsa_last_kernel() == ("fma_decode_q1" if variant == 3 else "fma_decode_q4")
                        finally:
                            elsa.elsa_set_workspace(None)
                        what = "decode v%d %dx%d d%d c%d pad%d s%d" % (variant, nq, nk, d, causal, kl is not None, splits)
                        assert_parity(out, ref, tolerance(nk, fp16), what)
                        assert np.all(out[~vis] == 0) and np.all(np.isneginf(lse[~vis])), what
                        assert np.max(np.abs(lse[vis] - ref_lse[vis]), initial=0.0) < (5e-3 if fp16 else 2e-5), what


@pytest.mark.parametrize("nq,name", [(1, "fma_decode_q1"), (3, "fma_decode_q4"), (4, "fma_decode_q4"), (5, None)])
def test_decode_kernel_is_the_default_for_up_to_four_queries(nq, name):
    from paper_2604_23798_amd import elsa
    q, k, v = _rect(1, 8, nq, 2048, 64, 500 + nq)
    ref, _ = _ref(q, k, v, 0.125, causal=True)
    out = G.fwd_cross(q, k, v, 0.125, causal=True)
    assert_parity(out, ref, tolerance(2048, False), "default decode nq=%d" % nq)
    last = elsa.elsa_last_kernel()
    assert last == name if name else not last.startswith("fma_decode")


def test_decode_kernel_wide_scores():
    """Scores spread over hundreds of units (sigma = 8 inputs): the lane states must merge without overflow."""
    q, k, v = _rect(1, 4, 1, 6000, 64, 600, sigma=8.0)
    ref, _ = _ref(q, k, v, 0.125)
    out = G.fwd_cross(q, k, v, 0.125)
    assert np.all(np.isfinite(out))
    assert_parity(out, ref, tolerance(6000, False), "decode wide")


def test_decode_kernel_reaches_eight_queries_for_fp32_at_d128():
    from paper_2604_23798_amd import elsa
    for nq, fp16, decode in ((8, False, True), (9, False, False), (8, True, False)):
        q, k, v = _rect(1, 4, nq, 3000, 128, 700 + nq, fp16=fp16)
        ref, _ = _ref(q, k, v, 128 ** -0.5, causal=True)
        out = G.fwd_cross(q, k, v, 128 ** -0.5, causal=True)
        assert_parity(out, ref, tolerance(3000, fp16), "d128 nq=%d fp16=%d" % (nq, fp16))
        assert elsa.elsa_last_kernel().startswith("fma_decode") == decode
        if decode:
            assert elsa.elsa_last_kernel() == "fma_decode_q8"      # one block per (head, chunk): K and V read once


def test_eight_query_decode_kernel_masks_and_chunks():
    import torch
    from paper_2604_23798_amd import elsa
    d = 128
    ws = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    for nq, nk in [(5, 1), (8, 64), (6, 777), (8, 4100), (13, 300), (8, 3)]:
        B, H = 2, 3
        q, k, v = _rect(B, H, nq, nk, d, 800 + nq + nk)
        kv_len = np.array([nk, max(0, nk // 3)], np.int32)
        for causal in (False, True):
            for kl in (None, kv_len):
                ref, ref_lse = _ref(q, k, v, d ** -0.5, causal=causal, kv_len=kl)
                vis = np.isfinite(ref_lse)
                for splits in (0, 3):
                    if splits > nk:
                        continue
                    elsa.elsa_set_workspace(ws if splits else None)
                    try:
                        with G.Options(path=1, variant=5, splits=splits):
                            out, lse = G.fwd_cross(q, k, v, d ** -0.5, causal=causal, kv_len=kl, want_lse=True)
                            assert elsa.elsa_last_kernel() == "fma_decode_q8"
                    finally:
                        elsa.elsa_set_workspace(None)
                    what = "decode q8 %dx%d c%d pad%d s%d" % (nq, nk, causal, kl is not None, splits)
                    assert_parity(out, ref, tolerance(nk, False), what)
                    assert np.all(out[~vis] == 0) and np.all(np.isneginf(lse[~vis])), what
                    assert np.max(np.abs(lse[vis] - ref_lse[vis]), initial=0.0) < 2e-5, what
    # other shapes do not have it
    q, k, v = _rect(1, 1, 8, 64, 64, 5)
    with G.Options(path=1, variant=5), pytest.raises(elsa.ElsaError):
        G.fwd_cross(q, k, v, 0.125)
    q, k, v = _rect(1, 1, 8, 64, 128, 5, fp16=True)
    with G.Options(path=1, variant=5), pytest.raises(elsa.ElsaError):
        G.fwd_cross(q, k, v, 0.1)


@pytest.mark.parametrize("fp16", [False, True])
def test_single_buffered_key_splitting_tile_at_d128(fp16):
    """mfma_xwave32: 32 query rows, four key waves on one 128-key LDS tile that is not doubled (the next
    tile waits in registers): key ranges of one and of many tiles, masks, chunks, more than one query tile."""
    import torch
    from paper_2604_23798_amd import elsa
    d = 128
    ws = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    for nq, nk in [(9, 100), (16, 128), (32, 129), (20, 1000), (32, 4100), (70, 300), (5, 3)]:
        q, k, v = _rect(2, 3, nq, nk, d, 900 + nq + nk, fp16=fp16)
        kv_len = np.array([nk, max(0, nk // 3)], np.int32)
        for causal in (False, True):
            for kl in (None, kv_len):
                ref, ref_lse = _ref(q, k, v, d ** -0.5, causal=causal, kv_len=kl)
                vis = np.isfinite(ref_lse)
                for splits in (0, 3):
                    if splits > nk:
                        continue
                    elsa.elsa_set_workspace(ws if splits else None)
                    try:
                        with G.Options(path=2, variant=12, splits=splits):
                            out, lse = G.fwd_cross(q, k, v, d ** -0.5, causal=causal, kv_len=kl, want_lse=True)
                            assert elsa.elsa_last_kernel() == "mfma_xwave32"
                    finally:
                        elsa.elsa_set_workspace(None)
                    what = "xwave32 %dx%d c%d pad%d s%d fp16=%d" % (nq, nk, causal, kl is not None, splits, fp16)
                    assert_parity(out, ref, tolerance(nk, fp16), what)
                    assert np.all(out[~vis] == 0) and np.all(np.isneginf(lse[~vis])), what
    # the default for 9 .. 32 FP32 queries against a long cache at d = 128; other head dimensions do not have it
    q, k, v = _rect(1, 4, 16, 3000, d, 950)
    G.fwd_cross(q, k, v, d ** -0.5, causal=True)
    assert elsa.elsa_last_kernel() == "mfma_xwave32"
    q, k, v = _rect(1, 1, 16, 64, 64, 5)
    with G.Options(path=2, variant=12), pytest.raises(elsa.ElsaError):
        G.fwd_cross(q, k, v, 0.125)


@pytest.mark.parametrize("fp16", [False, True])
def test_single_buffered_64_row_tile_at_d128(fp16):
    """mfma_q64_xw2_sb: the 64-row tile of two query waves x two key waves with one LDS buffer instead of two
    (two blocks per CU at d = 128): square and rectangular problems, masks, chunks, ragged tails."""
    import torch
    from paper_2604_23798_amd import elsa
    d = 128
    ws = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    for nq, nk in [(64, 64), (65, 65), (300, 300), (130, 1000), (1, 70), (200, 63)]:
        q, k, v = _rect(2, 3, nq, nk, d, 1900 + nq + nk, fp16=fp16)
        kv_len = np.array([nk, max(0, nk // 3)], np.int32)
        for causal in (False, True):
            for kl in (None, kv_len):
                ref, ref_lse = _ref(q, k, v, d ** -0.5, causal=causal, kv_len=kl)
                vis = np.isfinite(ref_lse)
                for splits in (0, 3):
                    if splits > nk:
                        continue
                    elsa.elsa_set_workspace(ws if splits else None)
                    try:
                        with G.Options(path=2, variant=13, splits=splits):
                            out, lse = G.fwd_cross(q, k, v, d ** -0.5, causal=causal, kv_len=kl, want_lse=True)
                            assert elsa.elsa_last_kernel() == "mfma_q64_xw2_sb"
                    finally:
                        elsa.elsa_set_workspace(None)
                    what = "q64_xw2_sb %dx%d c%d pad%d s%d fp16=%d" % (nq, nk, causal, kl is not None, splits, fp16)
                    assert_parity(out, ref, tolerance(nk, fp16), what)
                    assert np.all(out[~vis] == 0) and np.all(np.isneginf(lse[~vis])), what
    # the library's own choice for a causal launch of a few runs of blocks at d = 128; other head dimensions do not have the tile
    q, k, v = _rect(1, 40, 1024, 1024, d, 1950)
    rows = np.arange(0, 40 * 1024, 97, dtype=np.int64)
    ref, _ = oracle.dv_rows(q, k, v, d ** -0.5, causal=True, rows=rows)
    out = G.fwd_cross(q, k, v, d ** -0.5, causal=True)
    assert elsa.elsa_last_kernel() == "mfma_q64_xw2_sb"
    assert_parity(out[rows], ref, tolerance(1024), "q64_xw2_sb as the default")
    q, k, v = _rect(1, 1, 16, 64, 64, 5)
    with G.Options(path=2, variant=13), pytest.raises(elsa.ElsaError):
        G.fwd_cross(q, k, v, 0.125)
