"""elsa_attn_fwd_static: the internal key split with its chunk states in the library's own device array.

Checked against the existing entry point it is a variant of (elsa_attn_fwd_masked with a lent workspace
and the same number of key chunks: same kernels, so the outputs must be bit-identical) and against the
oracle, on two calls in a row -- the second on a smaller input, which finds the array still holding the
first call's states."""
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


def _problem(B, H, n, d, seed, fp16):
    cnt, sh = B * H * n * d, (B, H, n, d)
    q, k, v = (inputs.normal(seed, s, 0, cnt).reshape(sh) for s in (0, 1, 2))
    if fp16:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    return q, k, v


def _static(q, k, v, scale, causal, kv_len, splits):
    import torch
    from paper_2604_23798_amd import elsa
    tq, tk, tv, tl = G.to_dev(q), G.to_dev(k), G.to_dev(v), G.to_dev(kv_len)
    out = torch.full_like(tq, float("nan"))
    elsa.elsa_attn_fwd_static(tq, tk, tv, out, scale, causal, tl, splits)
    torch.cuda.synchronize()
    return out.reshape(-1, q.shape[-1]).double().cpu().numpy(), elsa.elsa_last_kernel(), elsa.elsa_last_splits()


def _lent(q, k, v, scale, causal, kv_len, splits):
    import torch
    from paper_2604_23798_amd import elsa
    ws = torch.empty(elsa.elsa_static_scratch_bytes(), dtype=torch.uint8, device="cuda")
    elsa.elsa_set_workspace(ws)
    try:
        with G.Options(splits=splits):
            out = G.fwd(q, k, v, scale, causal=causal, kv_len=kv_len, masked_entry=True)
            return out, elsa.elsa_last_kernel(), elsa.elsa_last_splits()
    finally:
        elsa.elsa_set_workspace(None)


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("splits", [0, 3])
def test_static_scratch_matches_the_lent_workspace_on_two_calls_in_a_row(splits, fp16):
    cases = [  # (B, H, n, d, causal, kv_len): the second problem is smaller than the first
        (2, 6, 1100, 64, False, np.array([1100, 700], np.int32)),
        (1, 5, 333, 64, True, None),
    ]
    for (B, H, n, d, causal, kv_len) in cases:
        q, k, v = _problem(B, H, n, d, 1400 + n, fp16)
        scale = d ** -0.5
        got, kern, C = _static(q, k, v, scale, causal, kv_len, splits)
        want, kern_w, C_w = _lent(q, k, v, scale, causal, kv_len, splits)
        assert (kern, C) == (kern_w, C_w), (kern, C, kern_w, C_w)
        if splits:
            assert C == splits
        assert np.array_equal(got, want), "static scratch and lent workspace differ (n=%d splits=%d fp16=%d)" % (n, C, fp16)
        f32 = lambda t: t.astype(np.float32)
        ref = oracle.attn_rows(f32(q), f32(k), f32(v), scale, causal=causal, kv_len=kv_len)
        assert_parity(got, ref, tolerance(n, fp16), "static scratch n=%d splits=%d kernel=%s" % (n, C, kern))


def test_static_scratch_limits_and_decoding_shape():
    import torch
    from paper_2604_23798_amd import elsa
    # a request whose chunk states exceed the array is refused before anything is launched
    assert elsa.elsa_static_scratch_bytes() == 64 << 20
    q = torch.zeros((1, 64, 4096, 128), device="cuda")
    out = torch.full_like(q, float("nan"))
    assert elsa.elsa_split_kv_workspace_bytes(1, 64, 4096, 128, 2) > elsa.elsa_static_scratch_bytes()
    with pytest.raises(elsa.ElsaError) as e:
        elsa.elsa_attn_fwd_static(q, q, q, out, 0.1, False, None, 2)
    assert e.value.code == elsa.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool(torch.isnan(out).all())
    with pytest.raises(elsa.ElsaError):
        elsa.elsa_attn_fwd_static(q, q, q, out, 0.1, False, None, -1)
    # one pass needs no scratch at any size
    elsa.elsa_attn_fwd_static(q, q, q, out, 0.1, False, None, 1)
    torch.cuda.synchronize()
    assert bool((out == 0).all()) and elsa.elsa_last_splits() == 1
