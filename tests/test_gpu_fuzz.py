"""Seeded random sweep over shapes, masks, options and entry points (all inputs valid), every case
checked against the FP64 oracle.  Meant to catch interactions that the structured tests do not
enumerate: work orders x key chunks x masks x tile shapes x head dimensions."""
import os

import numpy as np
import pytest

import oracle
from paper_2604_23798_amd import inputs
from tests import gpu_util as G
from tests.parity import assert_parity, tolerance

pytestmark = pytest.mark.gpu
f32 = lambda t: t.astype(np.float32)
# ELSA_FUZZ_OFFSET=k shifts every generator seed by k: other cases of the same distributions (default 0)
OFFSET = 100000 * int(os.environ.get("ELSA_FUZZ_OFFSET", "0"))


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not G.have_gpu():
        pytest.skip("no GPU")
    from paper_2604_23798_amd import elsa  # noqa: F401


def _case(rng):
    d = int(rng.choice([32, 64, 64, 96, 128, 256]))
    fp16 = bool(rng.integers(0, 2))
    B = int(rng.integers(1, 5))
    H = int(rng.integers(1, 5))
    kind = rng.choice(["square", "square", "cross", "decode", "varlen", "stream"])
    causal = bool(rng.integers(0, 2))
    nk = int(rng.choice([1, 7, 31, 32, 33, 64, 100, 129, 257, 500, 777, 1300]))
    if kind == "square":
        nq = nk
    elif kind == "decode":
        nq = int(rng.integers(1, 9))
    else:
        nq = int(rng.choice([1, 5, 9, 17, 32, 33, 64, 130, 300]))
    use_len = bool(rng.integers(0, 2)) and kind in ("square", "cross", "decode")
    kv_len = rng.integers(0, nk + 1, size=B).astype(np.int32) if use_len else None
    opts = {}
    wide = d in (96, 256)
    r = rng.integers(0, 4)
    if r == 1:
        opts = dict(path=2, variant=int(rng.choice([1, 3] if wide else [1, 2, 3, 4, 7, 8, 11] + ([12, 13] if d == 128 else []))))
    elif r == 2 and fp16:
        opts = dict(path=3, variant=int(rng.choice([1, 2, 3, 4] + ([6] if d >= 96 else []))))
    elif r == 3 and not wide:
        opts = dict(path=1, variant=int(rng.choice([1, 2])))
    opts["snake"] = int(rng.integers(0, 2))
    opts["xcd_map"] = int(rng.choice([0, 0, 1, 2]))
    splits = int(rng.choice([0, 0, 2, 3])) if kind in ("square", "cross", "decode") else 0
    if splits > nk:
        splits = 0
    return dict(kind=kind, B=B, H=H, nq=nq, nk=nk, d=d, fp16=fp16, causal=causal, kv_len=kv_len, opts=opts, splits=splits)


def _tensors(c, seed, sigma=1.0):
    B, H, nq, nk, d = c["B"], c["H"], c["nq"], c["nk"], c["d"]
    q = inputs.normal(seed, 0, 0, B * H * nq * d, sigma).reshape(B, H, nq, d)
    k = inputs.normal(seed, 1, 0, B * H * nk * d, sigma).reshape(B, H, nk, d)
    v = inputs.normal(seed, 2, 0, B * H * nk * d).reshape(B, H, nk, d)
    if c["fp16"]:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    return q, k, v


# sigma = 3: Q, K ~ N(0, 9), scores with a standard deviation of 9 nats -- the running maximum keeps moving, so the tiles
# renew their lagging reference again and again (sigma = 1 renews it on a row's first keys only)
@pytest.mark.parametrize("block,sigma", [(b, 1.0) for b in range(16)] + [(b, 3.0) for b in range(8)])
def test_random_cases(block, sigma):
    import torch
    from paper_2604_23798_amd import elsa
    rng = np.random.default_rng(9000 + block + OFFSET + (0 if sigma == 1.0 else 50000))
    wide = 1.0 if sigma == 1.0 else 4.0           # FP32 dot products of 9x the magnitude are rounded 9x as coarsely
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    for i in range(20):
        c = _case(rng)
        seed = 9100 + 100 * block + i + OFFSET
        d, scale = c["d"], float(np.float32(c["d"] ** -0.5))
        what = "fuzz %d/%d sigma=%g %s" % (block, i, sigma, {k_: v_ for k_, v_ in c.items() if k_ != "kv_len"})
        tol = wide * tolerance(max(c["nq"], c["nk"]), c["fp16"])
        if c["kind"] == "varlen":
            lengths = [int(x) for x in rng.integers(0, 200, size=int(rng.integers(1, 9)))]
            if sum(lengths) == 0:
                lengths[0] = 5
            q, k, v, cu = inputs.make_varlen(seed, H=c["H"], d=d, fp16=c["fp16"], lengths=lengths)
            ref = oracle.attn_varlen(f32(q), f32(k), f32(v), cu, scale, causal=c["causal"])
            with G.Options(**c["opts"]):
                out = G.fwd_varlen(q, k, v, cu, max(lengths), scale, causal=c["causal"])
            assert_parity(out.reshape(-1, d), ref.reshape(-1, d), tol, what)
            continue
        q, k, v = _tensors(c, seed, sigma)
        ref, ref_lse = oracle.cross_rows(f32(q), f32(k), f32(v), scale, causal=c["causal"], kv_len=c["kv_len"])
        opts = dict(c["opts"], splits=c["splits"])
        try:
            elsa.elsa_set_workspace(ws if c["splits"] else None)
            with G.Options(**opts):
                if c["kind"] == "stream":
                    cuts = sorted(set(int(x) for x in rng.integers(1, c["nk"], size=2))) if c["nk"] > 2 else []
                    edges = [0] + cuts + [c["nk"]]
                    tq = G.to_dev(q)
                    state = torch.empty(elsa.elsa_stream_state_bytes(c["B"], c["H"], c["nq"], d), dtype=torch.uint8, device="cuda")
                    for j in range(len(edges) - 1):
                        a, b = edges[j], edges[j + 1]
                        elsa.elsa_attn_stream_step(tq, G.to_dev(np.ascontiguousarray(k[:, :, a:b])),
                                                   G.to_dev(np.ascontiguousarray(v[:, :, a:b])), state, scale, first=(j == 0),
                                                   causal=c["causal"], causal_shift=(c["nk"] - c["nq"]) - a)
                    o = torch.full_like(tq, float("nan"))
                    elsa.elsa_attn_stream_finish(state, o)
                    torch.cuda.synchronize()
                    out = o.reshape(-1, d).double().cpu().numpy()
                elif c["kind"] == "square" and rng.integers(0, 2):
                    out = G.fwd(q, k, v, scale, causal=c["causal"], kv_len=c["kv_len"], masked_entry=True)
                else:
                    out, lse = G.fwd_cross(q, k, v, scale, causal=c["causal"], kv_len=c["kv_len"], want_lse=True)
                    vis = np.isfinite(ref_lse)
                    assert np.all(np.isneginf(lse[~vis])), what
                    assert np.max(np.abs(lse[vis] - ref_lse[vis]), initial=0.0) < wide * (5e-3 if c["fp16"] else 3e-5), what
        finally:
            elsa.elsa_set_workspace(None)
        assert_parity(out, ref, tol, what)


@pytest.mark.parametrize("block", range(6))
def test_random_cases_with_a_value_width_of_their_own(block):
    """The same sweep for elsa_attn_fwd_dv: pairs, shapes, masks, tiles, work orders, key chunks."""
    import torch
    from paper_2604_23798_amd import elsa
    rng = np.random.default_rng(9500 + block + OFFSET)
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    pairs = [(32, 64), (32, 128), (64, 32), (64, 128), (128, 32), (128, 64), (192, 128)]
    for i in range(20):
        d, dv = pairs[int(rng.integers(0, len(pairs)))]
        fp16 = bool(rng.integers(0, 2))
        B, H = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        nk = int(rng.choice([1, 7, 31, 32, 33, 64, 100, 129, 257, 500, 777, 1300]))
        nq = nk if rng.integers(0, 2) else int(rng.choice([1, 2, 5, 33, 64, 130, 300]))
        causal = bool(rng.integers(0, 2))
        kv_len = rng.integers(0, nk + 1, size=B).astype(np.int32) if rng.integers(0, 2) else None
        variant = int(rng.choice([0, 1, 3]))
        splits = int(rng.choice([0, 0, 2, 3]))
        if splits > nk:
            splits = 0
        opts = dict(variant=variant, snake=int(rng.integers(0, 2)), xcd_map=int(rng.choice([0, 0, 1, 2])), splits=splits)
        if fp16 and rng.integers(0, 4) == 0:
            opts["path"] = 2
        if variant == 3 and d == 192 and (not fp16 or opts.get("path") == 2):
            opts["variant"] = 0                  # the FP32 tiles have no key-splitting shape at d = 192
        seed = 9600 + 100 * block + i + OFFSET
        what = "fuzz dv %d/%d d=%d dv=%d fp16=%d B=%d H=%d nq=%d nk=%d causal=%d len=%s %s" % (
            block, i, d, dv, fp16, B, H, nq, nk, causal, kv_len is not None, opts)
        print(what, flush=True)
        q = inputs.normal(seed, 0, 0, B * H * nq * d).reshape(B, H, nq, d)
        k = inputs.normal(seed, 1, 0, B * H * nk * d).reshape(B, H, nk, d)
        v = inputs.normal(seed, 2, 0, B * H * nk * dv).reshape(B, H, nk, dv)
        if fp16:
            q, k, v = (t.astype(np.float16) for t in (q, k, v))
        scale = float(np.float32(d ** -0.5))
        ref, ref_lse = oracle.dv_rows(f32(q), f32(k), f32(v), scale, causal=causal, kv_len=kv_len)
        try:
            elsa.elsa_set_workspace(ws if splits else None)
            with G.Options(**opts):
                out, lse = G.fwd_dv(q, k, v, scale, causal=causal, kv_len=kv_len, want_lse=True)
        finally:
            elsa.elsa_set_workspace(None)
        vis = np.isfinite(ref_lse)
        assert np.all(np.isneginf(lse[~vis])), what
        assert np.max(np.abs(lse[vis] - ref_lse[vis]), initial=0.0) < (5e-3 if fp16 else 3e-5), what
        assert_parity(out, ref, tolerance(max(nq, nk), fp16), what)


@pytest.mark.parametrize("block", range(4))
def test_random_cases_with_the_library_choosing_tile_and_key_chunks(block):
    """Nothing forced and a workspace lent: tile shape and number of key chunks come from the library's
    own play-through of the launch, at the sizes where that model is active."""
    import torch
    from paper_2604_23798_amd import elsa
    rng = np.random.default_rng(9800 + block + OFFSET)
    ws = torch.empty(128 << 20, dtype=torch.uint8, device="cuda")
    seen = set()
    for i in range(10):
        d = int(rng.choice([32, 64, 64, 128]))
        fp16 = bool(rng.integers(0, 2)) and d <= 64
        B = int(rng.integers(1, 4))
        H = int(rng.choice([1, 3, 8, 12, 16]))
        nk = int(rng.choice([197, 300, 512, 640, 1000, 1536, 2048, 2500]))
        nq = nk if rng.integers(0, 3) else int(rng.choice([64, 130, 300]))
        if nq > nk:
            nq = nk
        causal = bool(rng.integers(0, 2))
        kv_len = rng.integers(nk // 2, nk + 1, size=B).astype(np.int32) if rng.integers(0, 3) == 0 else None
        seed = 9900 + 100 * block + i + OFFSET
        q = inputs.normal(seed, 0, 0, B * H * nq * d).reshape(B, H, nq, d)
        k = inputs.normal(seed, 1, 0, B * H * nk * d).reshape(B, H, nk, d)
        v = inputs.normal(seed, 2, 0, B * H * nk * d).reshape(B, H, nk, d)
        if fp16:
            q, k, v = (t.astype(np.float16) for t in (q, k, v))
        scale = float(np.float32(d ** -0.5))
        # the oracle on a sample of rows (all of them would take a minute at the larger sizes)
        per_head = np.unique(np.concatenate([[0, nq - 1], rng.integers(0, nq, size=48)])).astype(np.int64)
        rows = (np.arange(B * H, dtype=np.int64)[:, None] * nq + per_head[None, :]).reshape(-1)
        ref, ref_lse = oracle.dv_rows(f32(q), f32(k), f32(v), scale, causal=causal, kv_len=kv_len, rows=rows)
        try:
            elsa.elsa_set_workspace(ws)
            out, lse = G.fwd_cross(q, k, v, scale, causal=causal, kv_len=kv_len, want_lse=True)
            plan = (elsa.elsa_last_kernel(), elsa.elsa_last_splits())
        finally:
            elsa.elsa_set_workspace(None)
        seen.add(plan)
        what = "fuzz auto %d/%d d=%d fp16=%d B=%d H=%d nq=%d nk=%d causal=%d len=%s plan=%s" % (
            block, i, d, fp16, B, H, nq, nk, causal, kv_len is not None, plan)
        print(what, flush=True)
        out, lse = out[rows], lse[rows]
        vis = np.isfinite(ref_lse)
        assert np.all(np.isneginf(lse[~vis])), what
        assert np.max(np.abs(lse[vis] - ref_lse[vis]), initial=0.0) < (5e-3 if fp16 else 3e-5), what
        assert_parity(out, ref, tolerance(max(nq, nk), fp16), what)
    assert len(seen) >= 3, seen                 # the sweep does exercise several plans
