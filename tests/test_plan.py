"""Host logic without a GPU: with ELSA_OPT_DRY_RUN every entry point validates, chooses kernel, tile
and key chunks as usual and launches nothing, so the choices documented for the workloads can be
checked on the CPU.  Pointers are dummies that are never dereferenced."""
import ctypes

import pytest

from paper_2604_23798_amd import elsa

P = ctypes.c_void_p(1 << 20)          # 256-byte aligned, never dereferenced


@pytest.fixture(autouse=True)
def _dry_run():
    elsa.elsa_set_option(elsa.OPT_DRY_RUN, 1)
    yield
    for o in range(6):
        elsa.elsa_set_option(o, 0)
    elsa.raw().elsa_set_workspace(None, 0)


def plan(B, H, nq, nk, d, causal=False, dtype=0, kv_len=False, ws_mib=0, dv=None, scale=0.125, **opts):
    lib = elsa.raw()
    assert lib.elsa_set_workspace(P if ws_mib else None, ws_mib << 20) == 0
    for name, val in opts.items():
        elsa.elsa_set_option(getattr(elsa, "OPT_" + name.upper()), val)
    if dv is None:
        rc = lib.elsa_attn_fwd_cross(P, P, P, P, None, B, H, nq, nk, d, scale, int(causal), P if kv_len else None, dtype, None)
    else:
        rc = lib.elsa_attn_fwd_dv(P, P, P, P, None, B, H, nq, nk, d, dv, scale, int(causal), P if kv_len else None, dtype, None)
    for name in opts:
        elsa.elsa_set_option(getattr(elsa, "OPT_" + name.upper()), 0)
    assert rc == 0, elsa.status_string(rc)
    return elsa.elsa_last_kernel(), elsa.elsa_last_splits()


def test_headline_and_long_sequences_take_the_128_row_tiles_in_one_pass():
    assert plan(1, 16, 16384, 16384, 64, ws_mib=256) == ("mfma_q128_k32", 1)
    assert plan(1, 16, 65536, 65536, 64, ws_mib=256) == ("mfma_q128_k32", 1)
    assert plan(1, 40, 32768, 32768, 128, causal=True, ws_mib=256) == ("mfma_q128_w4", 1)
    assert plan(16, 12, 512, 512, 64, ws_mib=256) == ("mfma_q128_k32", 1)
    assert plan(1, 16, 16384, 16384, 64, dtype=1) == ("mfma16_q256_w4", 1)
    assert plan(1, 16, 16384, 16384, 64, dtype=1, causal=True) == ("mfma16_q256_w4", 1)   # long and many blocks: 961 against 927 TFLOP/s
    assert plan(1, 16, 8192, 8192, 64, dtype=1, causal=True) == ("mfma16_q128_w4", 1)     # else its diagonal tiles waste less
    assert plan(1, 8, 16384, 16384, 64, dtype=1, causal=True) == ("mfma16_q128_w4", 1)
    assert plan(1, 40, 4096, 4096, 64, dtype=1) == ("mfma16_q128_w4", 1)                  # 640 256-row blocks: 1.25 rounds
    # FP16 at d >= 96: the 256-row tile of eight query waves where its blocks fill the CUs evenly, else the 128-row tile
    assert plan(1, 40, 32768, 32768, 128, causal=True, dtype=1) == ("mfma16_q256_w8", 1)
    assert plan(1, 16, 8192, 8192, 128, dtype=1) == ("mfma16_q256_w8", 1)
    assert plan(1, 40, 4096, 4096, 128, dtype=1) == ("mfma16_q128_w4", 1)                    # 640 blocks: 2.5 rounds
    assert plan(1, 16, 8192, 8192, 128, dtype=1, causal=True) == ("mfma16_q128_w4", 1)
    assert plan(1, 40, 1024, 1024, 256, dtype=1) == ("mfma16_q256_w8", 1)
    assert plan(1, 40, 1024, 1024, 128, dtype=1) == ("mfma16_q256_w8", 1)                    # 160 blocks: 35.6 against 41-46 us
    assert plan(1, 16, 2048, 2048, 128, dtype=1) != ("mfma16_q256_w8", 1)                    # 128 blocks: too few
    assert plan(1, 16, 8192, 8192, 96) == ("mfma_q128_w4", 1) and plan(1, 16, 8192, 8192, 256) == ("mfma_q128_w4", 1)


def test_small_problems_follow_the_block_placement_model():
    # one image of ViT-B/16: 84 blocks of 32 rows whose waves split the keys
    assert plan(1, 12, 197, 197, 64) == ("mfma_xwave", 1)
    assert plan(1, 12, 197, 197, 64, ws_mib=64) == ("mfma_xwave", 1)         # never cut further
    assert plan(4, 12, 197, 197, 64) == ("mfma_q64_xw2", 1)
    assert plan(1, 16, 1024, 1024, 64, ws_mib=64) == ("mfma_q64_xw2", 1)
    assert plan(1, 16, 1024, 1024, 64, causal=True, ws_mib=64) == ("mfma_q64_xw2", 2)
    assert plan(1, 16, 1024, 1024, 64, causal=True) == ("mfma_xwave", 1)     # no workspace, no key chunks: 32-row tiles
    # 192 blocks of 128 rows would fill the CUs 0.75 times and 384 one and a half times: never one pass of that tile
    assert plan(1, 16, 1536, 1536, 64, ws_mib=64) in (("mfma_q64_xw2", 2), ("mfma_q128_k32", 4))
    assert plan(1, 16, 3072, 3072, 64, ws_mib=64) in (("mfma_q64_xw2", 1), ("mfma_q128_k32", 2))
    assert plan(1, 16, 3072, 3072, 64) == ("mfma_q64_xw2", 1)               # 768 blocks: exactly three rounds
    assert plan(1, 40, 1024, 1024, 128, ws_mib=256) == ("mfma_q128_w4", 4)   # 320 blocks -> 1280
    # d = 128, causal, a few runs of blocks: the single-buffered 64-row tile (two blocks per CU), never cut
    assert plan(1, 40, 1024, 1024, 128, causal=True, ws_mib=256) == ("mfma_q64_xw2_sb", 1)
    assert plan(1, 16, 3072, 3072, 128, causal=True, ws_mib=256) == ("mfma_q64_xw2_sb", 1)
    assert plan(1, 16, 3072, 3072, 64, causal=True, ws_mib=256)[0] != "mfma_q64_xw2_sb"       # d = 128 only
    # FP16 tiles: the shape is chosen the same way, the keys are never cut
    assert plan(1, 16, 2048, 2048, 64, dtype=1, ws_mib=64) == ("mfma16_q64_xw2", 1)
    assert plan(1, 16, 2048, 2048, 64, dtype=1, causal=True) in (("mfma16_q64_xw2", 1), ("mfma16_xwave", 1))   # 25.3 / 25.8 us
    assert plan(1, 16, 4096, 4096, 64, dtype=1, causal=True) == ("mfma16_q64_xw2", 1)
    assert plan(1, 16, 4096, 4096, 64, dtype=1) == ("mfma16_q128_w4", 1)
    # FP16 tiles at d = 128: causal launches of one or two runs of 128-row blocks take the 64-row tile (measured 25-36 % faster)
    assert plan(1, 16, 2048, 2048, 128, dtype=1, causal=True) == ("mfma16_q64_xw2", 1)
    assert plan(1, 8, 4096, 4096, 128, dtype=1, causal=True) == ("mfma16_q64_xw2", 1)
    assert plan(1, 40, 4096, 4096, 128, dtype=1, causal=True) == ("mfma16_q128_w4", 1)
    assert plan(1, 40, 4096, 4096, 128, dtype=1) == ("mfma16_q128_w4", 1)
    # d = 96 and d = 256 are played through as well (own step times; at d = 256 the FP32 tile owns its CU and may be cut under a causal mask)
    assert plan(1, 8, 2048, 2048, 96, causal=True, ws_mib=256) == ("mfma_q128_w4", 4)            # 84 against 118 us with two chunks
    assert plan(1, 16, 4096, 4096, 256, causal=True, ws_mib=256) == ("mfma_q128_w4", 2)          # 1.37 against 1.63 ms in one pass
    assert plan(1, 16, 2048, 2048, 96, dtype=1, causal=True) == ("mfma16_q64_xw2", 1)           # 33 against 48 us
    assert plan(1, 16, 2048, 2048, 256, dtype=1, causal=True) == ("mfma16_q64_xw2", 1)          # 114 against 167 us
    assert plan(1, 16, 16384, 16384, 256, dtype=1) == ("mfma16_q256_w8", 1)                       # 2.07 against 2.70 ms (H = 8)
    # a forced tile or chunk count switches the model off
    assert plan(1, 16, 1024, 1024, 64, ws_mib=64, variant=7) == ("mfma_q128_k32", 2)
    assert plan(1, 16, 1024, 1024, 64, ws_mib=64, splits=3)[1] == 3
    # FP16 tiles are not cut outside decoding
    assert plan(1, 16, 1024, 1024, 64, dtype=1, ws_mib=64) in (("mfma16_xwave", 1), ("mfma16_q64_xw2", 1))   # 14.8 / 15.3 us


def test_key_chunks_stay_few_and_causal_launches_of_two_runs_are_not_cut():
    # a causal launch whose 128-row blocks fill the CUs twice brings blocks of every length: one pass
    for H, n in ((8, 16384), (8, 12288), (16, 8192), (24, 6144)):
        assert plan(1, H, n, n, 64, causal=True, ws_mib=256)[1] == 1
        assert plan(1, H, n, n, 128, causal=True, ws_mib=256)[1] == 1
    # outside decoding the model never asks for more than four chunks
    for H in (1, 3, 8, 12, 16, 24):
        for n in (512, 1000, 1536, 2500, 3072, 6144):
            for d in (32, 64, 128):
                for causal in (False, True):
                    assert 1 <= plan(1, H, n, n, d, causal=causal, ws_mib=256)[1] <= 4
    # mid-sized launches that fill the last run badly are repaired (a smaller tile or two chunks)
    assert plan(1, 12, 12288, 12288, 64, ws_mib=256) != ("mfma_q128_k32", 1)


def test_value_width_entry_point_uses_the_same_model():
    # (measured before -> after, us)  FP16 d = 64, d_v = 128, H = 8, n = 4096 causal: 98.7 -> 57.9; FP32 d = 64, d_v = 128, H = 40, n = 2048: 600 -> 534
    assert plan(1, 8, 4096, 4096, 64, dv=128, dtype=1, causal=True) == ("mfma16_dv_xwave", 1)
    assert plan(1, 40, 2048, 2048, 64, dv=128, ws_mib=256) == ("mfma_dv_q128", 2)
    assert plan(1, 16, 16384, 16384, 64, dv=128, ws_mib=256) == ("mfma_dv_q128", 1)
    assert plan(1, 16, 8192, 8192, 192, dv=128, dtype=1, causal=True) == ("mfma16_dv_q128", 1)
    assert plan(1, 40, 2048, 2048, 192, dv=128, dtype=1) == ("mfma16_dv_q128", 1)
    assert plan(1, 16, 2048, 2048, 64, dv=128, ws_mib=256, variant=1, splits=1) == ("mfma_dv_q128", 1)   # forced: no model


def plan_varlen(num_seqs, total, max_len, H, d, causal=False, dtype=0):
    rc = elsa.raw().elsa_attn_fwd_varlen(P, P, P, P, P, num_seqs, total, max_len, H, d, 0.125, int(causal), dtype, None)
    assert rc == 0, elsa.status_string(rc)
    return elsa.elsa_last_kernel(), elsa.elsa_last_splits()


def test_packed_batches_take_the_64_row_tile_only_when_causal_and_long_enough():
    # the paper's padding-free workload: 8 sequences, lengths U[256,1792] (about 8 x 1024 tokens), H = 12, d = 64
    assert plan_varlen(8, 8192, 1792, 12, 64) == ("mfma_q128_k32", 1)
    assert plan_varlen(8, 8192, 1792, 12, 64, causal=True) == ("mfma_q64_xw2", 1)
    assert plan_varlen(8, 8192, 1792, 12, 64, causal=True, dtype=1) == ("mfma16_q64_xw2", 1)
    assert plan_varlen(32, 9000, 512, 12, 64, causal=True) == ("mfma_q128_k32", 1)          # short sequences
    assert plan_varlen(8, 8192, 1792, 32, 128, causal=True) == ("mfma_q128_w4", 1)          # d = 128
    assert plan_varlen(8, 65536, 16384, 16, 64, causal=True) == ("mfma_q128_k32", 1)        # many runs of blocks


def test_window_attention_takes_the_lds_free_tile():
    assert plan(512, 3, 49, 49, 32) == ("mfma_small_q32", 1)
    assert plan(392, 3, 64, 64, 32) == ("mfma_small_q32", 1)
    assert plan(128, 3, 196, 196, 32) == ("mfma_q128_k32", 1)
    assert plan(128, 3, 256, 256, 32) == ("mfma_q128_k32", 1)


def test_decoding_streams_the_cache_with_the_vector_kernel():
    assert plan(2, 40, 1, 32768, 128, causal=True) == ("fma_decode_q1", 1)
    assert plan(2, 40, 1, 32768, 128, causal=True, ws_mib=256) == ("fma_decode_q1", 16)   # five blocks per CU
    assert plan(2, 40, 4, 32768, 128, causal=True, dtype=1, ws_mib=256) == ("fma_decode_q4", 16)
    assert plan(2, 40, 8, 32768, 128, ws_mib=256)[0] == "fma_decode_q8"                  # FP32, d = 128: up to eight
    assert plan(2, 40, 8, 32768, 128, dtype=1, ws_mib=256)[0] == "mfma16_xwave"
    assert plan(2, 40, 16, 32768, 64, ws_mib=256)[0] == "mfma_xwave"
    assert plan(2, 40, 16, 32768, 128, ws_mib=256)[0] == "mfma_xwave32" and plan(2, 40, 40, 32768, 128, ws_mib=256)[0] == "mfma_xwave"
    assert plan(2, 40, 1, 32768, 256)[0] == "fma_decode_q1" and plan(2, 40, 3, 32768, 96)[0] == "fma_decode_q1"
    name, C = plan(1, 1, 1, 1 << 20, 64, ws_mib=256)
    assert name == "fma_decode_q1" and C == 64                                            # at most 64 chunks
    assert plan(1, 8, 1, 300, 64, ws_mib=256) == ("fma_decode_q1", 1)                     # chunks of >= 256 keys only


def test_value_width_of_its_own():
    assert plan(1, 16, 8192, 8192, 192, dv=128) == ("mfma_dv_q128", 1)
    assert plan(1, 16, 8192, 8192, 192, dv=128, dtype=1) == ("mfma16_dv_q128", 1)
    assert plan(1, 16, 8192, 8192, 64, dv=128, dtype=1, scale=0.0) == ("mfma_dv_q128", 1)     # FP16 tiles need a scale
    assert plan(2, 3, 1, 5000, 64, dv=128) == ("mfma_dv_xwave", 1)
    assert plan(2, 3, 1, 5000, 192, dv=128) == ("mfma_dv_q128", 1)       # no FP32 key-splitting tile at d = 192
    assert plan(2, 3, 1, 5000, 192, dv=128, dtype=1) == ("mfma16_dv_xwave", 1)
    name, C = plan(2, 3, 1, 5000, 64, dv=128, ws_mib=64)
    assert name == "mfma_dv_xwave" and C == 19                           # 5000 // 256 chunks
    assert plan(1, 4, 130, 500, 64, dv=64, causal=True) == plan(1, 4, 130, 500, 64, causal=True)   # forwarded


def test_a_dry_run_still_validates():
    lib = elsa.raw()
    assert lib.elsa_attn_fwd_cross(None, P, P, P, None, 1, 1, 8, 8, 64, 0.125, 0, None, 0, None) == elsa.ERR_INVALID_ARG
    assert lib.elsa_attn_fwd_cross(P, P, P, P, None, 1, 1, 8, 8, 80, 0.125, 0, None, 0, None) == elsa.ERR_UNSUPPORTED
    assert lib.elsa_attn_fwd_dv(P, P, P, P, None, 1, 1, 8, 8, 64, 96, 0.125, 0, None, 0, None) == elsa.ERR_UNSUPPORTED
    with pytest.raises(elsa.ElsaError):
        elsa.elsa_set_option(elsa.OPT_DRY_RUN, 2)
