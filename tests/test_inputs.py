"""The seeded generator: determinism, slice independence, distributions and workload shapes."""
import numpy as np

from paper_2604_23798_amd import inputs


def test_slices_regenerate_independently():
    full = inputs.normal(1003, 0, 0, 5000)
    assert np.array_equal(inputs.normal(1003, 0, 1234, 777), full[1234:2011])
    assert not np.array_equal(inputs.normal(1003, 1, 0, 100), full[:100])
    assert not np.array_equal(inputs.normal(1004, 0, 0, 100), full[:100])


def test_distributions():
    z = inputs.normal(5, 0, 0, 400000).astype(np.float64)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01 and np.all(np.isfinite(z))
    assert abs(np.mean(z ** 4) - 3.0) < 0.1
    z8 = inputs.normal(5, 0, 0, 100000, 8.0).astype(np.float64)
    assert abs(z8.std() - 8.0) < 0.1
    u = inputs.uniform_pm1(5, 2, 0, 400000).astype(np.float64)
    assert u.min() >= -1 and u.max() <= 1 and abs(u.mean()) < 0.01 and abs(u.var() - 1 / 3) < 0.01
    r = inputs.integers(5, 3, 20000, 256, 512)
    assert r.min() == 256 and r.max() == 512 and abs(r.mean() - 384) < 3


def test_workloads_match_the_stated_shapes():
    w = inputs.WORKLOADS
    assert (w["vit_b16_224"].B, w["vit_b16_224"].H, w["vit_b16_224"].n, w["vit_b16_224"].d) == (1, 12, 197, 64)
    assert w["vit_b16_224"].flops == 119221248
    assert w["bert_base"].flops == 12884901888
    assert w["sweep_n16384"].flops == 4 * 16 * 16384 * 16384 * 64
    assert w["llama13b_32k"].causal and w["llama13b_32k"].d == 128 and w["llama13b_32k"].v_dist == "uniform"
    assert w["hires_vit_64k"].qk_sigma == 8.0 and w["hires_vit_64k"].n == 65536
    q, k, v, kv_len = inputs.make(w["bert_base_padded"].with_(H=1))
    assert q.shape == (16, 1, 512, 64) and q.dtype == np.float32
    assert kv_len.shape == (16,) and kv_len.min() >= 256 and kv_len.max() <= 512
    q, k, v, _ = inputs.make(inputs.sweep(1024, fp16=True).with_(H=1))
    assert q.dtype == np.float16


def test_sample_rows():
    w = inputs.sweep(4096)
    rows = inputs.sample_rows(w, per_head=64)
    assert rows.size == 64 * 16 and len(set(rows.tolist())) == rows.size
    per = rows.reshape(16, 64) - (np.arange(16) * 4096)[:, None]
    assert np.all(per[:, 0] == 0) and np.all(per[:, -1] == 4095)
    assert np.array_equal(rows, inputs.sample_rows(w, per_head=64))
    small = inputs.WORKLOADS["vit_b16_224"].with_(n=5)
    assert inputs.sample_rows(small, per_head=64).size == 12 * 5
