"""Seeded synthetic inputs for the ELSA attention workloads.

This module holds no attention arithmetic: it only draws numbers.  Both the
CPU oracle's tests and the HIP path's tests/benchmark take their tensors from
here, so the two sides see bit-identical inputs.

Generator: counter-based.  Element ``idx`` of tensor ``stream`` under ``seed``
is a pure function of ``(seed, stream, idx)`` (SplitMix64 finaliser applied to
a keyed counter), so any slice can be regenerated independently of the rest and
nothing depends on a library's RNG stream.  Normals come from Box-Muller in
float64 and are rounded once to float32; FP16 experiments round that float32
draw to nearest-even FP16.

The workloads mirror the attention shapes of the paper's experiments (ViT-B/16
at 224 px, BERT-base with padding, the 1K-16K synthetic sweep, a LLaMA-13B
shaped causal long context, a high-resolution ViT).  The datasets and weights
behind those experiments are not used: only the shapes, with N(0,1) / U(-1,1)
stand-in values.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
STREAM_Q, STREAM_K, STREAM_V, STREAM_LEN = 0, 1, 2, 3


def _mix64(x):
    x = (x ^ (x >> np.uint64(30))) * _M1
    x = (x ^ (x >> np.uint64(27))) * _M2
    return x ^ (x >> np.uint64(31))


def _bits(seed, stream, sub, idx):
    """64 random bits for each counter in ``idx`` (uint64 array)."""
    with np.errstate(over="ignore"):
        key = _mix64(np.uint64(seed) * _GOLD + np.uint64(stream * 4 + sub + 1))
        return _mix64(key + (idx + np.uint64(1)) * _GOLD)


def _unit(bits):
    """Map 64 bits to the open interval (0, 1) using the top 53 bits."""
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def uniform01(seed, stream, start, count):
    idx = np.arange(start, start + count, dtype=np.uint64)
    return _unit(_bits(seed, stream, 0, idx))


def _chunked(count, fill):
    """Run ``fill(offset, length)`` over [0, count) in chunks, on a few host threads (every element is a
    pure function of its index, so the chunks are independent and the result does not depend on the split)."""
    step = 1 << 21
    chunks = [(s, min(step, count - s)) for s in range(0, count, step)]
    workers = min(len(chunks), 16, os.cpu_count() or 1)
    if workers <= 1:
        for s, c in chunks:
            fill(s, c)
        return
    with ThreadPoolExecutor(max_workers=workers) as ex:
        list(ex.map(lambda sc: fill(*sc), chunks))


def normal(seed, stream, start, count, sigma=1.0):
    """``count`` draws of N(0, sigma^2), elements [start, start+count), as float32."""
    out = np.empty(count, dtype=np.float32)

    def fill(s, c):
        idx = np.arange(start + s, start + s + c, dtype=np.uint64)
        u1 = _unit(_bits(seed, stream, 0, idx))
        u2 = _unit(_bits(seed, stream, 1, idx))
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * math.pi) * u2)
        out[s:s + c] = (sigma * z).astype(np.float32)
    _chunked(count, fill)
    return out


def uniform_pm1(seed, stream, start, count):
    """``count`` draws of U(-1, 1) as float32."""
    out = np.empty(count, dtype=np.float32)

    def fill(s, c):
        out[s:s + c] = (2.0 * uniform01(seed, stream, start + s, c) - 1.0).astype(np.float32)
    _chunked(count, fill)
    return out


def integers(seed, stream, count, lo, hi):
    """``count`` integers uniform on [lo, hi] as int32."""
    idx = np.arange(count, dtype=np.uint64)
    span = np.uint64(hi - lo + 1)
    return (lo + (_bits(seed, stream, 0, idx) % span).astype(np.int64)).astype(np.int32)


@dataclass(frozen=True)
class Workload:
    """One attention problem: shape, value distributions and seed."""
    name: str
    B: int
    H: int
    n: int
    d: int
    seed: int
    causal: bool = False
    qk_sigma: float = 1.0
    v_dist: str = "normal"          # "normal" = N(0,1), "uniform" = U(-1,1)
    padded: bool = False            # per-batch kv_len uniform on [kv_lo, n]
    kv_lo: int = 0
    fp16: bool = False              # FP16 I/O: inputs rounded to nearest-even FP16
    note: str = field(default="", compare=False)

    @property
    def scale(self) -> float:
        return float(np.float32(1.0 / math.sqrt(self.d)))

    @property
    def flops(self) -> int:
        """4 B H n^2 d  (QK^T and PV, square count)."""
        return 4 * self.B * self.H * self.n * self.n * self.d

    def with_(self, **kw) -> "Workload":
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


def sweep(n: int, fp16: bool = False) -> Workload:
    """Long-sequence sweep point: B=1, H=16, d=64, n in {1024, ..., 16384}."""
    lg = int(round(math.log2(n)))
    return Workload(name="sweep_n%d%s" % (n, "_fp16" if fp16 else ""), B=1, H=16, n=n, d=64,
                    seed=1003 + lg, fp16=fp16, note="synthetic 1K-16K sweep shape")


WORKLOADS = {
    "vit_b16_224": Workload("vit_b16_224", B=1, H=12, n=197, d=64, seed=1001,
                            note="ViT-B/16 at 224 px: 196 patches + class token"),
    "bert_base": Workload("bert_base", B=16, H=12, n=512, d=64, seed=1002,
                          note="BERT-base attention shape"),
    "bert_base_padded": Workload("bert_base_padded", B=16, H=12, n=512, d=64, seed=1002, padded=True,
                                 kv_lo=256, note="BERT-base with per-batch key padding"),
    "llama13b_32k": Workload("llama13b_32k", B=1, H=40, n=32768, d=128, seed=1004, causal=True,
                             v_dist="uniform", note="LLaMA-13B shaped causal long context"),
    "llama13b_32k_fp16": Workload("llama13b_32k_fp16", B=1, H=40, n=32768, d=128, seed=1004, causal=True,
                                  v_dist="uniform", fp16=True, note="same, FP16 I/O"),
    "swin_w7": Workload("swin_w7", B=512, H=3, n=49, d=32, seed=1007,
                        note="window attention: Swin-T stage 1 at 224 px, 7x7 windows, 64 windows x batch 8"),
    "swin_w14": Workload("swin_w14", B=128, H=3, n=196, d=32, seed=1008,
                         note="window attention with 14x14 windows (196 tokens, the largest window size the paper uses)"),
    "swin_w8": Workload("swin_w8", B=392, H=3, n=64, d=32, seed=1009,
                        note="window attention, 8x8 windows (W8): 49 windows x batch 8"),
    "swin_w16": Workload("swin_w16", B=128, H=3, n=256, d=32, seed=1010,
                         note="window attention, 16x16 windows (W16): 16 windows x batch 8"),
    "frames_416k": Workload("frames_416k", B=1, H=1, n=416400, d=64, seed=1011,
                            note="one head at the longest token count the paper mentions (multi-frame input, 416,400 tokens)"),
    "hires_vit_64k": Workload("hires_vit_64k", B=1, H=16, n=65536, d=64, seed=1005, qk_sigma=8.0,
                              note="1024x1024 image, 4x4 patches; wide score range"),
}
for _n in (1024, 2048, 4096, 8192, 16384):
    WORKLOADS[sweep(_n).name] = sweep(_n)
    WORKLOADS[sweep(_n, True).name] = sweep(_n, True)


def make(w: Workload):
    """Draw the tensors of a workload.

    Returns ``(q, k, v, kv_len)``: float32 arrays ``[B,H,n,d]`` (float16 when
    ``w.fp16``) and an int32 ``[B]`` array of valid key counts or ``None``."""
    count = w.B * w.H * w.n * w.d
    shape = (w.B, w.H, w.n, w.d)
    q = normal(w.seed, STREAM_Q, 0, count, w.qk_sigma).reshape(shape)
    k = normal(w.seed, STREAM_K, 0, count, w.qk_sigma).reshape(shape)
    if w.v_dist == "uniform":
        v = uniform_pm1(w.seed, STREAM_V, 0, count).reshape(shape)
    else:
        v = normal(w.seed, STREAM_V, 0, count, 1.0).reshape(shape)
    if w.fp16:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    kv_len = integers(w.seed, STREAM_LEN, w.B, w.kv_lo, w.n) if w.padded else None
    return q, k, v, kv_len


def make_varlen(seed: int, num_seqs: int = 8, lo: int = 256, hi: int = 1792, H: int = 12, d: int = 64,
                fp16: bool = False, lengths=None):
    """Packed variable-length batch: ``num_seqs`` sequences with lengths uniform on [lo, hi] (the
    paper's padding-free workload draws 8 lengths from [256, 1792]) or the given ``lengths``.

    Returns ``(q, k, v, cu_seqlens)``: ``[total_tokens, H, d]`` arrays and int32 ``[num_seqs + 1]``."""
    lens = integers(seed, STREAM_LEN, num_seqs, lo, hi) if lengths is None else np.asarray(lengths, np.int32)
    cu = np.zeros(lens.size + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    total = int(cu[-1])
    shape = (total, H, d)
    q = normal(seed, STREAM_Q, 0, total * H * d).reshape(shape)
    k = normal(seed, STREAM_K, 0, total * H * d).reshape(shape)
    v = normal(seed, STREAM_V, 0, total * H * d).reshape(shape)
    if fp16:
        q, k, v = (t.astype(np.float16) for t in (q, k, v))
    return q, k, v, cu


def sample_rows(w: Workload, per_head: int = 64, tile: int = 128, seed: int = 7) -> np.ndarray:
    """Seeded sample of flat query rows, ``per_head`` rows per (b,h) (all rows when n is smaller), taken in
    this order of priority: the first and the last row; the rows around one multiple of each kernel
    granularity (32-row wave groups, 64-, 128- and 256-row tiles: c*u - 1, c*u, c*u + 1 for a seeded c);
    for causal workloads the first and last row of the first, a middle and the last ``tile``-row query tile;
    the rows around a second multiple of each granularity; seeded random rows."""
    n = w.n
    rows = []
    for bh in range(w.B * w.H):
        budget = min(per_head, n)
        picks = []

        def take(i):
            if 0 <= i < n and i not in picks and len(picks) < budget:
                picks.append(int(i))
        take(0)
        take(n - 1)
        units = (32, 64, 128, 256)
        cuts = integers(seed + 1, bh, 2 * len(units), 0, (1 << 30) - 1)
        for rnd in range(2):
            for ui, u in enumerate(units):
                nb = n // u
                if nb < 2 or (rnd == 1 and nb < 3):
                    continue
                c = 1 + int(cuts[rnd * len(units) + ui]) % (nb - 1)
                for dlt in (0, -1, 1):
                    take(c * u + dlt)
            if rnd == 0 and w.causal and n > tile:
                nt = (n + tile - 1) // tile
                for t in (0, nt // 2, nt - 1):
                    take(t * tile)
                    take(min(n, (t + 1) * tile) - 1)
        extra = integers(seed, bh, max(0, 4 * per_head), 0, n - 1)
        for i in extra:
            if len(picks) >= budget:
                break
            take(int(i))
        i = 0
        while len(picks) < budget:       # tiny n: fill with the remaining rows
            take(i)
            i += 1
        rows.extend(bh * n + i for i in sorted(picks))
    return np.asarray(rows, dtype=np.int64)
