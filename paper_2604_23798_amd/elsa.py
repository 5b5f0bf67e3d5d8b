"""ctypes binding of libelsa.so: argument marshalling only.

Every step of the attention path runs in the HIP kernels behind the C ABI
declared in ``include/elsa.h``; PyTorch is used for device memory and streams.
Importing this module fails loudly when the library has not been built --
there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libelsa.so")

F32, F16 = 0, 1
OPT_PATH, OPT_VARIANT, OPT_SPLITS, OPT_XCD_MAP, OPT_SNAKE, OPT_DRY_RUN = 0, 1, 2, 3, 4, 5
PATH_AUTO, PATH_FMA, PATH_MFMA, PATH_MFMA16 = 0, 1, 2, 3
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, 1, 2, 3, 4

EXPORTS = ("elsa_attn_fwd", "elsa_attn_fwd_masked", "elsa_attn_fwd_static", "elsa_static_scratch_bytes", "elsa_attn_fwd_lse", "elsa_attn_fwd_cross", "elsa_attn_fwd_dv", "elsa_attn_fwd_varlen", "elsa_attn_fwd_split_kv", "elsa_combine",
           "elsa_stream_state_bytes", "elsa_attn_stream_step", "elsa_attn_stream_finish",
           "elsa_split_kv_workspace_bytes", "elsa_set_workspace", "elsa_set_option", "elsa_get_option",
           "elsa_variant_name", "elsa_last_kernel", "elsa_last_splits", "elsa_status_string", "elsa_debug_layout_probe", "elsa_debug_issue_probe")

if not os.path.exists(LIB_PATH):
    raise ImportError("libelsa.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or python paper_2604_23798_amd/build.py) first; there is no fallback path")

_lib = ctypes.CDLL(LIB_PATH)
_vp, _i, _f = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
_lib.elsa_attn_fwd.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _f, _i, _i, _vp]
_lib.elsa_attn_fwd_masked.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _f, _i, _vp, _i, _vp]
_lib.elsa_attn_fwd_static.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _f, _i, _vp, _i, _i, _vp]
_lib.elsa_static_scratch_bytes.restype = ctypes.c_size_t
_lib.elsa_attn_fwd_lse.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _f, _i, _vp, _i, _vp]
_lib.elsa_attn_fwd_cross.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _f, _i, _vp, _i, _vp]
_lib.elsa_attn_fwd_dv.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _f, _i, _vp, _i, _vp]
_lib.elsa_stream_state_bytes.argtypes = [_i, _i, _i, _i]
_lib.elsa_stream_state_bytes.restype = ctypes.c_size_t
_lib.elsa_attn_stream_step.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _f, _i, _i, _vp, _i, _i, _vp]
_lib.elsa_attn_stream_finish.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _i, _vp]
_lib.elsa_attn_fwd_varlen.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _f, _i, _i, _vp]
_lib.elsa_attn_fwd_split_kv.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _f, _i, _vp, _i, _i, _vp]
_lib.elsa_combine.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp]
_lib.elsa_split_kv_workspace_bytes.argtypes = [_i, _i, _i, _i, _i]
_lib.elsa_split_kv_workspace_bytes.restype = ctypes.c_size_t
_lib.elsa_set_workspace.argtypes = [_vp, ctypes.c_size_t]
_lib.elsa_set_option.argtypes = [_i, _i]
_lib.elsa_get_option.argtypes = [_i, ctypes.POINTER(_i)]
_lib.elsa_variant_name.argtypes = [_i, _i]
_lib.elsa_variant_name.restype = ctypes.c_char_p
_lib.elsa_last_kernel.restype = ctypes.c_char_p
_lib.elsa_status_string.argtypes = [_i]
_lib.elsa_status_string.restype = ctypes.c_char_p
_lib.elsa_debug_layout_probe.argtypes = [_vp, _vp]
_lib.elsa_debug_issue_probe.argtypes = [_vp, _i, _i, _i, _i, _vp]


class ElsaError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__("libelsa: %s (code %d)" % (status_string(code), code))


def status_string(code: int) -> str:
    return _lib.elsa_status_string(int(code)).decode()


def _check(rc):
    if rc != 0:
        raise ElsaError(rc)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


_raw_stream = None      # torch's fast accessor of the current raw stream, looked up once


def _stream(stream, like=None):
    """hipStream_t of ``stream`` (a torch stream), or of torch's current stream on the device of ``like``."""
    global _raw_stream
    if stream is not None:
        return ctypes.c_void_p(stream.cuda_stream)
    import torch
    if _raw_stream is None:
        _raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", False)
    if _raw_stream and like is not None:
        return ctypes.c_void_p(_raw_stream(like.device.index))
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.float16:
        return F16
    raise TypeError("q/k/v must be float32 or float16")


def _shape(q, k, v):
    assert q.is_cuda and k.is_cuda and v.is_cuda, "device tensors required"
    assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    assert q.dim() == 4 and q.shape == k.shape == v.shape and q.dtype == k.dtype == v.dtype
    return tuple(int(x) for x in q.shape)


def elsa_attn_fwd(q, k, v, out, scale, causal=False, stream=None):
    B, H, n, d = _shape(q, k, v)
    assert out.is_contiguous() and out.shape == q.shape and out.dtype == q.dtype
    _check(_lib.elsa_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, H, n, d, float(scale), int(bool(causal)),
                              _dtype_code(q), _stream(stream, q)))
    return out


def elsa_attn_fwd_masked(q, k, v, out, scale, causal=False, kv_len=None, stream=None):
    import torch
    B, H, n, d = _shape(q, k, v)
    assert out.is_contiguous() and out.shape == q.shape and out.dtype == q.dtype
    if kv_len is not None:
        assert kv_len.is_cuda and kv_len.dtype == torch.int32 and kv_len.shape == (B,) and kv_len.is_contiguous()
    _check(_lib.elsa_attn_fwd_masked(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, H, n, d, float(scale),
                                     int(bool(causal)), _ptr(kv_len), _dtype_code(q), _stream(stream, q)))
    return out


def elsa_attn_fwd_static(q, k, v, out, scale, causal=False, kv_len=None, num_splits=0, stream=None):
    """elsa_attn_fwd_masked whose key split keeps its chunk states in the library's own device array."""
    import torch
    B, H, n, d = _shape(q, k, v)
    assert out.is_contiguous() and out.shape == q.shape and out.dtype == q.dtype
    if kv_len is not None:
        assert kv_len.is_cuda and kv_len.dtype == torch.int32 and kv_len.shape == (B,) and kv_len.is_contiguous()
    _check(_lib.elsa_attn_fwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, H, n, d, float(scale), int(bool(causal)),
                                     _ptr(kv_len), int(num_splits), _dtype_code(q), _stream(stream, q)))
    return out


def elsa_static_scratch_bytes() -> int:
    return int(_lib.elsa_static_scratch_bytes())


def elsa_attn_fwd_lse(q, k, v, out, lse, scale, causal=False, kv_len=None, stream=None):
    import torch
    B, H, n, d = _shape(q, k, v)
    assert out.is_contiguous() and out.shape == q.shape and out.dtype == q.dtype
    assert lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, H, n)
    _check(_lib.elsa_attn_fwd_lse(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, n, d, float(scale),
                                  int(bool(causal)), _ptr(kv_len), _dtype_code(q), _stream(stream, q)))
    return out, lse


def elsa_attn_fwd_cross(q, k, v, out, scale, causal=False, kv_len=None, lse=None, stream=None):
    """q, out: [B, H, n_q, d]; k, v: [B, H, n_k, d]; lse (optional): float32 [B, H, n_q]."""
    import torch
    assert q.is_cuda and q.dim() == 4 and k.dim() == 4 and k.shape == v.shape
    assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous() and out.is_contiguous()
    assert q.dtype == k.dtype == v.dtype == out.dtype and out.shape == q.shape
    B, H, nq, d = q.shape
    nk = k.shape[2]
    assert tuple(k.shape) == (B, H, nk, d)
    if kv_len is not None:
        assert kv_len.is_cuda and kv_len.dtype == torch.int32 and tuple(kv_len.shape) == (B,)
    if lse is not None:
        assert lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, H, nq)
    _check(_lib.elsa_attn_fwd_cross(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, nq, nk, d, float(scale),
                                    int(bool(causal)), _ptr(kv_len), _dtype_code(q), _stream(stream, q)))
    return out


def elsa_attn_fwd_dv(q, k, v, out, scale, causal=False, kv_len=None, lse=None, stream=None):
    """q: [B, H, n_q, d]; k: [B, H, n_k, d]; v: [B, H, n_k, d_v]; out: [B, H, n_q, d_v]; lse (optional): float32 [B, H, n_q]."""
    import torch
    assert q.is_cuda and q.dim() == 4 and k.dim() == 4 and v.dim() == 4 and out.dim() == 4
    assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous() and out.is_contiguous()
    assert q.dtype == k.dtype == v.dtype == out.dtype
    B, H, nq, d = q.shape
    nk, dv = v.shape[2], v.shape[3]
    assert tuple(k.shape) == (B, H, nk, d) and tuple(v.shape) == (B, H, nk, dv) and tuple(out.shape) == (B, H, nq, dv)
    if kv_len is not None:
        assert kv_len.is_cuda and kv_len.dtype == torch.int32 and tuple(kv_len.shape) == (B,)
    if lse is not None:
        assert lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, H, nq)
    _check(_lib.elsa_attn_fwd_dv(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, nq, nk, d, dv, float(scale),
                                 int(bool(causal)), _ptr(kv_len), _dtype_code(q), _stream(stream, q)))
    return out


def elsa_stream_state_bytes(B, H, n_q, d) -> int:
    return int(_lib.elsa_stream_state_bytes(B, H, n_q, d))


def elsa_attn_stream_step(q, k_chunk, v_chunk, state, scale, first, causal=False, causal_shift=0, kv_len=None,
                          stream=None):
    """One chunk of keys/values merged into the running state (uint8 device buffer of elsa_stream_state_bytes)."""
    import torch
    assert q.is_cuda and q.dim() == 4 and k_chunk.dim() == 4 and k_chunk.shape == v_chunk.shape
    assert q.is_contiguous() and k_chunk.is_contiguous() and v_chunk.is_contiguous() and state.is_contiguous()
    assert q.dtype == k_chunk.dtype == v_chunk.dtype
    B, H, nq, d = q.shape
    nc = k_chunk.shape[2]
    assert tuple(k_chunk.shape) == (B, H, nc, d)
    assert state.is_cuda and state.numel() * state.element_size() >= elsa_stream_state_bytes(B, H, nq, d)
    if kv_len is not None:
        assert kv_len.is_cuda and kv_len.dtype == torch.int32 and tuple(kv_len.shape) == (B,)
    _check(_lib.elsa_attn_stream_step(_ptr(q), _ptr(k_chunk), _ptr(v_chunk), _ptr(state), B, H, nq, nc, d, float(scale),
                                      int(bool(causal)), int(causal_shift), _ptr(kv_len), int(bool(first)),
                                      _dtype_code(q), _stream(stream, q)))


def elsa_attn_stream_finish(state, out, lse=None, stream=None):
    import torch
    B, H, nq, d = out.shape
    assert out.is_cuda and out.is_contiguous() and state.is_cuda
    if lse is not None:
        assert lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, H, nq)
    _check(_lib.elsa_attn_stream_finish(_ptr(state), _ptr(out), _ptr(lse), B, H, nq, d, _dtype_code(out),
                                        _stream(stream, out)))
    return out


def elsa_attn_fwd_varlen(q, k, v, out, cu_seqlens, max_seqlen, scale, causal=False, stream=None):
    """Packed sequences: q, k, v, out are [total_tokens, H, d]; cu_seqlens is device int32 [num_seqs + 1]."""
    import torch
    assert q.is_cuda and q.dim() == 3 and q.shape == k.shape == v.shape == out.shape
    assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous() and out.is_contiguous()
    assert q.dtype == k.dtype == v.dtype == out.dtype
    assert cu_seqlens.is_cuda and cu_seqlens.dtype == torch.int32 and cu_seqlens.dim() == 1
    T, H, d = (int(x) for x in q.shape)
    _check(_lib.elsa_attn_fwd_varlen(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(cu_seqlens),
                                     int(cu_seqlens.numel()) - 1, T, int(max_seqlen), H, d, float(scale),
                                     int(bool(causal)), _dtype_code(q), _stream(stream, q)))
    return out


def elsa_attn_fwd_split_kv(q, k, v, part_m, part_S, part_W, scale, num_splits, causal=False, kv_len=None,
                           stream=None):
    import torch
    B, H, n, d = _shape(q, k, v)
    C = int(num_splits)
    for t, shp in ((part_m, (B, H, C, n)), (part_S, (B, H, C, n)), (part_W, (B, H, C, n, d))):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.float32 and tuple(t.shape) == shp
    _check(_lib.elsa_attn_fwd_split_kv(_ptr(q), _ptr(k), _ptr(v), _ptr(part_m), _ptr(part_S), _ptr(part_W),
                                       B, H, n, d, float(scale), int(bool(causal)), _ptr(kv_len), C,
                                       _dtype_code(q), _stream(stream, q)))
    return part_m, part_S, part_W


def elsa_combine(part_m, part_S, part_W, out, stream=None):
    import torch
    B, H, C, n, d = (int(x) for x in part_W.shape)
    assert tuple(part_m.shape) == (B, H, C, n) == tuple(part_S.shape)
    for t in (part_m, part_S, part_W):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.float32
    assert out.is_cuda and out.is_contiguous() and tuple(out.shape) == (B, H, n, d)
    _check(_lib.elsa_combine(_ptr(part_m), _ptr(part_S), _ptr(part_W), _ptr(out), B, H, n, d, C,
                             _dtype_code(out), _stream(stream, out)))
    return out


def elsa_split_kv_workspace_bytes(B, H, n, d, num_splits) -> int:
    return int(_lib.elsa_split_kv_workspace_bytes(B, H, n, d, num_splits))


def elsa_set_workspace(buf):
    """Lend a device byte buffer (torch uint8 tensor, kept alive by the caller) or None."""
    if buf is None:
        _check(_lib.elsa_set_workspace(None, 0))
    else:
        assert buf.is_cuda and buf.is_contiguous()
        _check(_lib.elsa_set_workspace(_ptr(buf), buf.numel() * buf.element_size()))


def elsa_set_option(option, value):
    _check(_lib.elsa_set_option(int(option), int(value)))


def elsa_get_option(option) -> int:
    v = ctypes.c_int(0)
    _check(_lib.elsa_get_option(int(option), ctypes.byref(v)))
    return v.value


def elsa_variant_name(path, variant):
    r = _lib.elsa_variant_name(int(path), int(variant))
    return None if r is None else r.decode()


def elsa_last_kernel() -> str:
    return _lib.elsa_last_kernel().decode()


def elsa_last_splits() -> int:
    return int(_lib.elsa_last_splits())


def elsa_debug_layout_probe(out, stream=None):
    _check(_lib.elsa_debug_layout_probe(_ptr(out), _stream(stream, out)))
    return out


def elsa_debug_issue_probe(out, kind_a, kind_b, waves_per_simd, iters, stream=None):
    """Measurement hook: ``out`` is a float32 device tensor of at least 8 + 256 * 512 elements."""
    import torch
    assert out.is_cuda and out.is_contiguous() and out.dtype == torch.float32 and out.numel() >= 8 + 256 * 512
    _check(_lib.elsa_debug_issue_probe(_ptr(out), int(kind_a), int(kind_b), int(waves_per_simd), int(iters), _stream(stream, out)))
    return out


def raw():
    """The ctypes library handle (for ABI tests)."""
    return _lib
