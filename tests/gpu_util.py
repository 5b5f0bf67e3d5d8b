"""Helpers for the GPU parity tests: run the HIP path through the C ABI and hand back numpy."""
import numpy as np


def have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


class Options:
    """Set libelsa options for a block of code and restore the defaults afterwards."""

    def __init__(self, path=0, variant=0, splits=0, xcd_map=0, snake=0):
        self.vals = (path, variant, splits, xcd_map, snake)

    def __enter__(self):
        from paper_2604_23798_amd import elsa
        for o, v in enumerate(self.vals):
            elsa.elsa_set_option(o, v)
        return self

    def __exit__(self, *a):
        from paper_2604_23798_amd import elsa
        for o in range(6):
            elsa.elsa_set_option(o, 0)
        return False


def to_dev(a):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def fwd(q, k, v, scale, causal=False, kv_len=None, rows=None, masked_entry=None):
    """elsa_attn_fwd[_masked] on numpy inputs -> float64 [R, d] (all rows, or the sampled ones)."""
    import torch
    from paper_2604_23798_amd import elsa
    tq, tk, tv, tl = to_dev(q), to_dev(k), to_dev(v), to_dev(kv_len)
    out = torch.full_like(tq, float("nan"))
    if kv_len is None and not masked_entry:
        elsa.elsa_attn_fwd(tq, tk, tv, out, scale, causal)
    else:
        elsa.elsa_attn_fwd_masked(tq, tk, tv, out, scale, causal, tl)
    torch.cuda.synchronize()
    d = q.shape[-1]
    o = out.reshape(-1, d)
    if rows is not None:
        # the whole NaN-prefilled output was written, not only the rows the oracle is asked about
        assert bool(torch.isfinite(out).all()), "rows of the output were left unwritten or are not finite"
        o = o[torch.from_numpy(np.asarray(rows)).cuda()]
    return o.double().cpu().numpy()


def split_kv(q, k, v, scale, C, causal=False, kv_len=None):
    """elsa_attn_fwd_split_kv -> (m [BHn... as [R,C]], S [R,C], W [R,C,d]) float64, rows flattened (b,h,i)."""
    import torch
    from paper_2604_23798_amd import elsa
    B, H, n, d = q.shape
    tq, tk, tv, tl = to_dev(q), to_dev(k), to_dev(v), to_dev(kv_len)
    pm = torch.full((B, H, C, n), float("nan"), device="cuda")
    pS = torch.full((B, H, C, n), float("nan"), device="cuda")
    pW = torch.full((B, H, C, n, d), float("nan"), device="cuda")
    elsa.elsa_attn_fwd_split_kv(tq, tk, tv, pm, pS, pW, scale, C, causal, tl)
    torch.cuda.synchronize()
    return pm, pS, pW


def parts_to_rows(pm, pS, pW):
    B, H, C, n, d = pW.shape
    m = pm.permute(0, 1, 3, 2).reshape(B * H * n, C).double().cpu().numpy()
    S = pS.permute(0, 1, 3, 2).reshape(B * H * n, C).double().cpu().numpy()
    W = pW.permute(0, 1, 3, 2, 4).reshape(B * H * n, C, d).double().cpu().numpy()
    return m, S, W


def fwd_varlen(q, k, v, cu, max_seqlen, scale, causal=False):
    """elsa_attn_fwd_varlen on packed numpy inputs [T,H,d] -> float64 [T,H,d]."""
    import torch
    from paper_2604_23798_amd import elsa
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    tcu = torch.from_numpy(np.asarray(cu, np.int32)).cuda()
    out = torch.full_like(tq, float("nan"))
    elsa.elsa_attn_fwd_varlen(tq, tk, tv, out, tcu, max_seqlen, scale, causal)
    torch.cuda.synchronize()
    return out.double().cpu().numpy()


def fwd_cross(q, k, v, scale, causal=False, kv_len=None, want_lse=False):
    """elsa_attn_fwd_cross on numpy inputs (q [B,H,nq,d]; k, v [B,H,nk,d]) -> float64 [R, d] (, lse [R])."""
    import torch
    from paper_2604_23798_amd import elsa
    tq, tk, tv, tl = to_dev(q), to_dev(k), to_dev(v), to_dev(kv_len)
    out = torch.full_like(tq, float("nan"))
    lse = torch.full(tq.shape[:3], float("nan"), device="cuda") if want_lse else None
    elsa.elsa_attn_fwd_cross(tq, tk, tv, out, scale, causal, tl, lse)
    torch.cuda.synchronize()
    o = out.reshape(-1, q.shape[-1]).double().cpu().numpy()
    return (o, lse.reshape(-1).double().cpu().numpy()) if want_lse else o


def fwd_dv(q, k, v, scale, causal=False, kv_len=None, want_lse=False):
    """elsa_attn_fwd_dv on numpy inputs (q [B,H,nq,d]; k [B,H,nk,d]; v [B,H,nk,dv]) -> float64 [R, dv] (, lse [R])."""
    import torch
    from paper_2604_23798_amd import elsa
    tq, tk, tv, tl = to_dev(q), to_dev(k), to_dev(v), to_dev(kv_len)
    out = torch.full(tq.shape[:3] + (v.shape[-1],), float("nan"), device="cuda", dtype=tq.dtype)
    lse = torch.full(tq.shape[:3], float("nan"), device="cuda") if want_lse else None
    elsa.elsa_attn_fwd_dv(tq, tk, tv, out, scale, causal, tl, lse)
    torch.cuda.synchronize()
    o = out.reshape(-1, v.shape[-1]).double().cpu().numpy()
    return (o, lse.reshape(-1).double().cpu().numpy()) if want_lse else o
