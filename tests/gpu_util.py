"""Helpers for the GPU parity tests: run the library through its C ABI and compare with the oracle."""
import numpy as np
import torch

import synth


def make_inputs(case, device="cuda"):
    """Seeded bf16 N(0,1) Q, K, V, dO for a ChunkCase (tensor ids 0..3)."""
    qs = (case.total_q, case.num_q_heads, case.head_dim)
    ks = (case.total_kv, case.num_kv_heads, case.head_dim)
    q = synth.normal_bf16(case.seed, 0, qs, device)
    k = synth.normal_bf16(case.seed, 1, ks, device)
    v = synth.normal_bf16(case.seed, 2, ks, device)
    do = synth.normal_bf16(case.seed, 3, qs, device)
    return q, k, v, do


def run_gpu(case, q, k, v, do=None, accumulate=False, dk_init=None, dv_init=None, scale=None, backward=True,
            f32kv=False):
    import paper_2509_21275_amd as ca
    scale = case.scale if scale is None else scale
    desc = ca.make_desc(case.segs, case.num_q_heads, case.num_kv_heads, case.head_dim, case.total_q, case.total_kv,
                        scale)
    ws = ca.alloc_workspace(desc)
    o = torch.full_like(q, float("nan"))
    lse = torch.full((case.num_q_heads, case.total_q), float("nan"), dtype=torch.float32, device=q.device)
    ca.chunk_attn_fwd(desc, q, k, v, o, lse, ws)
    if not backward:
        torch.cuda.synchronize()
        return o, lse
    dq = torch.full_like(q, float("nan"))
    if accumulate:
        dk = dk_init.clone(); dv = dv_init.clone()
    else:
        kv_dtype = torch.float32 if f32kv else k.dtype
        dk = torch.full_like(k, float("nan"), dtype=kv_dtype); dv = torch.full_like(v, float("nan"), dtype=kv_dtype)
    (ca.chunk_attn_bwd_f32kv if f32kv else ca.chunk_attn_bwd)(desc, q, k, v, o, do, lse, dq, dk, dv, accumulate, ws)
    torch.cuda.synchronize()
    return o, lse, dq, dk, dv


def rel_err(gpu, ref):
    """max |gpu - ref| / max |ref| over the compared elements (one ratio per tensor)."""
    g = gpu.detach().double().cpu().numpy() if isinstance(gpu, torch.Tensor) else np.asarray(gpu, dtype=np.float64)
    assert g.shape == ref.shape, (g.shape, ref.shape)
    assert np.all(np.isfinite(g)), "non-finite values in GPU result"
    denom = np.abs(ref).max()
    return float(np.abs(g - ref).max() / (denom if denom > 0 else 1.0))


TOL_O, TOL_GRAD = 2e-2, 5e-2
