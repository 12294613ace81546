"""Helpers shared by the GPU parity tests: bf16 bit patterns <-> torch tensors, oracle calls."""

import numpy as np
import torch

from oracle import s2_oracle as orc
from paper_2407_17678_amd import binding as B
from paper_2407_17678_amd import synth


def to_dev(bits):
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor on cuda:0 with the same bits."""
    return B.bf16_bits_to_device(bits)


def to_f64(t):
    """bf16 / fp32 device tensor -> float64 numpy (exact)."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def bits_f64(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def o_bound(want):
    """Per-element bound on |O - O_ref|: the stated max-abs 1e-2, except where a bf16 output cannot
    do that well: half a bf16 ulp at O_ref, 2^(floor(log2 |O_ref|) - 8), which exceeds 1e-2 only
    from |O_ref| = 4 on (0.0078 on [2, 4), 0.0156 on [4, 8))."""
    a = np.abs(np.asarray(want, dtype=np.float64))
    half_ulp = np.exp2(np.floor(np.log2(np.maximum(a, 2.0 ** -126))) - 8.0)
    return np.maximum(1e-2, half_ulp)


def o_excess(got, want):
    """Largest |got - want| minus o_bound(want).  Passing means <= 0."""
    return float((np.abs(got - want) - o_bound(want)).max())


def rel_l2(got, want):
    return float(np.linalg.norm((got - want).ravel()) / max(np.linalg.norm(want.ravel()), 1e-300))


def run_fwd(w, qb, kb, vb, dense=False):
    """Runs the library forward on bf16 bit patterns; returns (o, lse, layout, device tensors)."""
    q, k, v = to_dev(qb), to_dev(kb), to_dev(vb)
    Bt, H, N, D = q.shape
    o = torch.empty_like(q)
    lse = torch.empty((Bt, H, N), dtype=torch.float32, device="cuda")
    lay = None
    if dense:
        B.s2_dense_causal_fwd(q, k, v, o, lse, w.scale)
    else:
        lay = B.s2_layout_build(B.layout_params(H, N // w.block_size, w.block_size, w.local_blocks,
                                                w.stride, 0, w.window_blocks, 0))
        B.s2_attn_fwd(lay, q, k, v, o, lse, w.scale)
    torch.cuda.synchronize()
    return o, lse, lay, (q, k, v)


def oracle_mask(w, H, N, dense=False):
    return orc.block_mask(H, N // w.block_size, w.local_blocks, w.stride,
                          window_blocks=w.window_blocks, dense=dense)


def run_fwd_bwd(w, qb, kb, vb, gb, dense=False, keep_ds=False):
    """Library forward then backward; returns dict of device tensors.  keep_ds: the workspace of
    s2_attn_bwd_layout_workspace_bytes (filled with NaN patterns), which selects the backward that
    keeps dS where it applies."""
    q, k, v, g = to_dev(qb), to_dev(kb), to_dev(vb), to_dev(gb)
    Bt, H, N, D = q.shape
    o = torch.empty_like(q)
    lse = torch.empty((Bt, H, N), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(B.s2_attn_bwd_workspace_bytes(Bt, H, N, D), dtype=torch.uint8, device="cuda")
    if dense:
        B.s2_dense_causal_fwd(q, k, v, o, lse, w.scale)
        B.s2_dense_causal_bwd(q, k, v, o, lse, g, dq, dk, dv, w.scale, ws)
    else:
        lay = B.s2_layout_build(B.layout_params(H, N // w.block_size, w.block_size, w.local_blocks,
                                                w.stride, 0, w.window_blocks, 0))
        if keep_ds:
            ws = torch.full((B.s2_attn_bwd_layout_workspace_bytes(lay, Bt, H, N, D),), 0xFF, dtype=torch.uint8,
                            device="cuda")
        B.s2_attn_fwd(lay, q, k, v, o, lse, w.scale)
        B.s2_attn_bwd(lay, q, k, v, o, lse, g, dq, dk, dv, w.scale, ws)
    torch.cuda.synchronize()
    return dict(o=o, lse=lse, dq=dq, dk=dk, dv=dv, ws_bytes=ws.numel())
