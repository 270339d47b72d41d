"""The two variants' forward / backward passes as sequences of C-ABI calls.

Pure sequencing: sort or compact -> gather -> schedule -> attention.  Inputs and
outputs are ``[B,H,T,d]`` CUDA tensors in ORIGINAL order (paper Sec. 3, notations);
labels are ``[B,H,T]`` int32 bucket ids (hash) or uint8 keep flags (QK-dropping).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

from . import binding as sc


@dataclass
class Context:
    variant: int
    B: int
    H: int
    nb: int
    sm_scale: float
    flags: int
    q_p: torch.Tensor
    k_p: torch.Tensor
    v_p: torch.Tensor
    q_idx: torch.Tensor
    k_idx: torch.Tensor
    n_q: Optional[torch.Tensor]
    n_k: Optional[torch.Tensor]
    fwd_work: torch.Tensor
    bwd_work: Optional[torch.Tensor]
    counters: Optional[torch.Tensor]
    o: Optional[torch.Tensor] = None
    lse: Optional[torch.Tensor] = None
    o_f16: Optional[torch.Tensor] = None
    q_bucket_sorted: Optional[torch.Tensor] = None
    k_bucket_sorted: Optional[torch.Tensor] = None
    q_off: Optional[torch.Tensor] = None
    k_off: Optional[torch.Tensor] = None
    q_sort_key: Optional[torch.Tensor] = None
    k_sort_key: Optional[torch.Tensor] = None


def _seg(x):
    return x.reshape(x.shape[0] * x.shape[1], *x.shape[2:])


def _o_f16_buffer(q, need_bwd):
    """fp16 side copy of O for the backward's D = <dO, O> (bf16 path, training only).
    Rows of dropped queries are never written and never read back."""
    if not need_bwd or q.dtype != torch.bfloat16:
        return None
    return torch.empty(q.shape, dtype=torch.float16, device=q.device)


def hash_forward(q, k, v, bucket_q, bucket_k, nb, sm_scale, need_bwd=True, strict=False):
    """Hash-sparse attention forward (Sec. 3.2).  Returns (O, LSE, ctx)."""
    B, H, T, d = q.shape
    tiles = sc.scfa_tile_config(d, sc.dtype_code(q))
    flags = sc.SCFA_FLAG_STRICT_CAUSAL if strict else 0
    (q_idx, q_bs, q_off, q_key), (k_idx, k_bs, k_off, k_key) = sc.scfa_sort_by_bucket_pair(
        _seg(bucket_q), _seg(bucket_k), nb, want_sorted=False)
    q_p, k_p, v_p = sc.scfa_gather_qkv(_seg(q), _seg(k), _seg(v), q_idx, k_idx, to_f16=q.dtype == torch.bfloat16)
    fwd_work, bwd_work, counters = sc.scfa_block_ranges(sc.SCFA_HASH, q_idx, k_idx, q_off, k_off, nb, tiles,
                                                        want_bwd=need_bwd, flags=flags)
    o_f16 = _o_f16_buffer(q, need_bwd)
    o, lse = sc.scfa_hash_attn_fwd(q_p, k_p, v_p, q_key, k_key, fwd_work, B, H, sm_scale, o_f16_out=o_f16, flags=flags)
    ctx = Context(sc.SCFA_HASH, B, H, nb, sm_scale, flags, q_p, k_p, v_p, q_idx, k_idx, None, None, fwd_work, bwd_work,
                  counters, o, lse, o_f16, q_bs, k_bs, q_off, k_off, q_key, k_key)
    return o, lse, ctx


def hash_backward(ctx: Context, d_o, ws=None, outs=None):
    """dQ, dK, dV (fp32, original order) of hash-sparse attention."""
    return sc.scfa_hash_attn_bwd(ctx.q_p, ctx.k_p, ctx.v_p, ctx.q_sort_key, ctx.k_sort_key, ctx.fwd_work, ctx.bwd_work,
                                 ctx.o, ctx.lse, d_o, ctx.B, ctx.H, ctx.sm_scale, ws=ws, outs=outs, o_f16=ctx.o_f16, flags=ctx.flags)


def qkdrop_forward(q, k, v, keep_q, keep_k, sm_scale, need_bwd=True, strict=False):
    """QK-sparse attention forward (Sec. 3.1).  Returns (O, LSE, ctx)."""
    B, H, T, d = q.shape
    tiles = sc.scfa_tile_config(d, sc.dtype_code(q))
    flags = sc.SCFA_FLAG_STRICT_CAUSAL if strict else 0
    (q_idx, n_q), (k_idx, n_k) = sc.scfa_compact_keep_pair(_seg(keep_q), _seg(keep_k))
    q_c, k_c, v_c = sc.scfa_gather_qkv(_seg(q), _seg(k), _seg(v), q_idx, k_idx, n_q, n_k,
                                       to_f16=q.dtype == torch.bfloat16)
    fwd_work, bwd_work, counters = sc.scfa_block_ranges(sc.SCFA_QKDROP, q_idx, k_idx, n_q, n_k, 1, tiles,
                                                        want_bwd=need_bwd, flags=flags)
    o_f16 = _o_f16_buffer(q, need_bwd)
    o, lse = sc.scfa_qkdrop_attn_fwd(q_c, k_c, v_c, q_idx, k_idx, n_q, fwd_work, B, H, sm_scale, o_f16_out=o_f16, flags=flags)
    ctx = Context(sc.SCFA_QKDROP, B, H, 1, sm_scale, flags, q_c, k_c, v_c, q_idx, k_idx, n_q, n_k, fwd_work, bwd_work,
                  counters, o, lse, o_f16)
    return o, lse, ctx


def qkdrop_backward(ctx: Context, d_o, ws=None, outs=None):
    return sc.scfa_qkdrop_attn_bwd(ctx.q_p, ctx.k_p, ctx.v_p, ctx.q_idx, ctx.k_idx, ctx.n_q, ctx.n_k,
                                   ctx.fwd_work, ctx.bwd_work, ctx.o, ctx.lse, d_o, ctx.B, ctx.H, ctx.sm_scale,
                                   ws=ws, outs=outs, o_f16=ctx.o_f16, flags=ctx.flags)
