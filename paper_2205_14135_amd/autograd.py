"""torch.autograd front end of the attention library (argument marshalling only).

`flash_attention(q, k, v, ...)` returns O for [B,H,N,d] fp16/bf16 CUDA tensors and is
differentiable with respect to q, k and v: the forward saves O and the per-row logsumexp (the
O(N) state of Algorithm 2 of the paper) plus the dropout generator state (seed, offset), and the
backward regenerates the dropout mask and recomputes the probabilities tile by tile (Algorithm 4),
so no N x N tensor is ever kept.  Every step runs in the HIP library; there is no fallback.
"""
from __future__ import annotations

import math
from typing import Optional

import torch

from . import binding


class _FlashAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, softmax_scale, causal, dropout_p, seed, offset, key_lengths, block_mask):
        kw = dict(softmax_scale=softmax_scale, causal=causal, dropout_p=dropout_p, seed=seed, offset=offset,
                  key_lengths=key_lengths)
        if block_mask is None:
            out, lse = binding.attn_fwd(q, k, v, **kw)
        else:
            out, lse = binding.attn_blocksparse_fwd(q, k, v, block_mask, **kw)
        ctx.save_for_backward(q, k, v, out, lse)
        ctx.kw = kw
        ctx.block_mask = block_mask
        return out

    @staticmethod
    def backward(ctx, d_out):
        q, k, v, out, lse = ctx.saved_tensors
        if d_out.shape != q.shape or d_out.stride() != q.stride():
            # the library addresses dO with the strides of q
            d_out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device).copy_(d_out)
        if ctx.block_mask is None:
            dq, dk, dv = binding.attn_bwd(q, k, v, out, d_out, lse, **ctx.kw)
        else:
            dq, dk, dv = binding.attn_blocksparse_bwd(q, k, v, out, d_out, lse, ctx.block_mask, **ctx.kw)
        return dq, dk, dv, None, None, None, None, None, None, None


def flash_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, *, softmax_scale: Optional[float] = None,
                    causal: bool = False, dropout_p: float = 0.0, seed: Optional[int] = None, offset: int = 0,
                    key_lengths: Optional[torch.Tensor] = None,
                    block_mask: Optional[torch.Tensor] = None) -> torch.Tensor:
    """softmax(scale * q k^T + mask) v with dropout on the probabilities; exact attention.

    q, k, v: [B,H,N,d] fp16 or bf16 CUDA tensors with identical shape and strides, d contiguous,
    d in {16, 32, 64, 128}.  softmax_scale defaults to 1/sqrt(d).  key_lengths: int32 [B] true lengths
    (key-padding mask).  block_mask: uint8 [T,T] or [H,T,T] over 128 x 128 blocks (then N % 128 == 0).
    With dropout_p > 0 the mask is a pure function of (seed, offset, b, h, i, j); seed defaults to a
    draw from torch's CPU generator, so torch.manual_seed makes a run reproducible.
    """
    if not (q.is_cuda and k.is_cuda and v.is_cuda):
        raise RuntimeError("flash_attention runs on the GPU only: there is no CPU path")
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(q.shape[-1])
    if dropout_p > 0.0 and seed is None:
        seed = int(torch.randint(0, 2 ** 62, (), dtype=torch.int64).item())
    return _FlashAttention.apply(q, k, v, float(softmax_scale), bool(causal), float(dropout_p),
                                 int(seed or 0), int(offset), key_lengths, block_mask)
