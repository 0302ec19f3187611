"""torch.autograd front end of the attention library, for use inside a training step.

`attention(q, k, v)` and `attention_qkvpacked(qkv)` allocate the outputs, the saved log-sum-exp and the
backward workspace with torch and call the C-ABI entry points of `include/avion_attn.h` through the
binding in this package.  Nothing is computed here: every step of the forward and of the backward
runs in the HIP kernels, and there is no fallback if the library is missing.

What is saved for the backward is O(N) per (batch, head): q, k, v, o and the fp32 log-sum-exp -- no
N x N matrix (the memory saving of Sec. 4.1 of the paper).
"""
from __future__ import annotations

import math

import torch

from . import (attn_bwd, attn_bwd_causal, attn_bwd_f16, attn_bwd_qkvpacked, attn_bwd_workspace_bytes, attn_fwd,
               attn_fwd_causal, attn_fwd_f16, attn_fwd_qkvpacked)


def _workspace(B, H, N, d, device):
    return torch.empty(attn_bwd_workspace_bytes(B, H, N, d), dtype=torch.uint8, device=device)


class _Attention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, scale, causal):
        if q.dtype == torch.float16:
            if causal:
                raise ValueError("the causal entry points take bf16 tensors")
            fwd = attn_fwd_f16
        else:
            fwd = attn_fwd_causal if causal else attn_fwd
        q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
        B, N, H, d = q.shape
        o = torch.empty_like(q)
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
        fwd(q, k, v, o, lse, scale)
        ctx.save_for_backward(q, k, v, o, lse)
        ctx.scale, ctx.causal = scale, causal
        return o

    @staticmethod
    def backward(ctx, dO):
        q, k, v, o, lse = ctx.saved_tensors
        B, N, H, d = q.shape
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        if q.dtype == torch.float16:
            bwd = attn_bwd_f16
        else:
            bwd = attn_bwd_causal if ctx.causal else attn_bwd
        bwd(q, k, v, o, lse, dO.contiguous(), dq, dk, dv, ctx.scale, _workspace(B, H, N, d, q.device))
        return dq, dk, dv, None, None


class _AttentionPacked(torch.autograd.Function):
    @staticmethod
    def forward(ctx, qkv, scale):
        qkv = qkv.contiguous()
        B, N, _, H, d = qkv.shape
        o = torch.empty((B, N, H, d), dtype=qkv.dtype, device=qkv.device)
        lse = torch.empty((B, H, N), dtype=torch.float32, device=qkv.device)
        attn_fwd_qkvpacked(qkv, o, lse, scale)
        ctx.save_for_backward(qkv, o, lse)
        ctx.scale = scale
        return o

    @staticmethod
    def backward(ctx, dO):
        qkv, o, lse = ctx.saved_tensors
        B, N, _, H, d = qkv.shape
        dqkv = torch.empty_like(qkv)
        attn_bwd_qkvpacked(qkv, o, lse, dO.contiguous(), dqkv, ctx.scale, _workspace(B, H, N, d, qkv.device))
        return dqkv, None


def attention(q, k, v, scale: float | None = None, causal: bool = False):
    """softmax(scale * q k^T) v per (batch, head) for q, k, v of shape [B, N, H, d] (bf16, or fp16
    without `causal`), d in {64, 80}; differentiable.  scale defaults to 1/sqrt(d)."""
    return _Attention.apply(q, k, v, 1.0 / math.sqrt(q.shape[-1]) if scale is None else float(scale), bool(causal))


def attention_qkvpacked(qkv, scale: float | None = None):
    """The same for the [B, N, 3, H, d] bf16 output of a joint QKV projection; the gradient comes back
    in the same packing."""
    return _AttentionPacked.apply(qkv, 1.0 / math.sqrt(qkv.shape[-1]) if scale is None else float(scale))
