"""torch.autograd front end of the library, for use inside a training step.

`attention(q, k, v)` and `attention_qkvpacked(qkv)` allocate the outputs and the saved log-sum-exp with
torch and call the C-ABI entry points of `include/avion_attn.h` (the general forms, so every
combination of bf16 / fp16, causal or not, packed or not is available) through the binding in this
package.  Nothing is computed here: every step of the forward and of the backward runs in the HIP
kernels, and there is no fallback if the library is missing.

What is saved for the backward is O(N) per (batch, head): q, k, v, o and the fp32 log-sum-exp -- no
N x N matrix (the memory saving of Sec. 4.1 of the paper).

The backward's workspace is kept per (device, stream) and grown on demand, so a layer's backward does
not go through the allocator every step; backward calls on one stream are ordered and may share it.

`layer_norm(x, gamma, beta)` and `bias_gelu(x, bias)` wrap the layer-normalisation and bias + GELU
entry points the same way (what they keep for the backward is stated in their docstrings).
"""
from __future__ import annotations

import math

import torch

from . import (attn_bwd_ex, attn_bwd_workspace_bytes, attn_fwd_ex, bias_gelu_bwd, bias_gelu_bwd_workspace_bytes, bias_gelu_fwd,
               layernorm_bwd, layernorm_bwd_workspace_bytes, layernorm_fwd)

_workspaces: dict = {}


def _workspace_of(need, device):
    key = (device, torch.cuda.current_stream(device).cuda_stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < need:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def _workspace(B, H, N, d, device):
    return _workspace_of(attn_bwd_workspace_bytes(B, H, N, d), device)


class _Attention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, scale, causal):
        q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
        B, N, H, d = q.shape
        o = torch.empty_like(q)
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
        attn_fwd_ex(q, k, v, o, lse, scale, causal)
        ctx.save_for_backward(q, k, v, o, lse)
        ctx.scale, ctx.causal = scale, causal
        return o

    @staticmethod
    def backward(ctx, dO):
        q, k, v, o, lse = ctx.saved_tensors
        B, N, H, d = q.shape
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        attn_bwd_ex(q, k, v, o, lse, dO.contiguous(), dq, dk, dv, ctx.scale, _workspace(B, H, N, d, q.device), ctx.causal)
        return dq, dk, dv, None, None


class _AttentionPacked(torch.autograd.Function):
    @staticmethod
    def forward(ctx, qkv, scale, causal):
        qkv = qkv.contiguous()
        B, N, _, H, d = qkv.shape
        o = torch.empty((B, N, H, d), dtype=qkv.dtype, device=qkv.device)
        lse = torch.empty((B, H, N), dtype=torch.float32, device=qkv.device)
        attn_fwd_ex(qkv, None, None, o, lse, scale, causal)
        ctx.save_for_backward(qkv, o, lse)
        ctx.scale, ctx.causal = scale, causal
        return o

    @staticmethod
    def backward(ctx, dO):
        qkv, o, lse = ctx.saved_tensors
        B, N, _, H, d = qkv.shape
        dqkv = torch.empty_like(qkv)
        attn_bwd_ex(qkv, None, None, o, lse, dO.contiguous(), dqkv, None, None, ctx.scale,
                    _workspace(B, H, N, d, qkv.device), ctx.causal)
        return dqkv, None, None


class _LayerNorm(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, gamma, beta, eps):
        shape = x.shape
        x2 = x.contiguous().view(-1, shape[-1])
        M = x2.shape[0]
        y = torch.empty_like(x2)
        mean = torch.empty((M,), dtype=torch.float32, device=x.device)
        rstd = torch.empty((M,), dtype=torch.float32, device=x.device)
        layernorm_fwd(x2, gamma.contiguous(), beta.contiguous(), y, mean, rstd, eps)
        ctx.save_for_backward(x2, gamma, mean, rstd)   # the input and two floats per token; not y
        ctx.shape = shape
        return y.view(shape)

    @staticmethod
    def backward(ctx, dy):
        x2, gamma, mean, rstd = ctx.saved_tensors
        M, D = x2.shape
        dx = torch.empty_like(x2)
        dgamma, dbeta = torch.empty_like(gamma), torch.empty_like(gamma)
        layernorm_bwd(x2, gamma.contiguous(), mean, rstd, dy.contiguous().view(M, D), dx, dgamma, dbeta,
                      _workspace_of(layernorm_bwd_workspace_bytes(M, D), x2.device))
        return dx.view(ctx.shape), dgamma, dbeta, None


class _BiasGelu(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, bias):
        shape = x.shape
        x2 = x.contiguous().view(-1, shape[-1])
        y = torch.empty_like(x2)
        bias_gelu_fwd(x2, bias.contiguous(), y)
        ctx.save_for_backward(x2, bias)                # the pre-activation only; the derivative is rebuilt from it
        ctx.shape = shape
        return y.view(shape)

    @staticmethod
    def backward(ctx, dy):
        x2, bias = ctx.saved_tensors
        M, F = x2.shape
        dx, dbias = torch.empty_like(x2), torch.empty_like(bias)
        bias_gelu_bwd(x2, bias.contiguous(), dy.contiguous().view(M, F), dx, dbias,
                      _workspace_of(bias_gelu_bwd_workspace_bytes(M, F), x2.device))
        return dx.view(ctx.shape), dbias


class _BiasGeluLinear(torch.autograd.Function):
    """linear(GELU(x + bias), weight, out_bias) that keeps x only: the activation's output is rebuilt in the
    backward pass (one more avion_bias_gelu_fwd) for the weight gradient.  The two matrix products per
    direction are torch's (library GEMMs)."""

    @staticmethod
    def forward(ctx, x, bias, weight, out_bias):
        shape = x.shape
        x2 = x.contiguous().view(-1, shape[-1])
        y = torch.empty_like(x2)
        bias_gelu_fwd(x2, bias.contiguous(), y)
        out = torch.addmm(out_bias, y, weight.t()) if out_bias is not None else y @ weight.t()
        ctx.save_for_backward(x2, bias, weight)
        ctx.shape, ctx.has_out_bias = shape, out_bias is not None
        return out.view(*shape[:-1], weight.shape[0])

    @staticmethod
    def backward(ctx, dout):
        x2, bias, weight = ctx.saved_tensors
        M, F = x2.shape
        d2 = dout.contiguous().view(M, weight.shape[0])
        y = torch.empty_like(x2)
        bias_gelu_fwd(x2, bias.contiguous(), y)          # rebuilt, not kept
        dweight = d2.t() @ y
        dy = d2 @ weight
        del y
        dx, dbias = torch.empty_like(x2), torch.empty_like(bias)
        bias_gelu_bwd(x2, bias.contiguous(), dy, dx, dbias, _workspace_of(bias_gelu_bwd_workspace_bytes(M, F), x2.device))
        return dx.view(ctx.shape), dbias, dweight, (d2.sum(0) if ctx.has_out_bias else None)


def bias_gelu_linear(x, bias, weight, out_bias=None):
    """linear(GELU(x + bias), weight, out_bias): the second half of the encoder's MLP, keeping only x (the
    first matrix product's output) for the backward; x bf16 or fp16 [..., F], bias fp32 [F], weight
    [out, F] and out_bias [out] in the format of x."""
    return _BiasGeluLinear.apply(x, bias, weight, out_bias)


def layer_norm(x, gamma, beta, eps: float = 1e-5):
    """Layer normalisation over the last axis of x (bf16 or fp16, any leading shape, width <= 2048 and a
    multiple of 8) with fp32 gain and bias.  Differentiable in x, gamma and beta; keeps x and two floats
    per token for the backward."""
    return _LayerNorm.apply(x, gamma, beta, float(eps))


def bias_gelu(x, bias):
    """GELU(x + bias) (exact erf form) over the last axis of x (bf16 or fp16, width a multiple of 8) with
    an fp32 bias.  Differentiable in x and bias; keeps only x for the backward."""
    return _BiasGelu.apply(x, bias)


def attention(q, k, v, scale: float | None = None, causal: bool = False):
    """softmax(scale * q k^T) v per (batch, head) for q, k, v of shape [B, N, H, d], bf16 or fp16,
    d in {64, 80}; `causal`: query i attends to keys 0..i.  Differentiable.  scale defaults to 1/sqrt(d)."""
    return _Attention.apply(q, k, v, 1.0 / math.sqrt(q.shape[-1]) if scale is None else float(scale), bool(causal))


def attention_qkvpacked(qkv, scale: float | None = None, causal: bool = False):
    """The same for the [B, N, 3, H, d] output of a joint QKV projection (bf16 or fp16); the gradient
    comes back in the same packing."""
    return _AttentionPacked.apply(qkv, 1.0 / math.sqrt(qkv.shape[-1]) if scale is None else float(scale), bool(causal))
