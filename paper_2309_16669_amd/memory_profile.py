"""Activation memory and speed of a plain video-ViT encoder on one GPU, with and without this library.

    python -m paper_2309_16669_amd.memory_profile [--tokens 784] [--batch 16] [--layers 12] [--dtype bf16]

Measures what the paper's memory profile shows (Sec. 4.1, figure "memory footprint": MB per video kept
for the backward pass by the three kinds of layer -- LayerNorm, multi-head attention, MLP -- for a
plain ViT, the same with memory-efficient attention, and the same with gradient checkpointing) on a
randomly initialised ViT-B-shaped encoder (the paper's weights and clips are not available; shapes only:
by default 4 frames of 224 x 224 in 16 x 16 x 1 cubes = 784 tokens, width 768, 12 heads, 12 layers).

Variants
  plain        every step in PyTorch: the attention forms softmax(Q K^T / sqrt d) explicitly, so autograd
               keeps N x N tensors per head and layer
  attention    this library's attention (nothing N x N is kept: O, and one fp32 per head and token)
  all kernels  attention, layer normalisation and the MLP's bias + GELU from this library (the activation's
               output is rebuilt in the backward pass instead of kept)
  checkpoint   the last variant with every layer recomputed in the backward pass (Sec. 4.1)

The matrix products are torch's (library GEMMs) in every variant.  The bytes autograd keeps are counted
with saved-tensor hooks and attributed to the module that was running when the tensor was saved; a
tensor kept by several consumers counts once, for the first.  Nothing here is part of the kernels'
hot path or of any reported benchmark figure.
"""
from __future__ import annotations

import argparse
import json
import math
import time

import torch
import torch.nn.functional as F
import torch.utils.checkpoint
from torch import nn

from . import autograd as ag


class Norm(nn.Module):
    def __init__(self, width, fused):
        super().__init__()
        self.gamma = nn.Parameter(torch.ones(width))
        self.beta = nn.Parameter(torch.zeros(width))
        self.fused = fused

    def forward(self, x):
        if self.fused:
            return ag.layer_norm(x, self.gamma, self.beta, 1e-5)
        return F.layer_norm(x, (x.shape[-1],), self.gamma.to(x.dtype), self.beta.to(x.dtype), 1e-5)


class Attention(nn.Module):
    def __init__(self, width, heads, dtype, ours):
        super().__init__()
        self.heads, self.ours = heads, ours
        self.qkv = nn.Linear(width, 3 * width, dtype=dtype)
        self.proj = nn.Linear(width, width, dtype=dtype)

    def forward(self, x):
        B, N, W = x.shape
        d = W // self.heads
        qkv = self.qkv(x).view(B, N, 3, self.heads, d)
        if self.ours:
            o = ag.attention_qkvpacked(qkv)
        else:
            q, k, v = (qkv[:, :, i].transpose(1, 2) for i in range(3))          # [B, H, N, d]
            p = torch.softmax((q @ k.transpose(-1, -2)) * (1.0 / math.sqrt(d)), dim=-1)
            o = (p @ v).transpose(1, 2)
        return self.proj(o.reshape(B, N, W))


class Mlp(nn.Module):
    def __init__(self, width, dtype, fused):
        super().__init__()
        self.fused = fused
        self.fc1 = nn.Linear(width, 4 * width, bias=not fused, dtype=dtype)
        self.bias1 = nn.Parameter(torch.zeros(4 * width)) if fused else None
        self.fc2 = nn.Linear(4 * width, width, dtype=dtype)

    def forward(self, x):
        h = self.fc1(x)
        if self.fused:  # keeps h only: the activation's output is rebuilt in the backward pass
            return ag.bias_gelu_linear(h, self.bias1, self.fc2.weight, self.fc2.bias)
        return self.fc2(F.gelu(h))


class Layer(nn.Module):
    def __init__(self, width, heads, dtype, ours_attention, fused):
        super().__init__()
        self.norm1, self.norm2 = Norm(width, fused), Norm(width, fused)
        self.attn = Attention(width, heads, dtype, ours_attention)
        self.mlp = Mlp(width, dtype, fused)

    def forward(self, x):
        x = x + self.attn(self.norm1(x))
        return x + self.mlp(self.norm2(x))


class Encoder(nn.Module):
    def __init__(self, layers, width, heads, dtype, ours_attention, fused, checkpoint):
        super().__init__()
        self.layers = nn.ModuleList(Layer(width, heads, dtype, ours_attention, fused) for _ in range(layers))
        self.checkpoint = checkpoint

    def forward(self, x):
        for layer in self.layers:
            if self.checkpoint:
                x = torch.utils.checkpoint.checkpoint(layer, x, use_reentrant=False)
            else:
                x = layer(x)
        return x


KINDS = {Norm: "LayerNorm", Attention: "MHA", Mlp: "MLP"}


def saved_bytes_by_kind(model, x):
    """One forward pass under saved-tensor hooks: bytes kept for the backward, by kind of layer."""
    current = ["other"]
    seen, totals = set(), {"LayerNorm": 0, "MHA": 0, "MLP": 0, "other": 0}
    handles = []
    for m in model.modules():
        kind = KINDS.get(type(m))
        if kind:
            handles.append(m.register_forward_pre_hook(lambda mod, args, kind=kind: current.__setitem__(0, kind)))
            handles.append(m.register_forward_hook(lambda mod, args, out: current.__setitem__(0, "other")))
    params = {p.data_ptr() for p in model.parameters()}

    def pack(t):
        key = (t.data_ptr(), t.numel() * t.element_size())
        if t.data_ptr() not in params and key not in seen and t.is_cuda:
            seen.add(key)
            totals[current[0]] += t.numel() * t.element_size()
        return t

    with torch.autograd.graph.saved_tensors_hooks(pack, lambda t: t):
        y = model(x)
    for h in handles:
        h.remove()
    return totals, y


def step_time_and_peak(model, x, steps=5):
    def step():
        for p in model.parameters():
            p.grad = None
        y = model(x)
        y.float().square().mean().backward()
    step()
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    before = torch.cuda.memory_allocated()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps, torch.cuda.max_memory_allocated() - before


def profile(tokens=784, batch=16, layers=12, width=768, heads=12, dtype=torch.bfloat16, steps=5):
    variants = [("plain", False, False, False), ("attention", True, False, False), ("all kernels", True, True, False),
                ("checkpoint", True, True, True)]
    out = {"tokens": tokens, "batch": batch, "layers": layers, "width": width, "heads": heads, "dtype": str(dtype), "variants": {}}
    for name, ours, fused, ckpt in variants:
        torch.manual_seed(0)
        model = Encoder(layers, width, heads, dtype, ours, fused, ckpt).cuda()
        x = torch.randn((batch, tokens, width), device="cuda").to(dtype).requires_grad_()
        totals, _ = saved_bytes_by_kind(model, x)
        sec, peak = step_time_and_peak(model, x, steps)
        out["variants"][name] = {
            "saved_MB_per_video": {k: v / batch / 1e6 for k, v in totals.items()},
            "peak_activation_MB_per_video": peak / batch / 1e6,
            "videos_per_second": batch / sec,
        }
        del model, x
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--tokens", type=int, default=784)
    ap.add_argument("--batch", type=int, default=16)
    ap.add_argument("--layers", type=int, default=12)
    ap.add_argument("--dtype", choices=["bf16", "f16"], default="bf16")
    ap.add_argument("--steps", type=int, default=5)
    a = ap.parse_args()
    res = profile(a.tokens, a.batch, a.layers, dtype=torch.float16 if a.dtype == "f16" else torch.bfloat16, steps=a.steps)
    for name, v in res["variants"].items():
        s = v["saved_MB_per_video"]
        print(f"{name:12s} kept for backward, MB/video: LayerNorm {s['LayerNorm']:7.2f}  MHA {s['MHA']:8.2f}  MLP {s['MLP']:7.2f}  other {s['other']:6.2f}"
              f" | peak {v['peak_activation_MB_per_video']:8.1f} MB/video | {v['videos_per_second']:7.1f} videos/s", flush=True)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
