"""Seeded synthetic inputs for the attention hot path, shared by the CPU oracle's tests and the HIP path.

This module holds none of the method's arithmetic: it only produces bf16 bit patterns
(as numpy uint16) for Q, K, V and dO in the `[B, N, H, d]` layout, plus the workload table.
It imports neither the oracle nor the HIP binding, so both sides see byte-identical inputs.

Workload shapes follow the paper's video tokenisation (Sec. 3, "Video Transformer":
N = T/t * H/h * W/w cubes) and the VideoMAE setting of Sec. 5.5 (16 frames, cubes of
2x16x16 at 224^2 -> 8*14*14 = 1568 tokens).  The paper's activations come from real video
datasets with pretrained weights; here iid N(0,1) values rounded to bf16 stand in for them.

Generator: counter based.  Element `i` of stream `s` under `seed` draws two 64-bit words from
splitmix64 on a key built from (seed, s, i), maps them to uniforms in (0,1] and [0,1), and
applies the Box-Muller cosine branch in fp64; the result is rounded to fp32 and then to bf16
with round-to-nearest-even.  No state is kept, so any slice can be produced on its own.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on an array of uint64 (wraps modulo 2^64)."""
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even. NaN is not expected here."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp64, exact."""
    return bf16_bits_to_f32(b).astype(np.float64)


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> IEEE fp16 bit patterns (uint16), round to nearest even (numpy's conversion)."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """fp16 bit patterns (uint16) -> fp64, exact."""
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float64)


def _normal_f64(seed: int, stream: int, start: int, n: int) -> np.ndarray:
    """Elements start..start+n-1 of the N(0,1) stream (seed, stream), in fp64."""
    with np.errstate(over="ignore"):
        key = _mix64(np.uint64(seed & 0xFFFFFFFFFFFFFFFF) * _GOLD + np.uint64(stream + 1) * _M2)
        idx = np.arange(start, start + n, dtype=np.uint64)
        a = _mix64(key + (idx * np.uint64(2) + np.uint64(1)) * _GOLD)
        b = _mix64(key + (idx * np.uint64(2) + np.uint64(2)) * _GOLD)
    # u1 in (0,1], u2 in [0,1): 53-bit mantissas
    u1 = ((a >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
    u2 = (b >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * math.pi) * u2)


def normal_bf16_bits(seed: int, stream: int, count: int, offset: int = 0, chunk: int = 1 << 22,
                     to_bits=None) -> np.ndarray:
    """`count` iid N(0,1) draws, elements offset..offset+count-1 of (seed, stream), as bf16 bits
    (or, with to_bits=f32_to_f16_bits, the same draws rounded to fp16)."""
    to_bits = to_bits or f32_to_bf16_bits
    out = np.empty(count, dtype=np.uint16)
    for start in range(0, count, chunk):
        n = min(chunk, count - start)
        out[start:start + n] = to_bits(_normal_f64(seed, stream, offset + start, n).astype(np.float32))
    return out


def normal_f32(seed: int, stream: int, count: int, offset: int = 0, chunk: int = 1 << 22) -> np.ndarray:
    """The same draws, rounded to fp32 only (for fp32 parameters such as a normalisation's gain)."""
    out = np.empty(count, dtype=np.float32)
    for start in range(0, count, chunk):
        n = min(chunk, count - start)
        out[start:start + n] = _normal_f64(seed, stream, offset + start, n).astype(np.float32)
    return out


@dataclasses.dataclass(frozen=True)
class Workload:
    """One attention problem: Q, K, V, dO of shape [B, N, H, d] bf16; non-causal self-attention."""
    name: str
    B: int
    H: int
    N: int
    d: int
    scale: float
    seed: int
    k_mul: float = 1.0   # K is multiplied by this power of two after rounding (exact in bf16)
    note: str = ""

    @property
    def shape(self):
        return (self.B, self.N, self.H, self.d)

    @property
    def base(self) -> float:
        """B*H*N^2*d: fwd is 4*base flops, bwd 10*base, fwd+bwd 14*base."""
        return float(self.B) * self.H * self.N * self.N * self.d


WORKLOADS = {
    w.name: w
    for w in [
        Workload("vitb_clip", 1, 12, 1568, 64, 0.125, 230916691,
                 note="one ViT-B layer on one 16-frame 224^2 clip, cubes 2x16x16 -> 8*14*14 tokens"),
        Workload("vitb_batch", 32, 12, 1568, 64, 0.125, 230916692,
                 note="ViT-B video training batch of 32 clips"),
        Workload("vitl_batch_peaky", 16, 16, 1568, 64, 0.125, 230916693, k_mul=2.0,
                 note="ViT-L heads, K doubled for a peakier softmax"),
        Workload("vitb_long", 8, 12, 3136, 64, 0.125, 230916694,
                 note="32 frames -> 16*14*14 tokens"),
        Workload("vith_d80", 8, 16, 1568, 80, 1.0 / math.sqrt(80.0), 230916695,
                 note="ViT-H-width head dim 80"),
        Workload("vitl_336", 4, 16, 3528, 64, 0.125, 230916696,
                 note="16 frames at 336^2 -> 8*21*21 tokens"),
    ]
}

# Shapes of the small-sequence regime (not among the named benchmark configurations): the text encoder of
# the video-language model (at most 77 tokens, causal) for 2048 captions, and the two attentions of a
# divided space/time model (the comparison architecture of Sec. 4.1) on 32 clips of 8 frames.
WORKLOADS.update({
    w.name: w
    for w in [
        Workload("text_77", 2048, 8, 77, 64, 0.125, 230916701, note="text-encoder layer, 2048 captions of 77 tokens (use the causal entry points)"),
        Workload("temporal_16", 32 * 196, 12, 16, 64, 0.125, 230916702, note="temporal attention: one problem of T = 16 frames per spatial position"),
        Workload("spatial_196", 32 * 8, 12, 196, 64, 0.125, 230916703, note="spatial attention: one problem of 14 x 14 tokens per frame"),
    ]
})

STREAMS = {"q": 0, "k": 1, "v": 2, "dO": 3}


def make_inputs(w: Workload, names=("q", "k", "v", "dO"), fmt: str = "bf16") -> dict:
    """Bit patterns (uint16 arrays of shape [B,N,H,d]) for the requested tensors of a workload, in
    bf16 or, with fmt="f16", the same draws rounded to fp16."""
    if fmt not in ("bf16", "f16"):
        raise ValueError(f"unknown element format {fmt!r}")
    count = w.B * w.N * w.H * w.d
    out = {}
    for name in names:
        if fmt == "bf16":
            bits = normal_bf16_bits(w.seed, STREAMS[name], count)
            if name == "k" and w.k_mul != 1.0:
                scaled = bf16_bits_to_f32(bits) * np.float32(w.k_mul)
                bits = f32_to_bf16_bits(scaled)   # exact: a power-of-two multiple
        else:
            bits = normal_bf16_bits(w.seed, STREAMS[name], count, to_bits=f32_to_f16_bits)
            if name == "k" and w.k_mul != 1.0:
                scaled = bits.view(np.float16).astype(np.float32) * np.float32(w.k_mul)
                bits = f32_to_f16_bits(scaled)    # exact for these magnitudes: a power-of-two multiple
        out[name] = bits.reshape(w.shape)
    return out


def small_workload(B, H, N, d, seed, scale=None, k_mul=1.0, name=None) -> Workload:
    """A reduced problem with the same recipe, for parity cases the oracle finishes in seconds."""
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    return Workload(name or f"small_B{B}_H{H}_N{N}_d{d}", B, H, N, d, scale, seed, k_mul)



def layernorm_inputs(M: int, D: int, seed: int, fmt: str = "bf16") -> dict:
    """Seeded inputs of a layer normalisation over [M, D] tokens: x and dy ~ N(0,1) as bit patterns of
    `fmt`, gain 1 + 0.1 N(0,1) and bias 0.1 N(0,1) in fp32 (stand-ins for trained parameters)."""
    to_bits = f32_to_f16_bits if fmt == "f16" else f32_to_bf16_bits
    return {
        "x": normal_bf16_bits(seed, 10, M * D, to_bits=to_bits).reshape(M, D),
        "dy": normal_bf16_bits(seed, 11, M * D, to_bits=to_bits).reshape(M, D),
        "gamma": (np.float32(1.0) + np.float32(0.1) * normal_f32(seed, 12, D)).astype(np.float32),
        "beta": (np.float32(0.1) * normal_f32(seed, 13, D)).astype(np.float32),
    }


def gelu_inputs(M: int, F: int, seed: int, fmt: str = "bf16") -> dict:
    """Seeded inputs of a bias + GELU step over [M, F]: x ~ 1.5 N(0,1) (the first MLP layer's output
    without bias; wide enough to reach both tails of the activation) and dy ~ N(0,1) as bit patterns of
    `fmt`, bias 0.1 N(0,1) in fp32."""
    to_bits = f32_to_f16_bits if fmt == "f16" else f32_to_bf16_bits
    x = (np.float32(1.5) * normal_f32(seed, 20, M * F)).astype(np.float32)
    return {
        "x": to_bits(x).reshape(M, F),
        "dy": normal_bf16_bits(seed, 21, M * F, to_bits=to_bits).reshape(M, F),
        "bias": (np.float32(0.1) * normal_f32(seed, 22, F)).astype(np.float32),
    }

