"""MI355X-native exact O(N)-memory attention (forward + backward) behind a C ABI.

`attn_fwd`, `attn_bwd`, `attn_bwd_workspace_bytes`, `attn_fwd_qkvpacked`, ... mirror the entry points
of `include/avion_attn.h` one to one.  This module only marshals arguments (device pointers, sizes,
the current HIP stream); every step of the computation runs in the HIP kernels of
`libavion_attn.so`.  There is no CPU or PyTorch fallback: if the library is missing, loading fails.
PyTorch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libavion_attn.so")

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP, ESCRATCH = 0, -1, -2, -3, -4, -5
FLAG_F16, FLAG_CAUSAL, FLAG_QKVPACKED = 1, 2, 4

_lib = None


class AvionError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"avion_attn error {code}: {text}")
        self.code = code


def load_library() -> ctypes.CDLL:
    """Load the HIP library built in-tree. Raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
                "or python paper_2309_16669_amd/build.py); there is no fallback path")
        lib = ctypes.CDLL(LIB_PATH)
        p, i, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        lib.avion_version.restype = i
        lib.avion_version.argtypes = []
        lib.avion_strerror.restype = ctypes.c_char_p
        lib.avion_strerror.argtypes = [i]
        lib.avion_last_hip_error.restype = ctypes.c_char_p
        lib.avion_last_hip_error.argtypes = []
        lib.avion_attn_fwd.restype = i
        lib.avion_attn_fwd.argtypes = [p, p, p, p, p, i, i, i, i, f, p]
        lib.avion_attn_bwd_workspace_bytes.restype = sz
        lib.avion_attn_bwd_workspace_bytes.argtypes = [i, i, i, i]
        lib.avion_attn_bwd.restype = i
        lib.avion_attn_bwd.argtypes = [p, p, p, p, p, p, p, p, p, i, i, i, i, f, p, sz, p]
        lib.avion_attn_bwd_dq.restype = i
        lib.avion_attn_bwd_dq.argtypes = [p, p, p, p, p, p, p, i, i, i, i, f, p, sz, p]
        lib.avion_attn_bwd_dkdv.restype = i
        lib.avion_attn_bwd_dkdv.argtypes = [p, p, p, p, p, p, p, i, i, i, i, f, p, sz, p]
        lib.avion_attn_fwd_qkvpacked.restype = i
        lib.avion_attn_fwd_qkvpacked.argtypes = [p, p, p, i, i, i, i, f, p]
        lib.avion_attn_bwd_qkvpacked.restype = i
        lib.avion_attn_bwd_qkvpacked.argtypes = [p, p, p, p, p, i, i, i, i, f, p, sz, p]
        lib.avion_attn_fwd_f16.restype = i
        lib.avion_attn_fwd_f16.argtypes = lib.avion_attn_fwd.argtypes
        lib.avion_attn_bwd_f16.restype = i
        lib.avion_attn_bwd_f16.argtypes = lib.avion_attn_bwd.argtypes
        lib.avion_attn_fwd_causal.restype = i
        lib.avion_attn_fwd_causal.argtypes = lib.avion_attn_fwd.argtypes
        lib.avion_attn_bwd_causal.restype = i
        lib.avion_attn_bwd_causal.argtypes = lib.avion_attn_bwd.argtypes
        u = ctypes.c_uint
        lib.avion_attn_fwd_ex.restype = i
        lib.avion_attn_fwd_ex.argtypes = [p, p, p, p, p, i, i, i, i, f, u, p]
        lib.avion_attn_bwd_ex.restype = i
        lib.avion_attn_bwd_ex.argtypes = [p, p, p, p, p, p, p, p, p, i, i, i, i, f, u, p, sz, p]
        ll = ctypes.c_longlong
        lib.avion_layernorm_fwd.restype = i
        lib.avion_layernorm_fwd.argtypes = [p, p, p, p, p, p, ll, i, f, u, p]
        lib.avion_layernorm_bwd_workspace_bytes.restype = sz
        lib.avion_layernorm_bwd_workspace_bytes.argtypes = [ll, i]
        lib.avion_layernorm_bwd.restype = i
        lib.avion_layernorm_bwd.argtypes = [p, p, p, p, p, p, p, p, ll, i, u, p, sz, p]
        lib.avion_bias_gelu_fwd.restype = i
        lib.avion_bias_gelu_fwd.argtypes = [p, p, p, ll, i, u, p]
        lib.avion_bias_gelu_bwd_workspace_bytes.restype = sz
        lib.avion_bias_gelu_bwd_workspace_bytes.argtypes = [ll, i]
        lib.avion_bias_gelu_bwd.restype = i
        lib.avion_bias_gelu_bwd.argtypes = [p, p, p, p, p, ll, i, u, p, sz, p]
        lib.avion_attn_bwd_noalloc.restype = i
        lib.avion_attn_bwd_noalloc.argtypes = [p, p, p, p, p, p, p, p, p, i, i, i, i, f, p]
        _lib = lib
    return _lib


def version() -> int:
    return int(load_library().avion_version())


def strerror(code: int) -> str:
    return load_library().avion_strerror(int(code)).decode()


def _check(rc: int):
    if rc != OK:
        lib = load_library()
        text = strerror(rc)
        if rc == EHIP:
            text += ": " + lib.avion_last_hip_error().decode()
        raise AvionError(rc, text)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _stream_handle(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _require(t, name, dtype, shape=None):
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")


def attn_bwd_workspace_bytes(B: int, H: int, N: int, d: int) -> int:
    return int(load_library().avion_attn_bwd_workspace_bytes(B, H, N, d))


def _fwd(entry, dt, q, k, v, o, lse, scale, stream):
    import torch
    B, N, H, d = q.shape
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (o, "o")):
        _require(t, n, dt, (B, N, H, d))
    _require(lse, "lse", torch.float32, (B, H, N))
    _check(entry(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, H, N, d, float(scale), _stream_handle(stream)))


def _bwd(entry, dt, q, k, v, o, lse, dO, dq, dk, dv, scale, workspace, stream):
    import torch
    B, N, H, d = q.shape
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (o, "o"), (dO, "dO"), (dq, "dq"), (dk, "dk"), (dv, "dv")):
        _require(t, n, dt, (B, N, H, d))
    _require(lse, "lse", torch.float32, (B, H, N))
    _require(workspace, "workspace", torch.uint8)
    _check(entry(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(dO), _ptr(dq), _ptr(dk), _ptr(dv), B, H, N, d,
                 float(scale), _ptr(workspace), workspace.numel(), _stream_handle(stream)))


def attn_fwd(q, k, v, o, lse, scale: float, stream=None) -> None:
    """avion_attn_fwd on torch tensors: q,k,v,o bf16 [B,N,H,d] on the GPU; lse fp32 [B,H,N]."""
    import torch
    _fwd(load_library().avion_attn_fwd, torch.bfloat16, q, k, v, o, lse, scale, stream)


def attn_fwd_f16(q, k, v, o, lse, scale: float, stream=None) -> None:
    """avion_attn_fwd_f16: the same on fp16 tensors."""
    import torch
    _fwd(load_library().avion_attn_fwd_f16, torch.float16, q, k, v, o, lse, scale, stream)


def attn_bwd(q, k, v, o, lse, dO, dq, dk, dv, scale: float, workspace, stream=None) -> None:
    """avion_attn_bwd on torch tensors; `workspace` is a uint8 GPU tensor of at least
    attn_bwd_workspace_bytes(B,H,N,d) bytes."""
    import torch
    _bwd(load_library().avion_attn_bwd, torch.bfloat16, q, k, v, o, lse, dO, dq, dk, dv, scale, workspace, stream)


def attn_bwd_noalloc(q, k, v, o, lse, dO, dq, dk, dv, scale: float, stream=None) -> None:
    """avion_attn_bwd_noalloc: avion_attn_bwd without a workspace argument (the library's built-in
    32 MiB scratch takes its place; larger problems raise AvionError with code ESCRATCH)."""
    import torch
    B, N, H, d = q.shape
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (o, "o"), (dO, "dO"), (dq, "dq"), (dk, "dk"), (dv, "dv")):
        _require(t, n, torch.bfloat16, (B, N, H, d))
    _require(lse, "lse", torch.float32, (B, H, N))
    _check(load_library().avion_attn_bwd_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(dO), _ptr(dq),
                                                 _ptr(dk), _ptr(dv), B, H, N, d, float(scale), _stream_handle(stream)))


def attn_bwd_f16(q, k, v, o, lse, dO, dq, dk, dv, scale: float, workspace, stream=None) -> None:
    """avion_attn_bwd_f16: the same on fp16 tensors."""
    import torch
    _bwd(load_library().avion_attn_bwd_f16, torch.float16, q, k, v, o, lse, dO, dq, dk, dv, scale, workspace, stream)


def attn_fwd_causal(q, k, v, o, lse, scale: float, stream=None) -> None:
    """avion_attn_fwd_causal: bf16 tensors, query i attends to keys 0..i."""
    import torch
    _fwd(load_library().avion_attn_fwd_causal, torch.bfloat16, q, k, v, o, lse, scale, stream)


def attn_bwd_causal(q, k, v, o, lse, dO, dq, dk, dv, scale: float, workspace, stream=None) -> None:
    """avion_attn_bwd_causal: gradients of the causal forward."""
    import torch
    _bwd(load_library().avion_attn_bwd_causal, torch.bfloat16, q, k, v, o, lse, dO, dq, dk, dv, scale, workspace,
         stream)


def attn_bwd_dq(q, k, v, o, lse, dO, dq, scale: float, workspace, stream=None) -> None:
    """avion_attn_bwd_dq: first phase of the backward (delta into the workspace, and dQ)."""
    import torch
    B, N, H, d = q.shape
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (o, "o"), (dO, "dO"), (dq, "dq")):
        _require(t, n, torch.bfloat16, (B, N, H, d))
    _require(lse, "lse", torch.float32, (B, H, N))
    _require(workspace, "workspace", torch.uint8)
    _check(load_library().avion_attn_bwd_dq(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(dO), _ptr(dq),
                                            B, H, N, d, float(scale), _ptr(workspace), workspace.numel(),
                                            _stream_handle(stream)))


def attn_bwd_dkdv(q, k, v, lse, dO, dk, dv, scale: float, workspace, stream=None) -> None:
    """avion_attn_bwd_dkdv: second phase of the backward (dK, dV; reads delta from the workspace)."""
    import torch
    B, N, H, d = q.shape
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (dO, "dO"), (dk, "dk"), (dv, "dv")):
        _require(t, n, torch.bfloat16, (B, N, H, d))
    _require(lse, "lse", torch.float32, (B, H, N))
    _require(workspace, "workspace", torch.uint8)
    _check(load_library().avion_attn_bwd_dkdv(_ptr(q), _ptr(k), _ptr(v), _ptr(lse), _ptr(dO), _ptr(dk), _ptr(dv),
                                              B, H, N, d, float(scale), _ptr(workspace), workspace.numel(),
                                              _stream_handle(stream)))


def attn_fwd_qkvpacked(qkv, o, lse, scale: float, stream=None) -> None:
    """avion_attn_fwd_qkvpacked: qkv bf16 [B,N,3,H,d] (the joint projection's output), o bf16 [B,N,H,d],
    lse fp32 [B,H,N]."""
    import torch
    B, N, three, H, d = qkv.shape
    _require(qkv, "qkv", torch.bfloat16, (B, N, 3, H, d))
    _require(o, "o", torch.bfloat16, (B, N, H, d))
    _require(lse, "lse", torch.float32, (B, H, N))
    _check(load_library().avion_attn_fwd_qkvpacked(_ptr(qkv), _ptr(o), _ptr(lse), B, H, N, d, float(scale),
                                                   _stream_handle(stream)))


def attn_bwd_qkvpacked(qkv, o, lse, dO, dqkv, scale: float, workspace, stream=None) -> None:
    """avion_attn_bwd_qkvpacked: gradients of the packed tensor, in the same packing."""
    import torch
    B, N, three, H, d = qkv.shape
    for t, n in ((qkv, "qkv"), (dqkv, "dqkv")):
        _require(t, n, torch.bfloat16, (B, N, 3, H, d))
    for t, n in ((o, "o"), (dO, "dO")):
        _require(t, n, torch.bfloat16, (B, N, H, d))
    _require(lse, "lse", torch.float32, (B, H, N))
    _require(workspace, "workspace", torch.uint8)
    _check(load_library().avion_attn_bwd_qkvpacked(_ptr(qkv), _ptr(o), _ptr(lse), _ptr(dO), _ptr(dqkv), B, H, N, d,
                                                   float(scale), _ptr(workspace), workspace.numel(),
                                                   _stream_handle(stream)))


def _flags(dtype, causal: bool, packed: bool) -> int:
    import torch
    if dtype not in (torch.bfloat16, torch.float16):
        raise ValueError(f"tensors must be bf16 or fp16, got {dtype}")
    return (FLAG_F16 if dtype == torch.float16 else 0) | (FLAG_CAUSAL if causal else 0) | (FLAG_QKVPACKED if packed else 0)


def attn_fwd_ex(q, k, v, o, lse, scale: float, causal: bool = False, stream=None) -> None:
    """avion_attn_fwd_ex: any combination of format (bf16 / fp16, taken from q.dtype), masking (`causal`)
    and packing (k is None and v is None: q is the packed [B,N,3,H,d] tensor)."""
    import torch
    packed = k is None and v is None
    dt = q.dtype
    if packed:
        B, N, three, H, d = q.shape
        _require(q, "qkv", dt, (B, N, 3, H, d))
    else:
        B, N, H, d = q.shape
        for t, n in ((q, "q"), (k, "k"), (v, "v")):
            _require(t, n, dt, (B, N, H, d))
    _require(o, "o", dt, (B, N, H, d))
    _require(lse, "lse", torch.float32, (B, H, N))
    none = ctypes.c_void_p(None)
    _check(load_library().avion_attn_fwd_ex(_ptr(q), none if packed else _ptr(k), none if packed else _ptr(v), _ptr(o),
                                            _ptr(lse), B, H, N, d, float(scale), _flags(dt, causal, packed),
                                            _stream_handle(stream)))


def attn_bwd_ex(q, k, v, o, lse, dO, dq, dk, dv, scale: float, workspace, causal: bool = False, stream=None) -> None:
    """avion_attn_bwd_ex: the gradients for avion_attn_fwd_ex with the same format, masking and packing
    (packed: k, v, dk, dv are None, q and dq are the packed tensors)."""
    import torch
    packed = k is None and v is None
    dt = q.dtype
    if packed:
        B, N, three, H, d = q.shape
        for t, n in ((q, "qkv"), (dq, "dqkv")):
            _require(t, n, dt, (B, N, 3, H, d))
        if dk is not None or dv is not None:
            raise ValueError("packed call: dk and dv must be None (dq receives the packed gradient)")
    else:
        B, N, H, d = q.shape
        for t, n in ((q, "q"), (k, "k"), (v, "v"), (dq, "dq"), (dk, "dk"), (dv, "dv")):
            _require(t, n, dt, (B, N, H, d))
    for t, n in ((o, "o"), (dO, "dO")):
        _require(t, n, dt, (B, N, H, d))
    _require(lse, "lse", torch.float32, (B, H, N))
    _require(workspace, "workspace", torch.uint8)
    none = ctypes.c_void_p(None)
    opt = lambda t: none if t is None else _ptr(t)
    _check(load_library().avion_attn_bwd_ex(_ptr(q), opt(k), opt(v), _ptr(o), _ptr(lse), _ptr(dO), _ptr(dq), opt(dk),
                                            opt(dv), B, H, N, d, float(scale), _flags(dt, causal, packed),
                                            _ptr(workspace), workspace.numel(), _stream_handle(stream)))


def layernorm_bwd_workspace_bytes(M: int, D: int) -> int:
    return int(load_library().avion_layernorm_bwd_workspace_bytes(M, D))


def layernorm_fwd(x, gamma, beta, y, mean, rstd, eps: float, stream=None) -> None:
    """avion_layernorm_fwd: x, y bf16 or fp16 [M, D]; gamma, beta fp32 [D]; mean, rstd fp32 [M] (saved for the backward)."""
    import torch
    M, D = x.shape
    _require(x, "x", x.dtype, (M, D))
    _require(y, "y", x.dtype, (M, D))
    for t, n in ((gamma, "gamma"), (beta, "beta")):
        _require(t, n, torch.float32, (D,))
    for t, n in ((mean, "mean"), (rstd, "rstd")):
        _require(t, n, torch.float32, (M,))
    _check(load_library().avion_layernorm_fwd(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(mean), _ptr(rstd), M, D,
                                              float(eps), _flags(x.dtype, False, False), _stream_handle(stream)))


def layernorm_bwd(x, gamma, mean, rstd, dy, dx, dgamma, dbeta, workspace, stream=None) -> None:
    """avion_layernorm_bwd: dx [M, D] in the format of x; dgamma, dbeta fp32 [D]."""
    import torch
    M, D = x.shape
    for t, n in ((x, "x"), (dy, "dy"), (dx, "dx")):
        _require(t, n, x.dtype, (M, D))
    for t, n in ((gamma, "gamma"), (dgamma, "dgamma"), (dbeta, "dbeta")):
        _require(t, n, torch.float32, (D,))
    for t, n in ((mean, "mean"), (rstd, "rstd")):
        _require(t, n, torch.float32, (M,))
    _require(workspace, "workspace", torch.uint8)
    _check(load_library().avion_layernorm_bwd(_ptr(x), _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(dy), _ptr(dx), _ptr(dgamma),
                                              _ptr(dbeta), M, D, _flags(x.dtype, False, False), _ptr(workspace),
                                              workspace.numel(), _stream_handle(stream)))


def bias_gelu_bwd_workspace_bytes(M: int, F: int) -> int:
    return int(load_library().avion_bias_gelu_bwd_workspace_bytes(M, F))


def bias_gelu_fwd(x, bias, y, stream=None) -> None:
    """avion_bias_gelu_fwd: x, y bf16 or fp16 [M, F]; bias fp32 [F]."""
    import torch
    M, F = x.shape
    _require(x, "x", x.dtype, (M, F))
    _require(y, "y", x.dtype, (M, F))
    _require(bias, "bias", torch.float32, (F,))
    _check(load_library().avion_bias_gelu_fwd(_ptr(x), _ptr(bias), _ptr(y), M, F, _flags(x.dtype, False, False),
                                              _stream_handle(stream)))


def bias_gelu_bwd(x, bias, dy, dx, dbias, workspace, stream=None) -> None:
    """avion_bias_gelu_bwd: dx [M, F] in the format of x; dbias fp32 [F]."""
    import torch
    M, F = x.shape
    for t, n in ((x, "x"), (dy, "dy"), (dx, "dx")):
        _require(t, n, x.dtype, (M, F))
    for t, n in ((bias, "bias"), (dbias, "dbias")):
        _require(t, n, torch.float32, (F,))
    _require(workspace, "workspace", torch.uint8)
    _check(load_library().avion_bias_gelu_bwd(_ptr(x), _ptr(bias), _ptr(dy), _ptr(dx), _ptr(dbias), M, F,
                                              _flags(x.dtype, False, False), _ptr(workspace), workspace.numel(),
                                              _stream_handle(stream)))
