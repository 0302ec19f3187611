"""ctypes front end of the CPU oracle (`avion_oracle.c`).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
It shares nothing with the HIP path and never imports it.  Inputs are numpy arrays in the
`[B, N, H, d]` layout: uint16 bf16 bit patterns (`fwd`, `bwd`) or float64 (`fwd_f64`, `bwd_f64`);
all results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "avion_oracle.c")
_LIB = os.path.join(_HERE, "libavion_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, OpenMP threads over query rows). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        p = ctypes.c_void_p
        i = ctypes.c_int
        f = ctypes.c_double
        lib.avion_oracle_max_threads.restype = i
        lib.avion_oracle_fwd_f64.argtypes = [p, p, p, p, p, p, i, i, i, i, f, i]
        lib.avion_oracle_bwd_f64.argtypes = [p, p, p, p, p, p, p, i, i, i, i, f, i]
        lib.avion_oracle_fwd.argtypes = [p, p, p, p, p, i, i, i, i, f, i]
        lib.avion_oracle_bwd.argtypes = [p, p, p, p, p, p, p, i, i, i, i, f, i]
        lib.avion_oracle_fwd_causal_f64.argtypes = lib.avion_oracle_fwd_f64.argtypes
        lib.avion_oracle_bwd_causal_f64.argtypes = lib.avion_oracle_bwd_f64.argtypes
        lib.avion_oracle_fwd_causal.argtypes = lib.avion_oracle_fwd.argtypes
        lib.avion_oracle_bwd_causal.argtypes = lib.avion_oracle_bwd.argtypes
        for fn in (lib.avion_oracle_fwd_f64, lib.avion_oracle_bwd_f64, lib.avion_oracle_fwd,
                   lib.avion_oracle_bwd, lib.avion_oracle_fwd_causal_f64, lib.avion_oracle_bwd_causal_f64,
                   lib.avion_oracle_fwd_causal, lib.avion_oracle_bwd_causal):
            fn.restype = i
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().avion_oracle_max_threads())


def _chk(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"{what} failed with oracle error {rc}")


def _shape(x):
    if x.ndim != 4:
        raise ValueError("expected a [B, N, H, d] array")
    B, N, H, d = x.shape
    return B, N, H, d


def _c(x, dtype):
    return np.ascontiguousarray(x, dtype=dtype)


def fwd_f64(q, k, v, scale, want_weights=False, nthreads=0, causal=False):
    """Forward on float64 inputs. Returns (O [B,N,H,d], LSE [B,H,N]) and, if asked, P [B,H,N,N].
    causal=True: query i attends to keys 0..i only."""
    q, k, v = _c(q, np.float64), _c(k, np.float64), _c(v, np.float64)
    B, N, H, d = _shape(q)
    assert k.shape == q.shape and v.shape == q.shape
    o = np.empty((B, N, H, d), np.float64)
    lse = np.empty((B, H, N), np.float64)
    w = np.empty((B, H, N, N), np.float64) if want_weights else None
    fn = _load().avion_oracle_fwd_causal_f64 if causal else _load().avion_oracle_fwd_f64
    _chk(fn(q.ctypes.data, k.ctypes.data, v.ctypes.data, o.ctypes.data,
            lse.ctypes.data, w.ctypes.data if want_weights else None,
            B, H, N, d, float(scale), int(nthreads)), "oracle fwd")
    return (o, lse, w) if want_weights else (o, lse)


def bwd_f64(q, k, v, dO, scale, nthreads=0, causal=False):
    """Backward on float64 inputs. Returns (dQ, dK, dV), each [B,N,H,d] float64."""
    q, k, v, dO = (_c(x, np.float64) for x in (q, k, v, dO))
    B, N, H, d = _shape(q)
    assert k.shape == q.shape and v.shape == q.shape and dO.shape == q.shape
    dq, dk, dv = (np.empty((B, N, H, d), np.float64) for _ in range(3))
    fn = _load().avion_oracle_bwd_causal_f64 if causal else _load().avion_oracle_bwd_f64
    _chk(fn(q.ctypes.data, k.ctypes.data, v.ctypes.data, dO.ctypes.data, dq.ctypes.data, dk.ctypes.data, dv.ctypes.data,
            B, H, N, d, float(scale), int(nthreads)), "oracle bwd")
    return dq, dk, dv


def fwd(q_bits, k_bits, v_bits, scale, nthreads=0, causal=False):
    """Forward on bf16 bit patterns (uint16). Returns (O, LSE) in float64."""
    q, k, v = (_c(x, np.uint16) for x in (q_bits, k_bits, v_bits))
    B, N, H, d = _shape(q)
    assert k.shape == q.shape and v.shape == q.shape
    o = np.empty((B, N, H, d), np.float64)
    lse = np.empty((B, H, N), np.float64)
    fn = _load().avion_oracle_fwd_causal if causal else _load().avion_oracle_fwd
    _chk(fn(q.ctypes.data, k.ctypes.data, v.ctypes.data, o.ctypes.data, lse.ctypes.data, B, H, N, d, float(scale),
            int(nthreads)), "oracle fwd")
    return o, lse


def bwd(q_bits, k_bits, v_bits, dO_bits, scale, nthreads=0, causal=False):
    """Backward on bf16 bit patterns (uint16). Returns (dQ, dK, dV) in float64."""
    q, k, v, dO = (_c(x, np.uint16) for x in (q_bits, k_bits, v_bits, dO_bits))
    B, N, H, d = _shape(q)
    assert k.shape == q.shape and v.shape == q.shape and dO.shape == q.shape
    dq, dk, dv = (np.empty((B, N, H, d), np.float64) for _ in range(3))
    fn = _load().avion_oracle_bwd_causal if causal else _load().avion_oracle_bwd
    _chk(fn(q.ctypes.data, k.ctypes.data, v.ctypes.data, dO.ctypes.data, dq.ctypes.data, dk.ctypes.data, dv.ctypes.data,
            B, H, N, d, float(scale), int(nthreads)), "oracle bwd")
    return dq, dk, dv
