"""The C-ABI library: it loads, exports every symbol the header declares, and rejects bad
arguments before touching the GPU (these paths run on a machine without one)."""
import ctypes
import os
import re

import pytest

import paper_2309_16669_amd as av

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(avion_\w+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = av.load_library()
    names = declared_symbols()
    assert {"avion_attn_fwd", "avion_attn_bwd", "avion_attn_bwd_workspace_bytes", "avion_strerror",
            "avion_version", "avion_last_hip_error", "avion_attn_fwd_qkvpacked",
            "avion_attn_bwd_qkvpacked"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert av.version() >= 100


def test_error_texts():
    for code in (av.OK, av.EINVAL, av.EUNSUPPORTED, av.EWORKSPACE, av.EHIP, -99):
        assert isinstance(av.strerror(code), str) and av.strerror(code)


def test_workspace_is_linear_in_n():
    a = av.attn_bwd_workspace_bytes(2, 3, 1000, 64)
    b = av.attn_bwd_workspace_bytes(2, 3, 2000, 64)
    assert a % 256 == 0 and a >= 2 * 3 * 1000 * 4
    assert b <= 2 * a + 256            # O(N), never O(N^2)
    assert av.attn_bwd_workspace_bytes(2, 3, 1000, 48) == 0
    assert av.attn_bwd_workspace_bytes(0, 3, 1000, 64) == 0


FAKE = 0x1000   # a 16-byte aligned non-null "pointer"; never dereferenced on these paths


@pytest.mark.parametrize("kwargs,code", [
    (dict(q=0), av.EINVAL),
    (dict(lse=0), av.EINVAL),
    (dict(B=0), av.EINVAL),
    (dict(N=-3), av.EINVAL),
    (dict(scale=0.0), av.EINVAL),
    (dict(scale=float("nan")), av.EINVAL),
    (dict(scale=float("inf")), av.EINVAL),
    (dict(d=48), av.EUNSUPPORTED),
    (dict(d=128), av.EUNSUPPORTED),
    (dict(k=FAKE + 2), av.EUNSUPPORTED),
    (dict(N=(1 << 24) + 1), av.EUNSUPPORTED),
])
def test_fwd_rejects_bad_arguments_without_launching(kwargs, code):
    lib = av.load_library()
    a = dict(q=FAKE, k=FAKE, v=FAKE, o=FAKE, lse=FAKE, B=1, H=2, N=64, d=64, scale=0.125, stream=None)
    a.update(kwargs)
    rc = lib.avion_attn_fwd(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["H"], a["N"], a["d"],
                            ctypes.c_float(a["scale"]), a["stream"])
    assert rc == code


@pytest.mark.parametrize("kwargs,code", [
    (dict(dO=0), av.EINVAL),
    (dict(dv=0), av.EINVAL),
    (dict(H=0), av.EINVAL),
    (dict(d=96), av.EUNSUPPORTED),
    (dict(dq=FAKE + 8), av.EUNSUPPORTED),
    (dict(ws=0), av.EWORKSPACE),
    (dict(ws=FAKE + 16), av.EWORKSPACE),       # not 256-byte aligned
    (dict(ws_bytes=100), av.EWORKSPACE),
])
def test_bwd_rejects_bad_arguments_without_launching(kwargs, code):
    lib = av.load_library()
    a = dict(q=FAKE, k=FAKE, v=FAKE, o=FAKE, lse=FAKE, dO=FAKE, dq=FAKE, dk=FAKE, dv=FAKE,
             B=1, H=2, N=64, d=64, scale=0.125, ws=FAKE, ws_bytes=1 << 20)
    a.update(kwargs)
    rc = lib.avion_attn_bwd(a["q"], a["k"], a["v"], a["o"], a["lse"], a["dO"], a["dq"], a["dk"], a["dv"],
                            a["B"], a["H"], a["N"], a["d"], ctypes.c_float(a["scale"]),
                            a["ws"], a["ws_bytes"], None)
    assert rc == code


@pytest.mark.parametrize("kwargs,code", [
    (dict(qkv=0), av.EINVAL),
    (dict(dqkv=0), av.EINVAL),
    (dict(H=0), av.EINVAL),
    (dict(d=96), av.EUNSUPPORTED),
    (dict(qkv=FAKE + 8), av.EUNSUPPORTED),
    (dict(ws_bytes=100), av.EWORKSPACE),
    # a (batch, head) slice of the packed tensor must stay below 2^31 bytes: 3*H*d*2 bytes per token
    (dict(H=64, N=100000), av.EUNSUPPORTED),
])
def test_packed_entry_points_reject_bad_arguments_without_launching(kwargs, code):
    lib = av.load_library()
    a = dict(qkv=FAKE, o=FAKE, lse=FAKE, dO=FAKE, dqkv=FAKE, B=1, H=2, N=64, d=64, scale=0.125, ws=FAKE,
             ws_bytes=1 << 30)
    a.update(kwargs)
    rc = lib.avion_attn_bwd_qkvpacked(a["qkv"], a["o"], a["lse"], a["dO"], a["dqkv"], a["B"], a["H"], a["N"], a["d"],
                                      ctypes.c_float(a["scale"]), a["ws"], a["ws_bytes"], None)
    assert rc == code
    if "dqkv" not in kwargs and "ws_bytes" not in kwargs:
        rc = lib.avion_attn_fwd_qkvpacked(a["qkv"], a["o"], a["lse"], a["B"], a["H"], a["N"], a["d"],
                                          ctypes.c_float(a["scale"]), None)
        assert rc == code


@pytest.mark.parametrize("suffix", ["", "_f16", "_causal"])
def test_every_variant_checks_its_arguments(suffix):
    # the fp16 and causal entry points share the checks of the bf16 ones
    lib = av.load_library()
    fwd, bwd = getattr(lib, "avion_attn_fwd" + suffix), getattr(lib, "avion_attn_bwd" + suffix)
    c = ctypes.c_float
    assert fwd(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 2, 64, 48, c(0.1), None) == av.EUNSUPPORTED
    assert fwd(FAKE, 0, FAKE, FAKE, FAKE, 1, 2, 64, 64, c(0.1), None) == av.EINVAL
    assert fwd(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 2, 0, 64, c(0.1), None) == av.EINVAL
    assert fwd(FAKE, FAKE, FAKE, FAKE + 4, FAKE, 1, 2, 64, 64, c(0.1), None) == av.EUNSUPPORTED
    assert bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 2, 64, 80, c(-1.0), FAKE, 1 << 20, None) == av.EINVAL
    assert bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 2, 64, 80, c(0.1), FAKE, 8, None) == av.EWORKSPACE
    assert bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0, 1, 2, 64, 80, c(0.1), FAKE, 1 << 20, None) == av.EINVAL
    # short sequences take the one-launch path: same checks before anything is launched
    assert bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 2, 16, 64, c(0.1), FAKE + 64, 1 << 20, None) == av.EWORKSPACE


def test_binding_does_not_import_the_oracle():
    import sys
    src = open(os.path.join(ROOT, "paper_2309_16669_amd", "__init__.py")).read()
    assert "oracle" not in src.replace("no CPU or PyTorch fallback", "")
    for fn in os.listdir(os.path.join(ROOT, "paper_2309_16669_amd", "csrc")):
        assert "oracle" not in open(os.path.join(ROOT, "paper_2309_16669_amd", "csrc", fn)).read()
