"""GPU parity of the layer-normalisation kernels (through the C ABI) against the fp64 oracle
(oracle/layernorm.py) on the same seeded inputs.

Bounds (derived from the arithmetic: statistics and sums in fp32, outputs rounded once to the tensor
format, whose unit roundoff is u = 2^-9 for bf16 and 2^-12 for fp16):
  y, dx          relative Frobenius error <= 2.5 u  (the final rounding alone gives u / sqrt(3) per
                 element of its own size; measured 1.7e-3 for bf16, 2.1e-4 for fp16) and every element within
                 2 u max|ref| (one unit in the last place of the largest value)
  mean, rstd     relative error <= 1e-5 (fp32 sums over D <= 2048 channels)
  dgamma, dbeta  relative Frobenius error <= 1e-4 (fp32 sums over all rows, pairwise by construction:
                 per wavefront, per workgroup, then over the workgroups)
"""
import ctypes

import numpy as np
import pytest

import synth_inputs as si

pytestmark = pytest.mark.gpu


def _run(M, D, seed, fmt="bf16", eps=1e-5):
    import torch
    import paper_2309_16669_amd as av
    f16 = fmt == "f16"
    dt = torch.float16 if f16 else torch.bfloat16
    inp = si.layernorm_inputs(M, D, seed, fmt)
    up = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(dt)
    x, dy = up(inp["x"]), up(inp["dy"])
    gamma, beta = torch.from_numpy(inp["gamma"]).cuda(), torch.from_numpy(inp["beta"]).cuda()
    y = torch.full_like(x, float("nan"))
    dx = torch.full_like(x, float("nan"))
    mean = torch.full((M,), float("nan"), dtype=torch.float32, device="cuda")
    rstd = torch.full((M,), float("nan"), dtype=torch.float32, device="cuda")
    dgamma = torch.full((D,), float("nan"), dtype=torch.float32, device="cuda")
    dbeta = torch.full((D,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(av.layernorm_bwd_workspace_bytes(M, D), dtype=torch.uint8, device="cuda")
    av.layernorm_fwd(x, gamma, beta, y, mean, rstd, eps)
    av.layernorm_bwd(x, gamma, mean, rstd, dy, dx, dgamma, dbeta, ws)
    torch.cuda.synchronize()
    return inp, dict(y=y, dx=dx, mean=mean, rstd=rstd, dgamma=dgamma, dbeta=dbeta)


def _check(M, D, seed, fmt="bf16", eps=1e-5):
    from oracle import layernorm as ln
    inp, out = _run(M, D, seed, fmt, eps)
    widen = si.f16_bits_to_f64 if fmt == "f16" else si.bf16_bits_to_f64
    u = 2.0 ** -12 if fmt == "f16" else 2.0 ** -9
    x, dy = widen(inp["x"]), widen(inp["dy"])
    ry, rmean, rrstd = ln.fwd(x, inp["gamma"], inp["beta"], eps)
    rdx, rdg, rdb = ln.bwd(x, inp["gamma"], dy, eps)
    rep = {}
    for name, ref in (("y", ry), ("dx", rdx)):
        got = out[name].double().cpu().numpy()
        assert np.all(np.isfinite(got)), name
        err = np.abs(got - ref)
        rel = np.sqrt((err ** 2).sum() / max((ref ** 2).sum(), 1e-300))
        rep[name] = (float(err.max()), float(rel))
        assert err.max() <= 2 * u * max(np.abs(ref).max(), 1e-30) + 1e-30, (name, err.max())
        assert rel <= 2.5 * u, (name, rel)
    for name, ref in (("mean", rmean), ("rstd", rrstd)):
        got = out[name].double().cpu().numpy()
        assert np.abs(got - ref).max() <= 1e-5 * max(np.abs(ref).max(), 1.0), name
    for name, ref in (("dgamma", rdg), ("dbeta", rdb)):
        got = out[name].double().cpu().numpy()
        rel = np.sqrt(((got - ref) ** 2).sum() / max((ref ** 2).sum(), 1e-300))
        rep[name] = float(rel)
        assert rel <= 1e-4, (name, rel)
    return rep


# one and several chunks per lane, rows that do not fill a wavefront's chunks (D = 72, 200, 1288), the
# ViT widths (768, 1024, 1280), the largest supported width, row counts around the workgroup and grid sizes
SHAPES = [(1, 8), (3, 72), (5, 64), (33, 768), (130, 200), (1000, 1024), (257, 1280), (64, 2048), (4097, 768), (9, 1288)]


@pytest.mark.parametrize("M,D", SHAPES)
@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_shapes_match_the_oracle(M, D, fmt):
    rep = _check(M, D, seed=500 + M + D, fmt=fmt)
    print(f"\nlayernorm {fmt} M={M} D={D}: {rep}", flush=True)


def test_vitb_training_batch_every_element():
    # the tokens of the benchmark's attention workload: 32 clips x 1568 tokens, width 768 (12 heads of 64)
    rep = _check(32 * 1568, 768, seed=230916692)
    print(f"\nlayernorm vitb batch: {rep}", flush=True)


def test_large_eps_and_offset_rows():
    # eps comparable to the variance; rows with a large common offset (the mean must be removed before squaring)
    import torch
    import paper_2309_16669_amd as av
    from oracle import layernorm as ln
    M, D = 50, 256
    inp = si.layernorm_inputs(M, D, seed=77)
    x = si.bf16_bits_to_f32(inp["x"]) * np.float32(0.25) + np.float32(100.0)
    inp["x"] = si.f32_to_bf16_bits(x)
    xt = torch.from_numpy(inp["x"].view(np.int16)).cuda().view(torch.bfloat16)
    gamma, beta = torch.from_numpy(inp["gamma"]).cuda(), torch.from_numpy(inp["beta"]).cuda()
    y = torch.empty_like(xt)
    mean = torch.empty((M,), dtype=torch.float32, device="cuda")
    rstd = torch.empty((M,), dtype=torch.float32, device="cuda")
    av.layernorm_fwd(xt, gamma, beta, y, mean, rstd, 0.5)
    torch.cuda.synchronize()
    ry, rmean, rrstd = ln.fwd(si.bf16_bits_to_f64(inp["x"]), inp["gamma"], inp["beta"], 0.5)
    assert np.abs(mean.double().cpu().numpy() - rmean).max() <= 1e-5 * 100
    assert np.abs(rstd.double().cpu().numpy() - rrstd).max() <= 1e-5 * rrstd.max()
    assert np.abs(y.double().cpu().numpy() - ry).max() <= 2 * 2.0 ** -9 * np.abs(ry).max()


def test_bitwise_reproducible():
    import torch
    a = _run(3001, 768, seed=9)[1]
    b = _run(3001, 768, seed=9)[1]
    for n in a:
        assert torch.equal(a[n].view(torch.int16) if a[n].dtype != torch.float32 else a[n],
                           b[n].view(torch.int16) if b[n].dtype != torch.float32 else b[n]), n


def test_bad_arguments_are_rejected_without_launching():
    import paper_2309_16669_amd as av
    lib = av.load_library()
    fake, f = ctypes.c_void_p(0x1000), ctypes.c_float
    ok = dict(M=4, D=64, eps=1e-5, flags=0)

    def fwd(**kw):
        a = dict(ok, **kw)
        return lib.avion_layernorm_fwd(kw.get("x", fake), fake, fake, fake, fake, fake, a["M"], a["D"], f(a["eps"]), a["flags"], None)
    assert fwd(x=None) == av.EINVAL and fwd(M=0) == av.EINVAL and fwd(eps=-1.0) == av.EINVAL and fwd(flags=2) == av.EINVAL
    assert fwd(D=60) == av.EUNSUPPORTED and fwd(D=4096) == av.EUNSUPPORTED and fwd(x=ctypes.c_void_p(0x1004)) == av.EUNSUPPORTED
    assert av.layernorm_bwd_workspace_bytes(10, 60) == 0
    assert av.layernorm_bwd_workspace_bytes(10 ** 6, 768) == av.layernorm_bwd_workspace_bytes(10 ** 7, 768)   # independent of M
    assert lib.avion_layernorm_bwd(fake, fake, fake, fake, fake, fake, fake, fake, 4, 64, 0, fake, 16, None) == av.EWORKSPACE
