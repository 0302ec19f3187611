"""GPU parity of the general entry points (avion_attn_fwd_ex / avion_attn_bwd_ex): every combination of
element format (bf16, fp16), masking (none, causal) and packing ([B,N,H,d] x 3, or [B,N,3,H,d]) against
the fp64 oracle, and bit for bit against the specific entry points where those exist."""
import itertools

import numpy as np
import pytest

import synth_inputs as si
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu


def _upload(bits, f16):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch.float16 if f16 else torch.bfloat16)


def run_ex(w, x, f16, causal, packed):
    """fwd + bwd through the general entry points; x holds bit patterns of the chosen format."""
    import torch
    import paper_2309_16669_amd as av
    dO = _upload(x["dO"], f16)
    o = torch.full_like(dO, float("nan"))
    lse = torch.full((w.B, w.H, w.N), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(av.attn_bwd_workspace_bytes(w.B, w.H, w.N, w.d), dtype=torch.uint8, device="cuda")
    if packed:
        qkv = _upload(np.stack([x["q"], x["k"], x["v"]], axis=2), f16)
        dqkv = torch.full_like(qkv, float("nan"))
        av.attn_fwd_ex(qkv, None, None, o, lse, w.scale, causal)
        av.attn_bwd_ex(qkv, None, None, o, lse, dO, dqkv, None, None, w.scale, ws, causal)
        torch.cuda.synchronize()
        return dict(o=o, lse=lse, dq=dqkv[:, :, 0], dk=dqkv[:, :, 1], dv=dqkv[:, :, 2])
    q, k, v = (_upload(x[n], f16) for n in ("q", "k", "v"))
    dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
    av.attn_fwd_ex(q, k, v, o, lse, w.scale, causal)
    av.attn_bwd_ex(q, k, v, o, lse, dO, dq, dk, dv, w.scale, ws, causal)
    torch.cuda.synchronize()
    return dict(o=o, lse=lse, dq=dq, dk=dk, dv=dv)


def check(w, x, out, f16, causal):
    """Against the oracle on the exactly widened inputs.  Bounds: those of the format (fp16: eight
    times tighter than bf16); the absolute bound follows one unit in the last place of the largest
    reference value where that exceeds it (causal rows over few keys carry weights near one)."""
    import oracle
    widen = si.f16_bits_to_f64 if f16 else si.bf16_bits_to_f64
    q, k, v, dO = (widen(x[n]) for n in ("q", "k", "v", "dO"))
    ro, rl = oracle.fwd_f64(q, k, v, w.scale, causal=causal)
    refs = oracle.bwd_f64(q, k, v, dO, w.scale, causal=causal)
    max_abs_tol, rel_tol, ulp = (gh.MAX_ABS_F16, gh.REL_FRO_F16, 2.0 ** -10) if f16 else (gh.MAX_ABS, gh.REL_FRO, 2.0 ** -7)
    # fewer than 16 keys: the gradients' relative bound of tests/test_tolerance_model.py (an eighth of it in fp16)
    grad_tol = rel_tol if w.N >= 16 else (gh.REL_FRO_TINY_N / 8 if f16 else gh.REL_FRO_TINY_N)
    assert float(np.abs(out["lse"].double().cpu().numpy() - rl).max()) <= gh.LSE_ABS
    for name, key, ref in (("O", "o", ro), ("dQ", "dq", refs[0]), ("dK", "dk", refs[1]), ("dV", "dv", refs[2])):
        got = out[key].contiguous().double().cpu().numpy()
        assert np.all(np.isfinite(got)), name
        max_abs, rel = gh.errors(got, ref)
        assert max_abs <= max(max_abs_tol, float(np.abs(ref).max()) * ulp), (name, max_abs)
        assert rel <= (rel_tol if name == "O" else grad_tol), (name, rel)


# the last three run as windows of several problems per wavefront (N <= 32), with a ragged last window
SHAPES = [(2, 3, 197, 64), (3, 8, 77, 64), (1, 2, 300, 80), (1, 2, 785, 64), (7, 3, 12, 64), (5, 2, 5, 80), (9, 2, 32, 64)]


@pytest.mark.parametrize("f16,causal,packed", [c for c in itertools.product((False, True), repeat=3)])
@pytest.mark.parametrize("B,H,N,d", SHAPES)
def test_every_combination_matches_the_oracle(B, H, N, d, f16, causal, packed):
    w = si.small_workload(B, H, N, d, seed=9000 + N + d)
    x = si.make_inputs(w, fmt="f16" if f16 else "bf16")
    check(w, x, run_ex(w, x, f16, causal, packed), f16, causal)


def _same_bits(a, b):
    import torch
    for n in ("o", "dq", "dk", "dv"):
        assert torch.equal(a[n].contiguous().view(torch.int16), b[n].contiguous().view(torch.int16)), n
    assert torch.equal(a["lse"], b["lse"])


@pytest.mark.parametrize("B,H,N,d", [(2, 3, 197, 64), (1, 2, 300, 80), (2, 2, 100, 64)])
def test_general_entry_points_give_the_bits_of_the_specific_ones(B, H, N, d):
    w = si.small_workload(B, H, N, d, seed=9100 + N)
    x = si.make_inputs(w)
    _same_bits(run_ex(w, x, False, False, False), gh.run_hip(w, x))
    _same_bits(run_ex(w, x, False, True, False), gh.run_hip(w, x, causal=True))
    _same_bits(run_ex(w, x, False, False, True), gh.run_hip_packed(w, x))
    x16 = si.make_inputs(w, fmt="f16")
    _same_bits(run_ex(w, x16, True, False, False), gh.run_hip_f16(w, x16))
    # packing never changes the bits, whatever the format and the mask
    _same_bits(run_ex(w, x16, True, True, True), run_ex(w, x16, True, True, False))
    _same_bits(run_ex(w, x, False, True, True), run_ex(w, x, False, True, False))


def test_general_entry_points_reject_unknown_flags_and_mixed_packing():
    import ctypes
    import paper_2309_16669_amd as av
    lib = av.load_library()
    fake, null, f = ctypes.c_void_p(0x1000), ctypes.c_void_p(None), ctypes.c_float(0.125)
    assert lib.avion_attn_fwd_ex(fake, fake, fake, fake, fake, 1, 2, 64, 64, f, 8, None) == av.EINVAL
    assert lib.avion_attn_fwd_ex(fake, fake, null, fake, fake, 1, 2, 64, 64, f, av.FLAG_QKVPACKED, None) == av.EINVAL
    assert lib.avion_attn_bwd_ex(fake, null, null, fake, fake, fake, fake, fake, null, 1, 2, 64, 64, f,
                                 av.FLAG_QKVPACKED, fake, 1 << 20, None) == av.EINVAL
    assert lib.avion_attn_bwd_ex(fake, fake, fake, fake, fake, fake, fake, fake, fake, 1, 2, 64, 64, f, 16,
                                 fake, 1 << 20, None) == av.EINVAL


def test_autograd_front_end_covers_the_combinations():
    # loss = sum(O * W): fp16 + causal, and packed + causal, through torch.autograd
    import torch
    import oracle
    from paper_2309_16669_amd import autograd as ag
    w = si.small_workload(2, 3, 150, 64, seed=9200)
    x16 = si.make_inputs(w, fmt="f16")
    q, k, v = (_upload(x16[n], True).requires_grad_() for n in ("q", "k", "v"))
    dO = _upload(x16["dO"], True)
    o = ag.attention(q, k, v, w.scale, causal=True)
    (o.float() * dO.float()).sum().backward()
    check(w, x16, dict(o=o.detach(), lse=_lse_of(w, x16, True, True), dq=q.grad, dk=k.grad, dv=v.grad), True, True)
    x = si.make_inputs(w)
    qkv = _upload(np.stack([x["q"], x["k"], x["v"]], axis=2), False).requires_grad_()
    o = ag.attention_qkvpacked(qkv, w.scale, causal=True)
    (o.float() * _upload(x["dO"], False).float()).sum().backward()
    check(w, x, dict(o=o.detach(), lse=_lse_of(w, x, False, True), dq=qkv.grad[:, :, 0], dk=qkv.grad[:, :, 1],
                     dv=qkv.grad[:, :, 2]), False, True)
    # the workspace of the backward is kept per (device, stream): a second backward allocates none
    before = dict(ag._workspaces)
    q2, k2, v2 = (_upload(x[n], False).requires_grad_() for n in ("q", "k", "v"))
    ag.attention(q2, k2, v2, w.scale).float().sum().backward()
    assert {k_: v_.data_ptr() for k_, v_ in ag._workspaces.items()} == {k_: v_.data_ptr() for k_, v_ in before.items()}


def _lse_of(w, x, f16, causal):
    """LSE of the forward (the autograd front end keeps it to itself), recomputed through the binding."""
    import torch
    import paper_2309_16669_amd as av
    q, k, v = (_upload(x[n], f16) for n in ("q", "k", "v"))
    o = torch.empty_like(q)
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    av.attn_fwd_ex(q, k, v, o, lse, w.scale, causal)
    torch.cuda.synchronize()
    return lse
