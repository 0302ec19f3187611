"""The allocation-free backward entry point (avion_attn_bwd_noalloc) against avion_attn_bwd: same
kernels, the library's built-in scratch in place of the caller's workspace, so the results must be
the same bits.  Two calls in a row share the scratch, the second on a smaller problem (stale
contents of the first call lie behind and around what the second one uses)."""
import ctypes

import numpy as np
import pytest

import synth_inputs as si
from tests import gpu_harness as gh

pytestmark = pytest.mark.gpu


def _both_ways(w):
    """Returns (gradients through avion_attn_bwd, gradients through the raw C entry point
    avion_attn_bwd_noalloc) on the same forward results."""
    import torch
    import paper_2309_16669_amd as av
    lib = av.load_library()
    x = si.make_inputs(w)
    q, k, v, dO = (gh.to_gpu_bf16(x[n]) for n in ("q", "k", "v", "dO"))
    o = torch.empty_like(q)
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    av.attn_fwd(q, k, v, o, lse, w.scale)
    ref = [torch.full_like(q, float("nan")) for _ in range(3)]
    ws = torch.empty(av.attn_bwd_workspace_bytes(w.B, w.H, w.N, w.d), dtype=torch.uint8, device="cuda")
    av.attn_bwd(q, k, v, o, lse, dO, *ref, w.scale, ws)
    got = [torch.full_like(q, float("nan")) for _ in range(3)]
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = lib.avion_attn_bwd_noalloc(p(q), p(k), p(v), p(o), p(lse), p(dO), p(got[0]), p(got[1]), p(got[2]),
                                    w.B, w.H, w.N, w.d, ctypes.c_float(w.scale),
                                    ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == av.OK, av.strerror(rc)
    torch.cuda.synchronize()
    return x, dict(o=o, lse=lse, dq=ref[0], dk=ref[1], dv=ref[2]), got


def test_noalloc_backward_equals_the_workspace_backward_on_two_calls_in_a_row():
    import torch
    # first a problem of several tiles with a ragged tail, then a smaller one (other N, other head
    # count) that reuses the front of the scratch the first call has filled
    for shape, seed in (((2, 3, 700, 64), 71), ((1, 2, 197, 64), 72)):
        w = si.small_workload(*shape, seed=seed)
        x, ref, got = _both_ways(w)
        for name, a, b in zip(("dq", "dk", "dv"), (ref["dq"], ref["dk"], ref["dv"]), got):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), (shape, name)
        # and the reference itself is right (oracle, stated tolerances)
        gh.check_against_oracle(w, x, ref)


def test_noalloc_backward_rejects_what_does_not_fit_its_scratch():
    import paper_2309_16669_amd as av
    lib = av.load_library()
    fake = ctypes.c_void_p(0x1000)
    # 2^22 rows of 8 bytes fill the 32 MiB scratch exactly; one 64-row block more does not fit
    B, H, N = 1, 4096, 1024
    assert av.attn_bwd_workspace_bytes(B, H, N, 64) == 32 << 20
    args = lambda h: (fake,) * 9 + (B, h, N, 64, ctypes.c_float(0.125), None)
    assert lib.avion_attn_bwd_noalloc(*args(H + 1)) == av.ESCRATCH
    assert "scratch" in av.strerror(av.ESCRATCH)
    # argument errors are reported as by avion_attn_bwd, before anything else
    assert lib.avion_attn_bwd_noalloc(*((None,) + (fake,) * 8 + (B, H, N, 64, ctypes.c_float(0.125), None))) == av.EINVAL
