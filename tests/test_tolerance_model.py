"""Where the two relaxed bounds of the GPU parity tests come from (tests/gpu_harness.py):

  REL_FRO_TINY_N   relative Frobenius bound for gradients when N < 16 (2e-2 instead of 5e-3)
  one-ulp rule     absolute bound = one bf16 unit in the last place (2^-7) of the largest reference
                   value, once that exceeds the stated 2e-2 (near one-hot rows: peaky and causal cases)
  PEAKY_DQ_ABS     the same rule with the largest dQ element of the whole workload, for dQ of the
                   named workload with the peaky softmax (tests/test_parity_gpu.py)

Both follow from the rounding points of the method, not from any kernel: P and dS are rounded to bf16
before they enter a contraction, O is divided by the sum of the rounded weights and rounded to bf16,
delta is built from that rounded O, and the outputs are rounded once.  This file carries out exactly
that arithmetic in fp64 with explicit bf16 roundings (every accumulation exact) and measures it against
the oracle: the stated bounds hold for it, and the strict ones do not.  Runs on the CPU.
"""
import numpy as np
import pytest

import oracle
import synth_inputs as si


def rb(x):
    """round to bf16 (nearest even), as fp64 values"""
    return si.bf16_bits_to_f64(si.f32_to_bf16_bits(np.asarray(x, dtype=np.float64).astype(np.float32)))


def rounded_arithmetic(w, x, causal=False):
    """O, dQ, dK, dV of one workload computed with the method's rounding points and nothing else."""
    q, k, v, dO = (si.bf16_bits_to_f64(x[n]) for n in ("q", "k", "v", "dO"))
    s = np.einsum("bnhc,bmhc->bhnm", q, k) * w.scale
    if causal:
        s = np.where(np.tril(np.ones((w.N, w.N), dtype=bool)), s, -np.inf)
    m = s.max(-1, keepdims=True)
    e = np.exp(s - m)
    lse = m + np.log(e.sum(-1, keepdims=True))
    e_r = rb(e)                                                  # weights as the second contraction sees them
    o = rb(np.einsum("bhnm,bmhc->bnhc", e_r, v) / e_r.sum(-1).transpose(0, 2, 1)[..., None])
    p = np.exp(s - lse)
    delta = np.einsum("bnhc,bnhc->bhn", dO, o)                   # from the rounded O
    dP = np.einsum("bnhc,bmhc->bhnm", dO, v)
    dS = rb(p * (dP - delta[..., None]))
    dq = rb(w.scale * np.einsum("bhnm,bmhc->bnhc", dS, k))
    dk = rb(w.scale * np.einsum("bhnm,bnhc->bmhc", dS, q))
    dv = rb(np.einsum("bhnm,bnhc->bmhc", rb(p), dO))
    return dict(O=o, dQ=dq, dK=dk, dV=dv)


def errors_against_oracle(w, causal=False):
    x = si.make_inputs(w)
    got = rounded_arithmetic(w, x, causal)
    ro, _ = oracle.fwd(x["q"], x["k"], x["v"], w.scale, causal=causal)
    rdq, rdk, rdv = oracle.bwd(x["q"], x["k"], x["v"], x["dO"], w.scale, causal=causal)
    out = {}
    for name, ref in (("O", ro), ("dQ", rdq), ("dK", rdk), ("dV", rdv)):
        diff = got[name] - ref
        den = np.sqrt((ref ** 2).sum())
        out[name] = (float(np.abs(diff).max()), float(np.sqrt((diff ** 2).sum()) / den) if den > 0 else 0.0,
                     float(np.abs(ref).max()))
    return out


def test_below_16_keys_the_method_itself_exceeds_the_strict_relative_bound_and_meets_the_relaxed_one():
    from tests.gpu_harness import REL_FRO, REL_FRO_TINY_N
    worst = 0.0
    for N in (2, 3, 4, 5, 8, 12, 15):
        for seed in range(12):
            for name, (_, rel, _) in errors_against_oracle(si.small_workload(2, 2, N, 64, seed=100 * N + seed)).items():
                if name != "O":
                    worst = max(worst, rel)
                    assert rel <= REL_FRO_TINY_N, (N, seed, name, rel)
    assert worst > REL_FRO          # the strict bound is not one this arithmetic can meet at these sizes


@pytest.mark.parametrize("N", [16, 33, 64, 150])
def test_from_16_keys_on_the_method_meets_the_strict_relative_bound(N):
    from tests.gpu_harness import REL_FRO
    for seed in range(4):
        for name, (_, rel, _) in errors_against_oracle(si.small_workload(2, 2, N, 64, seed=7 * N + seed)).items():
            assert rel <= REL_FRO, (N, seed, name, rel)


# the stress cases of the GPU suite that use the one-ulp rule: peaky softmax, and causal rows
ONE_ULP_CASES = [
    (dict(B=2, H=4, N=333, d=64, seed=4242, scale=0.125, k_mul=2.0), False),
    (dict(B=1, H=2, N=200, d=80, seed=4243, k_mul=4.0), False),
    (dict(B=3, H=8, N=77, d=64, seed=7700 + 5 * 77 + 64), True),
    (dict(B=2, H=2, N=300, d=64, seed=7700 + 5 * 300 + 64), True),
]


def test_near_one_hot_rows_need_and_meet_the_one_ulp_absolute_bound():
    from tests.gpu_harness import MAX_ABS, REL_FRO
    exceeded_strict = False
    for kw, causal in ONE_ULP_CASES:
        w = si.small_workload(**kw)
        for name, (max_abs, rel, ref_max) in errors_against_oracle(w, causal).items():
            assert max_abs <= max(MAX_ABS, ref_max * 2.0 ** -7), (kw, name, max_abs, ref_max)
            assert rel <= REL_FRO, (kw, name, rel)
            exceeded_strict |= max_abs > MAX_ABS
    assert exceeded_strict          # at least one of these cases cannot meet 2e-2 by the method's arithmetic


def test_named_workload_shape_meets_the_strict_bounds_in_this_arithmetic():
    # one head of the ViT-B shape (N = 1568): the strict bounds are the right ones for the named workloads
    from tests.gpu_harness import MAX_ABS, REL_FRO
    w = si.small_workload(1, 1, 1568, 64, seed=230916691, scale=0.125)
    for name, (max_abs, rel, _) in errors_against_oracle(w).items():
        assert max_abs <= MAX_ABS and rel <= REL_FRO, (name, max_abs, rel)


def test_peaky_named_workload_dq_exceeds_the_absolute_bound_through_delta_alone():
    # ViT-L batch with K doubled, head (8, 4): everything exact in fp64 -- weights, dS, contractions,
    # unrounded dQ -- except that delta = rowsum(dO o O) is built from O rounded to bf16, which is all
    # the backward's interface hands over.  That alone moves one dQ element by 2.6e-2 (delta off by
    # 3.0e-2, times scale, times |sum_j P_ij k_j| = 6.9): no kernel behind this interface can meet 2e-2
    # on this head, while the relative Frobenius error of the same tensor is far inside its bound.
    from tests.gpu_harness import MAX_ABS, REL_FRO
    w = si.WORKLOADS["vitl_batch_peaky"]
    b, h = 8, 4
    one_head = si.small_workload(1, 1, w.N, w.d, seed=0, scale=w.scale)
    x = {n: a[b:b + 1, :, h:h + 1] for n, a in si.make_inputs(w).items()}
    q, k, v, dO = (si.bf16_bits_to_f64(x[n])[0, :, 0, :] for n in ("q", "k", "v", "dO"))
    s = q @ k.T * one_head.scale
    p = np.exp(s - s.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    dP = dO @ v.T
    o = p @ v
    ref = one_head.scale * (p * (dP - (dO * o).sum(-1, keepdims=True))) @ k
    got = one_head.scale * (p * (dP - (dO * rb(o)).sum(-1, keepdims=True))) @ k
    rdq = oracle.bwd(x["q"], x["k"], x["v"], x["dO"], one_head.scale)[0][0, :, 0, :]
    assert np.abs(ref - rdq).max() < 1e-9                       # the plain formulas above are the oracle's
    err = np.abs(got - ref)
    assert err.max() > MAX_ABS
    assert np.sqrt((err ** 2).sum() / (ref ** 2).sum()) < REL_FRO / 4
    # the bound the GPU test takes for this tensor: one bf16 ulp of the workload's largest dQ element
    from tests.test_parity_gpu import PEAKY_DQ_ABS
    assert err.max() + np.abs(ref).max() * 2.0 ** -9 <= PEAKY_DQ_ABS    # delta's share plus the output rounding
