"""Pins for the CPU oracle: each ties it to something other than itself.

The operation is the one of Sec. 3 ("Flash Attention") of the paper: a weighted average of the
value features with weights from query-key dot products, computed exactly (Sec. 1).  The paper
prints no worked numerical example, so the pins are closed forms, invariants, finite differences,
a hand-derived tiny case (tests/golden/attn_n2_d1.txt) and a dense library computation.
A dropped term, a wrong sign or index, a missing `scale` or a transposed operand in the oracle
fails at least one of them.
"""
import math
import os

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(20230916)


def rand(B, N, H, d, s=1.0):
    return RNG.standard_normal((B, N, H, d)) * s


def dense_reference(q, k, v, scale):
    """softmax(QK^T*scale)V through dense einsum in numpy, for cross-checks of tiny cases."""
    s = np.einsum("bnhc,bmhc->bhnm", q, k) * scale
    m = s.max(-1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(-1, keepdims=True)
    p = e / l
    o = np.einsum("bhnm,bmhc->bnhc", p, v)
    return o, (m + np.log(l))[..., 0], p


# ---------------------------------------------------------------- P1: rows of P sum to one
@pytest.mark.parametrize("N,d", [(1, 4), (7, 3), (33, 16), (130, 8)])
def test_weights_are_a_distribution(N, d):
    q, k, v = rand(2, N, 3, d, 2.0), rand(2, N, 3, d, 2.0), rand(2, N, 3, d)
    o, lse, p = oracle.fwd_f64(q, k, v, 0.7, want_weights=True)
    assert p.shape == (2, 3, N, N)
    assert np.all(p >= 0.0)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=0, atol=1e-12)
    # the weights are exp(s - LSE) and O is their average of V
    s = np.einsum("bnhc,bmhc->bhnm", q, k) * 0.7
    np.testing.assert_allclose(p, np.exp(s - lse[..., None]), rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(o, np.einsum("bhnm,bmhc->bnhc", p, v), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- P2: identical keys -> mean of V
def test_identical_keys_give_mean_of_v():
    B, N, H, d = 2, 19, 2, 5
    q, v = rand(B, N, H, d), rand(B, N, H, d)
    k1 = rand(B, 1, H, d)
    k = np.repeat(k1, N, axis=1)
    scale = 0.3
    o, lse = oracle.fwd_f64(q, k, v, scale)
    mean_v = v.mean(axis=1, keepdims=True)
    np.testing.assert_allclose(o, np.broadcast_to(mean_v, o.shape), rtol=0, atol=1e-13)
    s = scale * np.einsum("bnhc,bhc->bhn", q, k1[:, 0])
    np.testing.assert_allclose(lse, s + math.log(N), rtol=0, atol=1e-12)
    # gradients: dK gets nothing in total per row (dS sums to zero), dV_j = mean over... = sum_i dO_i / N
    dO = rand(B, N, H, d)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, scale)
    np.testing.assert_allclose(dv, np.broadcast_to(dO.sum(1, keepdims=True) / N, dv.shape), atol=1e-13)
    # dS_ij = (1/N)(dP_ij - mean_j dP_ij); dQ_i = scale * sum_j dS_ij k = 0 since all k_j are equal
    np.testing.assert_allclose(dq, 0.0, atol=1e-13)


# ---------------------------------------------------------------- P3: N = 1
def test_single_token():
    B, H, d = 3, 2, 6
    q, k, v, dO = rand(B, 1, H, d), rand(B, 1, H, d), rand(B, 1, H, d), rand(B, 1, H, d)
    scale = 1.7
    o, lse = oracle.fwd_f64(q, k, v, scale)
    np.testing.assert_array_equal(o, v)
    np.testing.assert_allclose(lse[..., 0], scale * (q * k).sum(-1)[:, 0], rtol=1e-14, atol=1e-14)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, scale)
    np.testing.assert_array_equal(dv, dO)
    np.testing.assert_array_equal(dq, np.zeros_like(dq))
    np.testing.assert_array_equal(dk, np.zeros_like(dk))


# ---------------------------------------------------------------- P4: Q = 0 -> uniform weights
def test_zero_queries_give_uniform_weights():
    B, N, H, d = 1, 23, 2, 4
    q = np.zeros((B, N, H, d))
    k, v, dO = rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d)
    o, lse, p = oracle.fwd_f64(q, k, v, 0.5, want_weights=True)
    np.testing.assert_allclose(p, 1.0 / N, rtol=1e-14)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(1, keepdims=True), o.shape), atol=1e-14)
    np.testing.assert_allclose(lse, math.log(N), atol=1e-14)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, 0.5)
    np.testing.assert_allclose(dv, np.broadcast_to(dO.sum(1, keepdims=True) / N, dv.shape), atol=1e-14)
    np.testing.assert_allclose(dk, 0.0, atol=1e-14)   # dK_j = scale * sum_i dS_ij q_i with q = 0
    # dQ_i = scale * sum_j dS_ij k_j with dS_ij = (dP_ij - mean_j dP_ij)/N, dP_ij = <dO_i, v_j>
    dP = np.einsum("bnhc,bmhc->bhnm", dO, v)
    dS = (dP - dP.mean(-1, keepdims=True)) / N
    np.testing.assert_allclose(dq, 0.5 * np.einsum("bhnm,bmhc->bnhc", dS, k), atol=1e-13)


# ---------------------------------------------------------------- P11: hand-derived N=2, d=1 case
def _parse_golden(path):
    env = {"ln3": math.log(3.0), "ln4": math.log(4.0), "ln2": math.log(2.0)}
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = np.array([eval(x, {"__builtins__": {}}, env) for x in vals], dtype=np.float64)
    return out


def test_hand_derived_two_token_case():
    g = _parse_golden(os.path.join(os.path.dirname(__file__), "golden", "attn_n2_d1.txt"))
    sh = (1, 2, 1, 1)
    q, k, v, dO = (g[n].reshape(sh) for n in ("q", "k", "v", "dO"))
    o, lse, p = oracle.fwd_f64(q, k, v, 1.0, want_weights=True)
    np.testing.assert_allclose(p.ravel(), g["P"], rtol=1e-14)
    np.testing.assert_allclose(o.ravel(), g["O"], rtol=1e-14)
    np.testing.assert_allclose(lse.ravel(), g["LSE"], rtol=1e-14)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, 1.0)
    np.testing.assert_allclose(dq.ravel(), g["dQ"], rtol=1e-13)
    np.testing.assert_allclose(dk.ravel(), g["dK"], rtol=1e-13)
    np.testing.assert_allclose(dv.ravel(), g["dV"], rtol=1e-13)


def test_two_keys_are_a_sigmoid():
    # N = 2: P_i0 = sigmoid(s_i0 - s_i1), for any d
    q, k, v = rand(1, 2, 1, 5), rand(1, 2, 1, 5), rand(1, 2, 1, 5)
    scale = 0.9
    _, _, p = oracle.fwd_f64(q, k, v, scale, want_weights=True)
    s = scale * np.einsum("nc,mc->nm", q[0, :, 0], k[0, :, 0])
    np.testing.assert_allclose(p[0, 0, :, 0], 1.0 / (1.0 + np.exp(-(s[:, 0] - s[:, 1]))), rtol=1e-13)


# ---------------------------------------------------------------- P5: finite differences
@pytest.mark.parametrize("B,N,H,d,scale", [(1, 5, 1, 3, 0.6), (2, 8, 2, 4, 0.5), (1, 3, 2, 8, 1.3)])
def test_gradients_match_central_differences(B, N, H, d, scale):
    q, k, v, dO = rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, scale)

    def loss(q_, k_, v_):
        o, _ = oracle.fwd_f64(q_, k_, v_, scale, nthreads=1)
        return float((o * dO).sum())

    h = 1e-6
    for name, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += h
            xm[idx] -= h
            args_p = {"q": q, "k": k, "v": v}
            args_m = dict(args_p)
            args_p[name], args_m[name] = xp, xm
            num[idx] = (loss(**{a + "_": args_p[a] for a in args_p}) -
                        loss(**{a + "_": args_m[a] for a in args_m})) / (2 * h)
        denom = max(np.abs(num).max(), 1e-3)
        assert np.abs(num - grad).max() / denom < 1e-6, name


# ---------------------------------------------------------------- P6, P7: invariants of the gradients
def test_gradient_invariants():
    B, N, H, d = 2, 37, 3, 8
    q, k, v, dO = rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d)
    scale = 0.35
    o, lse, p = oracle.fwd_f64(q, k, v, scale, want_weights=True)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, scale)
    # every row of dS sums to zero, hence: sum_j dV_j = sum_i dO_i (P rows sum to 1) and
    # <dQ_i, q_i> summed over i equals <dK_j, k_j> summed over j (both are scale * sum dS*S/scale)
    np.testing.assert_allclose(dv.sum(1), dO.sum(1), atol=1e-12)
    np.testing.assert_allclose((dq * q).sum((1, 3)), (dk * k).sum((1, 3)), atol=1e-11)
    # P7: sum_k P_ik dP_ik == sum_c dO_ic O_ic  (the shortcut the fused backward uses)
    dP = np.einsum("bnhc,bmhc->bhnm", dO, v)
    np.testing.assert_allclose((p * dP).sum(-1), np.einsum("bnhc,bnhc->bhn", dO, o), atol=1e-12)
    # dK from the definition with dS = P*(dP - delta)
    delta = np.einsum("bnhc,bnhc->bhn", dO, o)
    dS = p * (dP - delta[..., None])
    np.testing.assert_allclose(dS.sum(-1), 0.0, atol=1e-12)
    np.testing.assert_allclose(dk, scale * np.einsum("bhnm,bnhc->bmhc", dS, q), atol=1e-12)
    np.testing.assert_allclose(dq, scale * np.einsum("bhnm,bmhc->bnhc", dS, k), atol=1e-12)
    np.testing.assert_allclose(dv, np.einsum("bhnm,bnhc->bmhc", p, dO), atol=1e-12)


# ---------------------------------------------------------------- P8: block-merge identity (Sec. 1)
@pytest.mark.parametrize("split", [1, 13, 40])
def test_blockwise_results_combine_to_the_final_output(split):
    # Splitting the keys into two blocks and merging (O1, L1), (O2, L2) through their log-sum-exps
    # gives the one-shot result: this is what "combines the block-wise results" means.
    B, N, H, d = 1, 41, 2, 6
    q, k, v = rand(B, N, H, d, 1.5), rand(B, N, H, d, 1.5), rand(B, N, H, d)
    scale = 0.4
    o, lse = oracle.fwd_f64(q, k, v, scale)

    def partial(keys):
        # queries against a subset of keys: evaluate with the dense helper (different code)
        oo, ll, _ = dense_reference(q, k[:, keys], v[:, keys], scale)
        return oo, ll

    o1, l1 = partial(slice(0, split))
    o2, l2 = partial(slice(split, N))
    L = np.logaddexp(l1, l2)
    w1 = np.exp(l1 - L).transpose(0, 2, 1)[..., None]
    w2 = np.exp(l2 - L).transpose(0, 2, 1)[..., None]
    np.testing.assert_allclose(lse, L, atol=1e-12)
    np.testing.assert_allclose(o, w1 * o1 + w2 * o2, atol=1e-12)


# ---------------------------------------------------------------- P9: shift / permutation invariance
def test_key_shift_and_permutation():
    B, N, H, d = 1, 29, 2, 7
    q, k, v, dO = rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d)
    scale = 0.45
    o, lse = oracle.fwd_f64(q, k, v, scale)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, scale)
    c = rand(B, 1, H, d)
    o2, lse2 = oracle.fwd_f64(q, k + c, v, scale)
    np.testing.assert_allclose(o2, o, atol=1e-12)
    np.testing.assert_allclose(lse2 - lse, scale * np.einsum("bnhc,bhc->bhn", q, c[:, 0]), atol=1e-12)
    perm = RNG.permutation(N)
    o3, lse3 = oracle.fwd_f64(q, k[:, perm], v[:, perm], scale)
    np.testing.assert_allclose(o3, o, atol=1e-12)
    np.testing.assert_allclose(lse3, lse, atol=1e-12)
    dq3, dk3, dv3 = oracle.bwd_f64(q, k[:, perm], v[:, perm], dO, scale)
    np.testing.assert_allclose(dq3, dq, atol=1e-12)
    np.testing.assert_allclose(dk3, dk[:, perm], atol=1e-12)
    np.testing.assert_allclose(dv3, dv[:, perm], atol=1e-12)


def test_heads_and_batches_do_not_mix():
    # [B,N,H,d] indexing: each (b,h) slice run alone gives the same numbers as inside the batch
    B, N, H, d = 2, 11, 3, 4
    q, k, v, dO = rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d)
    o, lse = oracle.fwd_f64(q, k, v, 0.5)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, 0.5)
    for b in range(B):
        for h in range(H):
            sl = (slice(b, b + 1), slice(None), slice(h, h + 1))
            o1, l1 = oracle.fwd_f64(q[sl], k[sl], v[sl], 0.5)
            np.testing.assert_allclose(o[sl], o1, atol=1e-14)
            np.testing.assert_allclose(lse[b, h], l1[0, 0], atol=1e-14)
            g = oracle.bwd_f64(q[sl], k[sl], v[sl], dO[sl], 0.5)
            for full, part in zip((dq, dk, dv), g):
                np.testing.assert_allclose(full[sl], part, atol=1e-13)


# ---------------------------------------------------------------- P10: dense library computation + autograd
@pytest.mark.parametrize("B,N,H,d", [(2, 50, 3, 16), (1, 257, 2, 64), (1, 96, 1, 80)])
def test_matches_dense_softmax_and_autograd(B, N, H, d):
    torch = pytest.importorskip("torch")
    q, k, v, dO = rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d)
    scale = 1.0 / math.sqrt(d)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    s = torch.einsum("bnhc,bmhc->bhnm", tq, tk) * scale
    to = torch.einsum("bhnm,bmhc->bnhc", torch.softmax(s, dim=-1), tv)
    to.backward(torch.tensor(dO))
    o, lse = oracle.fwd_f64(q, k, v, scale)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, scale)
    np.testing.assert_allclose(o, to.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(lse, torch.logsumexp(s, dim=-1).detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-11)


# ---------------------------------------------------------------- bf16 entry points and threads
def test_bf16_entry_points_widen_exactly_and_threads_agree():
    import synth_inputs as si
    w = si.small_workload(2, 2, 45, 16, seed=7)
    x = si.make_inputs(w)
    f = {n: si.bf16_bits_to_f64(x[n]) for n in x}
    o, lse = oracle.fwd(x["q"], x["k"], x["v"], w.scale)
    o2, lse2 = oracle.fwd_f64(f["q"], f["k"], f["v"], w.scale)
    np.testing.assert_array_equal(o, o2)
    np.testing.assert_array_equal(lse, lse2)
    g = oracle.bwd(x["q"], x["k"], x["v"], x["dO"], w.scale, nthreads=3)
    g2 = oracle.bwd_f64(f["q"], f["k"], f["v"], f["dO"], w.scale, nthreads=1)
    for a, b in zip(g, g2):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_large_scores_do_not_overflow():
    q = np.full((1, 4, 1, 2), 30.0)
    k = np.full((1, 4, 1, 2), 30.0)
    k[0, 2] = -30.0
    v = rand(1, 4, 1, 2)
    o, lse = oracle.fwd_f64(q, k, v, 1.0)
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))
    # three keys tie at s = 1800, one is at -1800 (weight exactly 0 in fp64)
    np.testing.assert_allclose(o[0, 0, 0], v[0, [0, 1, 3], 0].mean(0), atol=1e-13)
    np.testing.assert_allclose(lse, 1800.0 + math.log(3.0), atol=1e-10)


# ================================================================ causal variant (GPT-like text encoder)
# ---------------------------------------------------------------- C1: closed forms of the first and last rows
def test_causal_first_row_is_v0_and_last_row_is_unmasked():
    B, N, H, d = 2, 23, 3, 5
    q, k, v = rand(B, N, H, d, 1.5), rand(B, N, H, d, 1.5), rand(B, N, H, d)
    scale = 0.4
    o, lse, p = oracle.fwd_f64(q, k, v, scale, want_weights=True, causal=True)
    # token 0 sees only itself: O_0 = v_0 and LSE_0 = s_00
    np.testing.assert_allclose(o[:, 0], v[:, 0], rtol=0, atol=1e-15)
    np.testing.assert_allclose(lse[:, :, 0], scale * np.einsum("bhc,bhc->bh", q[:, 0], k[:, 0]), rtol=0, atol=1e-13)
    # the last token sees every key: same as the unmasked operation
    o_full, lse_full = oracle.fwd_f64(q, k, v, scale)
    np.testing.assert_allclose(o[:, -1], o_full[:, -1], rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse[:, :, -1], lse_full[:, :, -1], rtol=0, atol=1e-13)
    # weights: zero above the diagonal, a distribution over the visible keys
    assert np.all(np.triu(p, 1) == 0.0)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- C2: prefix property
@pytest.mark.parametrize("M", [1, 6, 17])
def test_causal_prefix_does_not_depend_on_later_tokens(M):
    B, N, H, d = 1, 30, 2, 4
    q, k, v, dO = rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d)
    o, lse = oracle.fwd_f64(q, k, v, 0.5, causal=True)
    om, lsem = oracle.fwd_f64(q[:, :M], k[:, :M], v[:, :M], 0.5, causal=True)
    np.testing.assert_allclose(o[:, :M], om, rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse[:, :, :M], lsem, rtol=0, atol=1e-13)
    # and the gradient with respect to the first M queries, when only their outputs carry gradient
    g = dO.copy()
    g[:, M:] = 0.0
    dq, dk, dv = oracle.bwd_f64(q, k, v, g, 0.5, causal=True)
    dqm, dkm, dvm = oracle.bwd_f64(q[:, :M], k[:, :M], v[:, :M], dO[:, :M], 0.5, causal=True)
    np.testing.assert_allclose(dq[:, :M], dqm, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dk[:, :M], dkm, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dv[:, :M], dvm, rtol=0, atol=1e-13)
    assert np.all(dq[:, M:] == 0.0) and np.all(dk[:, M:] == 0.0) and np.all(dv[:, M:] == 0.0)


# ---------------------------------------------------------------- C3: dense masked softmax + autograd
@pytest.mark.parametrize("B,N,H,d", [(2, 1, 2, 8), (2, 50, 3, 16), (1, 77, 2, 64)])
def test_causal_matches_dense_masked_softmax_and_autograd(B, N, H, d):
    torch = pytest.importorskip("torch")
    q, k, v, dO = rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d)
    scale = 1.0 / math.sqrt(d)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    s = torch.einsum("bnhc,bmhc->bhnm", tq, tk) * scale
    s = s.masked_fill(torch.triu(torch.ones(N, N, dtype=torch.bool), diagonal=1), float("-inf"))
    to = torch.einsum("bhnm,bmhc->bnhc", torch.softmax(s, dim=-1), tv)
    to.backward(torch.tensor(dO))
    o, lse = oracle.fwd_f64(q, k, v, scale, causal=True)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, scale, causal=True)
    np.testing.assert_allclose(o, to.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(lse, torch.logsumexp(s, dim=-1).detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-11)


# ---------------------------------------------------------------- C4: finite differences, last key's closed form
def test_causal_gradients_match_central_differences_and_last_key_closed_form():
    B, N, H, d, scale = 1, 6, 2, 3, 0.7
    q, k, v, dO = rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d), rand(B, N, H, d)
    dq, dk, dv = oracle.bwd_f64(q, k, v, dO, scale, causal=True)
    _, _, p = oracle.fwd_f64(q, k, v, scale, want_weights=True, causal=True)
    # only the last query sees the last key: dV_last = P_last,last * dO_last
    np.testing.assert_allclose(dv[:, -1], p[:, :, -1, -1][..., None] * dO[:, -1], rtol=0, atol=1e-14)

    def loss(q_, k_, v_):
        o, _ = oracle.fwd_f64(q_, k_, v_, scale, nthreads=1, causal=True)
        return float((o * dO).sum())

    h = 1e-6
    for name, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += h
            xm[idx] -= h
            a_p = {"q": q, "k": k, "v": v}
            a_m = dict(a_p)
            a_p[name], a_m[name] = xp, xm
            num[idx] = (loss(a_p["q"], a_p["k"], a_p["v"]) - loss(a_m["q"], a_m["k"], a_m["v"])) / (2 * h)
        denom = max(np.abs(num).max(), 1e-3)
        assert np.abs(num - grad).max() / denom < 1e-6, name


def test_causal_bf16_entry_points_widen_exactly():
    import synth_inputs as si
    w = si.small_workload(2, 2, 45, 16, seed=8)
    x = si.make_inputs(w)
    f = {n: si.bf16_bits_to_f64(x[n]) for n in x}
    o1, l1 = oracle.fwd(x["q"], x["k"], x["v"], w.scale, causal=True)
    o2, l2 = oracle.fwd_f64(f["q"], f["k"], f["v"], w.scale, causal=True)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    g1 = oracle.bwd(x["q"], x["k"], x["v"], x["dO"], w.scale, causal=True)
    g2 = oracle.bwd_f64(f["q"], f["k"], f["v"], f["dO"], w.scale, causal=True)
    for a, b in zip(g1, g2):
        assert np.array_equal(a, b)
