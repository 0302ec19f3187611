"""Pins of the layer-normalisation oracle (oracle/layernorm.py) to things other than itself: a
hand-derived worked case, invariances that the definition implies, central finite differences of
every input coordinate, and a dense library computation with autograd.  Runs on the CPU."""
import math
import os

import numpy as np
import pytest

from oracle import layernorm as ln

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "layernorm_d2.txt")


def _golden():
    r = 1.0 / math.sqrt(6.5)
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, *vals = line.split()
        out[name] = np.array([eval(v, {"r": r}) for v in vals], dtype=np.float64)
    return out


def test_hand_derived_rows():
    g = _golden()
    y, mu, rstd = ln.fwd(g["row1_x"][None], g["row1_gamma"], g["row1_beta"], 0.0)
    assert np.allclose(y[0], g["row1_y"], atol=1e-13) and abs(mu[0] - 2) < 1e-15 and abs(rstd[0] - 1) < 1e-15
    dx, dg, db = ln.bwd(g["row1_x"][None], g["row1_gamma"], g["row1_dy"][None], 0.0)
    assert np.allclose(dx[0], g["row1_dx"], atol=1e-13)
    assert np.allclose(dg, g["row1_dgamma"], atol=1e-13) and np.allclose(db, g["row1_dbeta"], atol=1e-13)
    eps = float(g["row2_eps"][0])
    y, _, _ = ln.fwd(g["row2_x"][None], np.ones(3), np.zeros(3), eps)
    assert np.allclose(y[0], g["row2_y"], atol=1e-13)
    dx, _, _ = ln.bwd(g["row2_x"][None], np.ones(3), g["row2_dy"][None], eps)
    assert np.allclose(dx[0], g["row2_dx"], atol=1e-13)


def _case(M, D, seed):
    rng = np.random.default_rng(seed)
    return (rng.normal(size=(M, D)) * 1.7 + 0.4, rng.normal(size=D) * 0.5 + 1.0, rng.normal(size=D) * 0.3,
            rng.normal(size=(M, D)))


@pytest.mark.parametrize("M,D", [(1, 1), (3, 2), (5, 7), (4, 64), (2, 768)])
def test_forward_invariants(M, D):
    x, gamma, beta, _ = _case(M, D, 11 * M + D)
    eps = 1e-5
    y, mu, rstd = ln.fwd(x, np.ones(D), np.zeros(D), eps)
    var = x.var(axis=1)                      # numpy's own biased variance
    assert np.allclose(mu, x.mean(axis=1), atol=1e-13)
    assert np.allclose(rstd, 1.0 / np.sqrt(var + eps), rtol=1e-13)
    # unit gain, zero bias: rows have mean 0 and second moment var / (var + eps)
    assert np.allclose(y.mean(axis=1), 0.0, atol=1e-13)
    assert np.allclose((y * y).mean(axis=1), var / (var + eps), rtol=1e-12, atol=1e-15)
    # a constant added to a row changes nothing; gain and bias act channel by channel
    y2, _, _ = ln.fwd(x + 123.0, gamma, beta, eps)
    assert np.allclose(y2, y * gamma + beta, atol=1e-10)
    # without eps the output does not depend on the scale of the row
    if D > 1:
        a, _, _ = ln.fwd(x, gamma, beta, 0.0)
        b, _, _ = ln.fwd(x * 37.5, gamma, beta, 0.0)
        assert np.allclose(a, b, atol=1e-11)


@pytest.mark.parametrize("M,D", [(3, 2), (4, 5), (2, 33)])
def test_gradients_against_central_finite_differences(M, D):
    x, gamma, beta, dy = _case(M, D, 1000 + D)
    eps = 1e-3
    dx, dg, db = ln.bwd(x, gamma, dy, eps)
    loss = lambda xx, gg, bb: float((ln.fwd(xx, gg, bb, eps)[0] * dy).sum())
    h = 1e-6
    for i in range(M):
        for c in range(D):
            e = np.zeros_like(x)
            e[i, c] = h
            assert abs((loss(x + e, gamma, beta) - loss(x - e, gamma, beta)) / (2 * h) - dx[i, c]) < 1e-6 * (1 + abs(dx[i, c]))
    for c in range(D):
        e = np.zeros(D)
        e[c] = h
        assert abs((loss(x, gamma + e, beta) - loss(x, gamma - e, beta)) / (2 * h) - dg[c]) < 1e-6 * (1 + abs(dg[c]))
        assert abs((loss(x, gamma, beta + e) - loss(x, gamma, beta - e)) / (2 * h) - db[c]) < 1e-6 * (1 + abs(db[c]))


@pytest.mark.parametrize("M,D", [(4, 3), (3, 64), (2, 1024)])
def test_gradient_identities(M, D):
    x, gamma, _, dy = _case(M, D, 2000 + D)
    eps = 1e-5
    dx, dg, db = ln.bwd(x, gamma, dy, eps)
    y, mu, rstd = ln.fwd(x, np.ones(D), np.zeros(D), eps)        # y = xhat here
    # the output ignores a constant shift of the row, so dx sums to zero over the channels
    assert np.allclose(dx.sum(axis=1), 0.0, atol=1e-11)
    # along xhat only the eps part of the scale dependence survives:
    #   sum_c dx_c xhat_c = rstd * sum_c g_c xhat_c * eps / (var + eps)
    g = dy * gamma
    var = x.var(axis=1)
    assert np.allclose((dx * y).sum(axis=1), rstd * (g * y).sum(axis=1) * eps / (var + eps), rtol=1e-9, atol=1e-13)
    # linearity in dy, and the parameter gradients are plain column sums
    dx2, dg2, db2 = ln.bwd(x, gamma, 3.0 * dy, eps)
    assert np.allclose(dx2, 3.0 * dx) and np.allclose(dg2, 3.0 * dg) and np.allclose(db2, 3.0 * db)
    assert np.allclose(db, dy.sum(axis=0)) and np.allclose(dg, (dy * y).sum(axis=0))


@pytest.mark.parametrize("M,D", [(7, 16), (5, 768)])
def test_matches_library_layer_norm_and_autograd(M, D):
    import torch
    x, gamma, beta, dy = _case(M, D, 3000 + D)
    eps = 1e-5
    xt, gt, bt = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, gamma, beta))
    yt = torch.nn.functional.layer_norm(xt, (D,), gt, bt, eps)
    (yt * torch.tensor(dy)).sum().backward()
    y, _, _ = ln.fwd(x, gamma, beta, eps)
    dx, dg, db = ln.bwd(x, gamma, dy, eps)
    assert np.allclose(y, yt.detach().numpy(), atol=1e-12)
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-11)
    assert np.allclose(dg, gt.grad.numpy(), atol=1e-11) and np.allclose(db, bt.grad.numpy(), atol=1e-11)


def test_constant_row():
    # every channel equal: xhat = 0, y = beta, and dx = rstd * (g - mean g) with rstd = 1/sqrt(eps)
    D, eps = 6, 0.25
    x = np.full((1, D), 4.0)
    gamma = np.arange(1.0, D + 1)
    dy = np.linspace(-1, 1, D)[None]
    y, mu, rstd = ln.fwd(x, gamma, np.full(D, 0.5), eps)
    assert np.allclose(y, 0.5) and mu[0] == 4.0 and abs(rstd[0] - 2.0) < 1e-15
    dx, dg, _ = ln.bwd(x, gamma, dy, eps)
    g = dy[0] * gamma
    assert np.allclose(dx[0], 2.0 * (g - g.mean()), atol=1e-13) and np.allclose(dg, 0.0)
