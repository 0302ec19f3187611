"""Pins of the bias + GELU oracle (oracle/gelu.py) to things other than itself: entries of the standard
normal table, the reflection identity, limits, the distribution function obtained by integrating the
density numerically (no erf), central finite differences in every coordinate, and a dense library
computation with autograd.  Runs on the CPU."""
import os

import numpy as np
import pytest

from oracle import gelu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "gelu_normal_table.txt")


def _table():
    rows = [tuple(float(v) for v in line.split()) for line in open(GOLDEN) if line.strip() and not line.startswith("#")]
    return np.array(rows)


def test_values_of_the_standard_normal_table():
    t = _table()
    h, cdf, pdf = t[:, 0], t[:, 1], t[:, 2]
    zero = np.zeros(1)
    for sign in (1.0, -1.0):
        x = (sign * h)[:, None]
        want = x[:, 0] * (cdf if sign > 0 else 1.0 - cdf)
        assert np.abs(gelu.fwd(x, zero)[:, 0] - want).max() < 6e-10 * max(1.0, h.max())   # table printed to ten decimals
        dx, db = gelu.bwd(x, zero, np.ones_like(x))
        want_d = (cdf if sign > 0 else 1.0 - cdf) + sign * h * pdf
        assert np.abs(dx[:, 0] - want_d).max() < 6e-10 * (1.0 + h.max())
        assert abs(db[0] - want_d.sum()) < 1e-8
    # the bias is added before the activation: GELU(0.25 + 0.75) is the table's row h = 1
    assert abs(gelu.fwd(np.full((1, 1), 0.25), np.array([0.75]))[0, 0] - 0.8413447461) < 6e-10


def test_reflection_identity_and_limits():
    rng = np.random.default_rng(5)
    x = rng.normal(size=(7, 33)) * 3.0
    b = rng.normal(size=33)
    h = x + b
    # Phi(h) + Phi(-h) = 1  =>  GELU(h) - GELU(-h) = h, and GELU'(h) + GELU'(-h) = 1
    assert np.abs(gelu.fwd(x, b) - gelu.fwd(-x, -b) - h).max() < 1e-14
    one = np.ones_like(x)
    assert np.abs(gelu.bwd(x, b, one)[0] + gelu.bwd(-x, -b, one)[0] - 1.0).max() < 1e-14
    big = np.array([[12.0, 30.0, -12.0, -30.0]])
    y = gelu.fwd(big, np.zeros(4))[0]
    assert abs(y[0] - 12.0) < 1e-12 and y[1] == 30.0 and abs(y[2]) < 1e-12 and abs(y[3]) < 1e-300
    d = gelu.bwd(big, np.zeros(4), np.ones((1, 4)))[0][0]
    assert abs(d[0] - 1.0) < 1e-12 and abs(d[2]) < 1e-12
    # the minimum of GELU lies where Phi(h) + h phi(h) = 0: h = -0.7517915..., a known constant of the function
    hmin = np.array([[-0.75179157]])
    assert abs(gelu.bwd(hmin, np.zeros(1), np.ones((1, 1)))[0][0, 0]) < 1e-7
    assert abs(gelu.fwd(hmin, np.zeros(1))[0, 0] + 0.16997120) < 1e-7


def test_distribution_function_by_numerical_integration_of_the_density():
    # Phi(h) = 1/2 + int_0^h phi(t) dt by composite Simpson on 4000 panels: no erf anywhere
    def cdf(hv):
        n = 4000
        t = np.linspace(0.0, hv, n + 1)
        f = np.exp(-0.5 * t * t) / np.sqrt(2.0 * np.pi)
        return 0.5 + (hv / n) / 3.0 * (f[0] + f[-1] + 4.0 * f[1:-1:2].sum() + 2.0 * f[2:-1:2].sum())
    hs = np.array([-3.7, -2.2, -0.9, -0.1, 0.3, 1.1, 2.6, 4.4])
    want = np.array([hv * cdf(hv) for hv in hs])
    got = gelu.fwd(hs[None, :], np.zeros(len(hs)))[0]
    assert np.abs(got - want).max() < 1e-12


@pytest.mark.parametrize("M,F", [(1, 1), (3, 5), (4, 16)])
def test_backward_by_central_differences_in_every_coordinate(M, F):
    rng = np.random.default_rng(100 * M + F)
    x, b, dy = rng.normal(size=(M, F)) * 1.5, rng.normal(size=F), rng.normal(size=(M, F))
    dx, db = gelu.bwd(x, b, dy)
    loss = lambda xx, bb: float((gelu.fwd(xx, bb) * dy).sum())
    step = 1e-5
    for i in range(M):
        for j in range(F):
            e = np.zeros_like(x)
            e[i, j] = step
            fd = (loss(x + e, b) - loss(x - e, b)) / (2 * step)
            assert abs(fd - dx[i, j]) < 1e-8 * (1 + abs(dx[i, j])), (i, j)
    for j in range(F):
        e = np.zeros_like(b)
        e[j] = step
        fd = (loss(x, b + e) - loss(x, b - e)) / (2 * step)
        assert abs(fd - db[j]) < 1e-8 * (1 + abs(db[j])), j


def test_structure_of_the_gradients():
    rng = np.random.default_rng(9)
    x, b = rng.normal(size=(6, 10)), rng.normal(size=10)
    dy1, dy2 = rng.normal(size=(6, 10)), rng.normal(size=(6, 10))
    d1, b1 = gelu.bwd(x, b, dy1)
    d2, b2 = gelu.bwd(x, b, dy2)
    d3, b3 = gelu.bwd(x, b, 2.0 * dy1 - 0.5 * dy2)
    assert np.abs(d3 - (2.0 * d1 - 0.5 * d2)).max() < 1e-14 and np.abs(b3 - (2.0 * b1 - 0.5 * b2)).max() < 1e-13   # linear in dy
    assert np.abs(b1 - d1.sum(axis=0)).max() < 1e-14                      # the bias gradient is the column sum of dx
    assert np.abs(gelu.fwd(x, b) - gelu.fwd(x + b[None, :], np.zeros(10))).max() == 0.0   # the bias only shifts the argument
    # rows are independent: permuting the rows permutes y and dx and leaves dbias alone
    perm = rng.permutation(6)
    assert np.abs(gelu.fwd(x[perm], b) - gelu.fwd(x, b)[perm]).max() == 0.0
    dp, bp = gelu.bwd(x[perm], b, dy1[perm])
    assert np.abs(dp - d1[perm]).max() == 0.0 and np.abs(bp - b1).max() < 1e-14


def test_against_a_dense_library_computation_with_autograd():
    import torch
    rng = np.random.default_rng(21)
    x, b, dy = rng.normal(size=(9, 40)) * 2.0, rng.normal(size=40), rng.normal(size=(9, 40))
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tb = torch.tensor(b, dtype=torch.float64, requires_grad=True)
    ty = torch.nn.functional.gelu(tx + tb)            # the exact (erf) form is the library's default
    ty.backward(torch.tensor(dy, dtype=torch.float64))
    assert np.abs(gelu.fwd(x, b) - ty.detach().numpy()).max() < 1e-14
    dx, db = gelu.bwd(x, b, dy)
    assert np.abs(dx - tx.grad.numpy()).max() < 1e-13 and np.abs(db - tb.grad.numpy()).max() < 1e-12
