"""CPU oracle for the bias + GELU step of the encoder's two-layer MLP, forward and backward.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this module; it shares
nothing with the HIP path and never imports it.

What it computes.  Every encoder layer of the paper's plain video ViT holds a two-layer MLP (Sec. 3,
"Video Transformer"), the third consumer of activation memory in the paper's memory profile (Sec. 4.1,
figure "memory footprint").  Between the MLP's two matrix products sits an elementwise step: add the
first layer's bias and apply the activation.  The paper names neither; the reading taken is the exact
Gaussian-error linear unit of the plain ViT, in fp64, per element h = x + b:

    forward :  y  = h * Phi(h) ,                  Phi(h) = (1 + erf(h / sqrt 2)) / 2
    backward:  dx = dy * (Phi(h) + h * phi(h)) ,  phi(h) = exp(-h^2 / 2) / sqrt(2 pi)
               dbias_c = sum_rows dx_c

x is the [M, F] output of the first matrix product (without bias), bias is [F].  erf is the library's
(scipy.special.erf); nothing is blocked or fused: one vectorised numpy expression per line above.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf


def fwd(x, bias):
    """Returns y [M, F], float64."""
    h = np.asarray(x, dtype=np.float64) + np.asarray(bias, dtype=np.float64)[None, :]
    return h * (0.5 * (1.0 + erf(h / np.sqrt(2.0))))


def bwd(x, bias, dy):
    """Returns dx [M, F], dbias [F], float64."""
    h = np.asarray(x, dtype=np.float64) + np.asarray(bias, dtype=np.float64)[None, :]
    cdf = 0.5 * (1.0 + erf(h / np.sqrt(2.0)))
    pdf = np.exp(-0.5 * h * h) / np.sqrt(2.0 * np.pi)
    dx = np.asarray(dy, dtype=np.float64) * (cdf + h * pdf)
    return dx, dx.sum(axis=0)
