"""CPU oracle for layer normalisation over the channel axis, forward and backward.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this module; it shares
nothing with the HIP path and never imports it.

What it computes.  Every encoder layer of the paper's plain video ViT (Sec. 3, "Video Transformer":
multi-head self-attention and a two-layer MLP per layer) normalises its tokens before each of the two
blocks, and the paper's memory profile (Sec. 4.1, figure "memory profile") lists LayerNorm as one of
the three consumers of activation memory.  The paper writes no formula; this is the textbook
definition, per token row x in R^D, in fp64:

    forward :  mu = (1/D) sum_c x_c ,  var = (1/D) sum_c (x_c - mu)^2 ,  rstd = 1 / sqrt(var + eps)
               xhat_c = (x_c - mu) * rstd ,  y_c = xhat_c * gamma_c + beta_c
    backward, for a given upstream gradient dy (any loss), by differentiating the lines above:
               dbeta_c  = sum_rows dy_c ,  dgamma_c = sum_rows dy_c * xhat_c
               g_c = dy_c * gamma_c
               dx_c = rstd * ( g_c - (1/D) sum_k g_k - xhat_c * (1/D) sum_k g_k xhat_k )

The variance is the biased one (divisor D) taken about the mean (two passes), as in every ViT.
Inputs are fp64 arrays [M, D] (M = tokens), or bf16 / fp16 bit patterns widened exactly by the caller.
No blocking, no fusion: one vectorised numpy expression per line of the definition.
"""
from __future__ import annotations

import numpy as np


def fwd(x, gamma, beta, eps):
    """Returns y [M, D], mean [M], rstd [M], all float64."""
    x = np.asarray(x, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    mu = x.sum(axis=1) / x.shape[1]
    centred = x - mu[:, None]
    var = (centred * centred).sum(axis=1) / x.shape[1]
    rstd = 1.0 / np.sqrt(var + eps)
    y = centred * rstd[:, None] * gamma[None, :] + beta[None, :]
    return y, mu, rstd


def bwd(x, gamma, dy, eps):
    """Returns dx [M, D], dgamma [D], dbeta [D], all float64."""
    x = np.asarray(x, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    D = x.shape[1]
    mu = x.sum(axis=1) / D
    centred = x - mu[:, None]
    var = (centred * centred).sum(axis=1) / D
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = centred * rstd[:, None]
    dbeta = dy.sum(axis=0)
    dgamma = (dy * xhat).sum(axis=0)
    g = dy * gamma[None, :]
    dx = rstd[:, None] * (g - g.sum(axis=1)[:, None] / D - xhat * ((g * xhat).sum(axis=1)[:, None] / D))
    return dx, dgamma, dbeta
