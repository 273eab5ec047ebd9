"""Float64 NumPy oracle of Group Layer Normalization (GLN) and of the gated form GLN(A) * U.

TEST INFRASTRUCTURE ONLY: it exists to check the GPU library and is never part of the product path.

What it computes (Section 3.2.2: the tokens of a layer's input are assigned to groups -- one per history sequence,
per real-time sequence, per scenario -- and group layer normalization is applied, X~ = GLN(X); the layer's output
is f2(GLN(A) (.) U) + X): every token is normalised over its d_model features like a LayerNorm, and the affine
parameters are those of the token's group,
    mean_i = (1/d) sum_c x_ic,   var_i = (1/d) sum_c (x_ic - mean_i)^2,   xhat_i = (x_i - mean_i) / sqrt(var_i + eps)
    y_i = gamma[g_i] * xhat_i + beta[g_i]            (times u_i elementwise when a gate U is given)
Reading where the paper is silent: the statistics are per token (a LayerNorm), what is "grouped" are the parameters;
the variance is the biased one; eps is an explicit argument.
Backward for an upstream gradient dy (written out from the definition):
    dz_i = dy_i * u_i (or dy_i),  du_i = dy_i * (gamma[g_i] * xhat_i + beta[g_i])
    dgamma[g] = sum_{i in g} dz_i * xhat_i,   dbeta[g] = sum_{i in g} dz_i
    w_i = dz_i * gamma[g_i],   dx_i = rstd_i * (w_i - mean_c(w_i) - xhat_i * mean_c(w_i * xhat_i))
"""
from __future__ import annotations

import numpy as np


def forward(x, group_id, gamma, beta, eps, gate=None):
    """Returns (y, mean, rstd) in float64: y [n, d], mean and rstd [n]."""
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(group_id, dtype=np.int64)
    gamma = np.asarray(gamma, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    assert x.ndim == 2 and g.shape == (x.shape[0],) and gamma.shape == beta.shape and gamma.shape[1] == x.shape[1]
    assert g.size == 0 or (g.min() >= 0 and g.max() < gamma.shape[0])
    n, d = x.shape
    y = np.zeros((n, d))
    mean = np.zeros(n)
    rstd = np.zeros(n)
    for i in range(n):
        mean[i] = x[i].sum() / d
        var = ((x[i] - mean[i]) ** 2).sum() / d
        rstd[i] = 1.0 / np.sqrt(var + eps)
        xhat = (x[i] - mean[i]) * rstd[i]
        y[i] = gamma[g[i]] * xhat + beta[g[i]]
        if gate is not None:
            y[i] = y[i] * np.asarray(gate[i], dtype=np.float64)
    return y, mean, rstd


def backward(dy, x, group_id, gamma, beta, eps, gate=None):
    """Returns (dx, dgamma, dbeta, du) in float64; du is None without a gate."""
    dy = np.asarray(dy, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(group_id, dtype=np.int64)
    gamma = np.asarray(gamma, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    n, d = x.shape
    dx = np.zeros((n, d))
    du = None if gate is None else np.zeros((n, d))
    dgamma = np.zeros(gamma.shape)
    dbeta = np.zeros(beta.shape)
    for i in range(n):
        mean = x[i].sum() / d
        var = ((x[i] - mean) ** 2).sum() / d
        rstd = 1.0 / np.sqrt(var + eps)
        xhat = (x[i] - mean) * rstd
        dz = dy[i]
        if gate is not None:
            du[i] = dy[i] * (gamma[g[i]] * xhat + beta[g[i]])
            dz = dy[i] * np.asarray(gate[i], dtype=np.float64)
        dgamma[g[i]] += dz * xhat
        dbeta[g[i]] += dz
        w = dz * gamma[g[i]]
        dx[i] = rstd * (w - w.sum() / d - xhat * (w * xhat).sum() / d)
    return dx, dgamma, dbeta, du
