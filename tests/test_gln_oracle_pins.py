"""Pins for the float64 oracle of group layer normalization: the library LayerNorm for every group, autograd through
an independently written expression, central differences, and the invariants a per-token normalisation with
group-wise parameters has.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import gln_oracle as G
from paper_2602_11235_amd import inputs


def small(gated, n=23, d=12, groups=3, seed=5):
    return inputs.make_gln_case("small", n, d, groups, dtype="fp32", gated=gated, seed=seed)


@pytest.mark.parametrize("gated", [False, True])
def test_every_group_is_the_library_layer_norm_with_that_groups_parameters(gated):
    c = small(gated)
    y, mean, rstd = G.forward(c.x, c.group_id, c.gamma, c.beta, c.eps, c.gate)
    x = torch.tensor(c.x, dtype=torch.float64)
    for g in range(c.gamma.shape[0]):
        rows = np.nonzero(c.group_id == g)[0]
        ref = torch.nn.functional.layer_norm(x[rows], (x.shape[1],), torch.tensor(c.gamma[g], dtype=torch.float64),
                                             torch.tensor(c.beta[g], dtype=torch.float64), c.eps).numpy()
        if gated:
            ref = ref * c.gate[rows].astype(np.float64)
        assert np.allclose(y[rows], ref, rtol=1e-12, atol=1e-12)
    assert np.allclose(mean, c.x.astype(np.float64).mean(axis=1), atol=1e-13)
    assert np.allclose(rstd, 1.0 / np.sqrt(c.x.astype(np.float64).var(axis=1) + c.eps), rtol=1e-12)


@pytest.mark.parametrize("gated", [False, True])
def test_backward_equals_autograd(gated):
    c = small(gated)
    x = torch.tensor(c.x, dtype=torch.float64, requires_grad=True)
    gamma = torch.tensor(c.gamma, dtype=torch.float64, requires_grad=True)
    beta = torch.tensor(c.beta, dtype=torch.float64, requires_grad=True)
    u = torch.tensor(c.gate, dtype=torch.float64, requires_grad=True) if gated else None
    gid = torch.tensor(c.group_id, dtype=torch.long)
    mu = x.mean(dim=1, keepdim=True)
    xc = x - mu
    xhat = xc / torch.sqrt((xc * xc).mean(dim=1, keepdim=True) + c.eps)
    y = gamma[gid] * xhat + beta[gid]
    if gated:
        y = y * u
    (y * torch.tensor(c.dy, dtype=torch.float64)).sum().backward()
    dx, dgamma, dbeta, du = G.backward(c.dy, c.x, c.group_id, c.gamma, c.beta, c.eps, c.gate)
    assert np.allclose(dx, x.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dgamma, gamma.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dbeta, beta.grad.numpy(), rtol=1e-10, atol=1e-12)
    if gated:
        assert np.allclose(du, u.grad.numpy(), rtol=1e-10, atol=1e-12)
    else:
        assert du is None


def test_backward_equals_central_differences():
    c = small(True, n=5, d=6, groups=2)
    dy = c.dy.astype(np.float64)

    def loss(x, gamma, beta, u):
        return float((G.forward(x, c.group_id, gamma, beta, c.eps, u)[0] * dy).sum())

    base = [c.x.astype(np.float64), c.gamma.astype(np.float64), c.beta.astype(np.float64), c.gate.astype(np.float64)]
    dx, dgamma, dbeta, du = G.backward(c.dy, c.x, c.group_id, c.gamma, c.beta, c.eps, c.gate)
    h = 1e-6
    for which, grad in enumerate((dx, dgamma, dbeta, du)):
        num = np.zeros_like(grad)
        for idx in np.ndindex(*grad.shape):
            hi = [a.copy() for a in base]
            lo = [a.copy() for a in base]
            hi[which][idx] += h
            lo[which][idx] -= h
            num[idx] = (loss(*hi) - loss(*lo)) / (2 * h)
        assert np.allclose(grad, num, rtol=1e-6, atol=1e-8)


def test_unit_parameters_give_zero_mean_unit_variance_tokens():
    c = small(False, n=9, d=64)
    y, _, _ = G.forward(c.x, c.group_id, np.ones_like(c.gamma), np.zeros_like(c.beta), 0.0)
    assert np.allclose(y.mean(axis=1), 0.0, atol=1e-13) and np.allclose((y * y).mean(axis=1), 1.0, rtol=1e-12)


def test_a_token_is_invariant_to_shift_and_positive_scale_of_its_features():
    c = small(False, n=7, d=32)
    y0, _, _ = G.forward(c.x, c.group_id, c.gamma, c.beta, 0.0)
    y1, _, _ = G.forward(3.5 * c.x.astype(np.float64) - 11.0, c.group_id, c.gamma, c.beta, 0.0)
    assert np.allclose(y0, y1, rtol=1e-11, atol=1e-12)


def test_tokens_are_independent_and_only_the_group_selects_the_parameters():
    c = small(True)
    y, _, _ = G.forward(c.x, c.group_id, c.gamma, c.beta, c.eps, c.gate)
    perm = np.arange(c.x.shape[0])[::-1].copy()
    yp, _, _ = G.forward(c.x[perm], c.group_id[perm], c.gamma, c.beta, c.eps, c.gate[perm])
    assert np.array_equal(yp, y[perm])
    # renaming the groups together with their parameter rows changes nothing; changing a token's group does
    ren = np.array([2, 0, 1])
    inv = np.argsort(ren)
    yr, _, _ = G.forward(c.x, ren[c.group_id], c.gamma[inv], c.beta[inv], c.eps, c.gate)
    assert np.array_equal(yr, y)
    other = (c.group_id + 1) % 3
    yo, _, _ = G.forward(c.x, other, c.gamma, c.beta, c.eps, c.gate)
    assert not np.allclose(yo, y)


def test_parameter_gradients_collect_only_their_own_group():
    c = small(False)
    dx, dgamma, dbeta, _ = G.backward(c.dy, c.x, c.group_id, c.gamma, c.beta, c.eps)
    for g in range(3):
        rows = c.group_id == g
        assert np.allclose(dbeta[g], c.dy[rows].astype(np.float64).sum(axis=0), rtol=1e-12, atol=1e-12)
    # with eps = 0 the gradient of a normalised token is orthogonal to the constant vector and to the centred token
    dx0 = G.backward(c.dy, c.x, c.group_id, c.gamma, c.beta, 0.0)[0]
    xc = c.x.astype(np.float64) - c.x.astype(np.float64).mean(axis=1, keepdims=True)
    assert np.allclose(dx0.sum(axis=1), 0.0, atol=1e-10) and np.allclose((dx0 * xc).sum(axis=1), 0.0, atol=1e-9)
    assert np.allclose(dx.sum(axis=1), 0.0, atol=1e-10)
