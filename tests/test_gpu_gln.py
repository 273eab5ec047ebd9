"""GPU parity of the fused group layer normalization (forward, backward, gated and plain) against the float64
oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import gln_oracle as G
from paper_2602_11235_amd import gln, hta, inputs
from hta_testlib import say

pytestmark = pytest.mark.gpu

# |gpu - ref| <= ATOL + RTOL |ref| per element.  y, dx, dgate are computed in float32 and rounded once to the
# storage type (bf16: 2^-9 relative); the statistics and the parameter gradients are float32 in both cases.
TOL = {"bf16": (2e-2, 2e-2), "fp32": (1e-4, 1e-4)}
TOL_F32 = (1e-4, 1e-4)


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def close(name, got, ref, tol):
    atol, rtol = tol
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    err = np.abs(got - ref)
    bad = err > atol + rtol * np.abs(ref)
    assert not bad.any(), (f"{name}: {int(bad.sum())} of {bad.size} elements off, max abs err {err.max():.3e} at "
                           f"{np.unravel_index(err.argmax(), err.shape)}")


def run_gpu(c: inputs.GlnCase, group_id=None):
    gid = dev(c.group_id if group_id is None else group_id)
    x, dy = dev(c.x, c.dtype), dev(c.dy, c.dtype)
    u = None if c.gate is None else dev(c.gate, c.dtype)
    gamma, beta = dev(c.gamma), dev(c.beta)
    y, mean, rstd = gln.mtfm_gln_fwd(x, gid, gamma, beta, c.eps, gate=u)
    dx, dgamma, dbeta, du = gln.mtfm_gln_bwd(dy, x, gid, gamma, beta, mean, rstd, gate=u)
    torch.cuda.synchronize()
    return dict(y=host(y), mean=host(mean), rstd=host(rstd), dx=host(dx), dgamma=host(dgamma), dbeta=host(dbeta),
                du=None if du is None else host(du))


def check_case(c: inputs.GlnCase, group_id=None):
    got = run_gpu(c, group_id)
    gid = c.group_id if group_id is None else np.clip(group_id, 0, c.gamma.shape[0] - 1)
    y, mean, rstd = G.forward(c.x, gid, c.gamma, c.beta, c.eps, c.gate)
    dx, dgamma, dbeta, du = G.backward(c.dy, c.x, gid, c.gamma, c.beta, c.eps, c.gate)
    tol = TOL[c.dtype]
    close("y", got["y"], y, tol)
    close("mean", got["mean"], mean, TOL_F32)
    close("rstd", got["rstd"], rstd, TOL_F32)
    close("dx", got["dx"], dx, tol)
    close("dgamma", got["dgamma"], dgamma, TOL_F32)
    close("dbeta", got["dbeta"], dbeta, TOL_F32)
    if c.gate is not None:
        close("dgate", got["du"], du, tol)
    else:
        assert got["du"] is None
    return got


SHAPES = [
    # n_tokens, d_model, n_groups, dtype, gated
    (1000, 512, 8, "bf16", True),     # the model width of the headline workload: one 512-feature chunk per token
    (1000, 512, 8, "bf16", False),
    (20011, 512, 8, "bf16", True),    # more tokens than one pass of the persistent grid, odd count
    (777, 64, 3, "bf16", True),       # a row narrower than the wave's chunk: most lanes idle
    (513, 1024, 4, "bf16", True),     # two chunks per token
    (300, 1536, 5, "bf16", False),    # three
    (257, 2048, 4, "bf16", True),     # four: the widest row
    (400, 520, 3, "bf16", True),      # ragged last chunk
    (1000, 512, 8, "fp32", True),
    (333, 200, 5, "fp32", False),
    (9000, 1024, 8, "fp32", True),    # the full LDS table (8 x 1024), several passes of the grid
    (300, 2048, 4, "fp32", True),     # the widest row in float32 (the instantiation with the largest register need)
    (260, 1536, 5, "fp32", False),
    (1, 8, 1, "fp32", False),         # the smallest call
]


@pytest.mark.parametrize("n, d, groups, dtype, gated", SHAPES)
def test_forward_and_backward_match_the_oracle(n, d, groups, dtype, gated):
    say(f"[gln] n={n} d={d} groups={groups} {dtype} gated={gated}")
    check_case(inputs.make_gln_case("t", n, d, groups, dtype=dtype, gated=gated, seed=300 + n % 97))


def test_groups_without_tokens_get_zero_parameter_gradients():
    c = inputs.make_gln_case("t", 600, 512, 6, dtype="bf16", gated=True, seed=11)
    c.group_id[c.group_id == 4] = 1
    got = check_case(c)
    assert not got["dgamma"][4].any() and not got["dbeta"][4].any() and got["dgamma"][1].any()


def test_no_tokens_zeroes_the_parameter_gradients():
    say("[gln] n=0")
    gamma = torch.ones(3, 64, device="cuda")
    x = torch.empty(0, 64, device="cuda", dtype=torch.bfloat16)
    gid = torch.empty(0, device="cuda", dtype=torch.int32)
    y, mean, rstd = gln.mtfm_gln_fwd(x, gid, gamma, gamma, 1e-5)
    out = (torch.empty_like(x), torch.full_like(gamma, 7.0), torch.full_like(gamma, 7.0), None)
    dx, dgamma, dbeta, _ = gln.mtfm_gln_bwd(x, x, gid, gamma, gamma, mean, rstd, out=out)
    torch.cuda.synchronize()
    assert y.shape == (0, 64) and not dgamma.any() and not dbeta.any()


def test_group_ids_outside_the_range_act_as_the_nearest_group():
    c = inputs.make_gln_case("t", 500, 512, 4, dtype="bf16", gated=False, seed=12)
    gid = c.group_id.copy()
    gid[::7] = -3
    gid[3::11] = 9
    with pytest.raises(hta.HtaError):
        gln.mtfm_gln_validate_host(torch.from_numpy(gid), 4)
    check_case(c, group_id=gid)


def test_constant_tokens_and_large_offsets():
    say("[gln] degenerate tokens")
    c = inputs.make_gln_case("t", 64, 512, 2, dtype="fp32", gated=False, seed=13)
    c.x[0] = 3.25                    # zero variance: y = beta, rstd = eps^-1/2
    c.x[1] = 0.0
    c.x[2] = c.x[2] * 0.25 + 50.0    # a spread small against the offset
    got = check_case(c)
    assert np.allclose(got["y"][0], c.beta[c.group_id[0]], atol=1e-6)
    assert np.isclose(got["rstd"][1], 1.0 / np.sqrt(c.eps), rtol=1e-5)


def test_forward_keeps_float32_accuracy_when_the_offset_dwarfs_the_spread():
    # spread 1e-3 on an offset of 1000: a mean rounded to float32 would already be off by a few percent of the spread
    c = inputs.make_gln_case("t", 40, 1024, 2, dtype="fp32", gated=True, seed=16)
    c.x[:] = (c.x * 1e-3 + 1000.0).astype(np.float32)
    y, _, _ = gln.mtfm_gln_fwd(dev(c.x), dev(c.group_id), dev(c.gamma), dev(c.beta), 1e-12, gate=dev(c.gate))
    ref, _, _ = G.forward(c.x, c.group_id, c.gamma, c.beta, 1e-12, c.gate)
    close("y", host(y), ref, (1e-4, 1e-4))


def test_results_do_not_depend_on_previous_calls_and_y_dx_are_reproducible():
    c = inputs.make_gln_case("t", 3000, 512, 8, dtype="bf16", gated=True, seed=14)
    a = run_gpu(c)
    small = inputs.make_gln_case("t", 100, 64, 2, dtype="bf16", gated=True, seed=15)
    check_case(small)                # a different shape in between, sharing nothing
    b = run_gpu(c)
    for k in ("y", "mean", "rstd", "dx", "du"):
        assert np.array_equal(a[k], b[k]), k
    close("dgamma again", b["dgamma"], a["dgamma"], (1e-5, 1e-5))


def test_headline_width_at_full_size_on_sampled_tokens():
    """All tokens of the headline workload (B=256, 512..1024 history + 64 targets, d_model = 8 heads x 64): every
    token is independent, so y / dx / dgate are checked on a sample of tokens the oracle computes one by one, the
    statistics on all tokens in closed form, and dgamma / dbeta against the oracle's sum over all tokens."""
    hta_case_tokens = int(inputs.make_case(inputs.CONFIGS["C3"]).total_kv)
    n, d, groups = hta_case_tokens, 512, 8
    say(f"[gln] full size n={n}")
    c = inputs.make_gln_case("full", n, d, groups, dtype="bf16", gated=True, seed=100)
    got = run_gpu(c)
    x64 = c.x.astype(np.float64)
    close("mean", got["mean"], x64.mean(axis=1), TOL_F32)
    close("rstd", got["rstd"], 1.0 / np.sqrt(x64.var(axis=1) + c.eps), TOL_F32)
    pick = np.unique(np.concatenate([np.arange(0, 40), np.arange(n - 40, n),
                                     (inputs.uniform01(inputs.stream_key(5, 1), 0, 1500) * n).astype(np.int64)]))
    y, _, _ = G.forward(c.x[pick], c.group_id[pick], c.gamma, c.beta, c.eps, c.gate[pick])
    dx, _, _, du = G.backward(c.dy[pick], c.x[pick], c.group_id[pick], c.gamma, c.beta, c.eps, c.gate[pick])
    close("y", got["y"][pick], y, TOL["bf16"])
    close("dx", got["dx"][pick], dx, TOL["bf16"])
    close("dgate", got["du"][pick], du, TOL["bf16"])
    _, dgamma, dbeta, _ = G.backward(c.dy, c.x, c.group_id, c.gamma, c.beta, c.eps, c.gate)
    # sums of ~27 000 float32 terms of magnitude ~1 per element: relative to the root-sum-square of the terms
    scale = np.sqrt(n / groups)
    assert np.abs(got["dgamma"] - dgamma).max() <= 1e-4 * scale and np.abs(got["dbeta"] - dbeta).max() <= 1e-4 * scale
    close("dgamma", got["dgamma"], dgamma, (1e-3, 1e-3))
    close("dbeta", got["dbeta"], dbeta, (1e-3, 1e-3))
