"""Pins for the oracle's pointwise reading of phi2 (out_i = norm * sum over visible j of silu(scale <q_i, k_j>) v_j):
a dense brute force with the library SiLU and autograd, closed forms, central differences, and the properties a
non-normalised pointwise weight has that a softmax does not.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import hta_oracle as O
from paper_2602_11235_amd import inputs

FULL, TARGET = inputs.LAYER_FULL, inputs.LAYER_TARGET
NORM = 1.0 / 37.0


def small_case(layer, rt=False, seed=5):
    kw = dict(rt_len=[3, 0, 4]) if rt else {}
    return inputs.make_case(inputs.custom_config("pw", layer, [5, 0, 9], [3, 2, 0], 4, 2, 8, dtype="fp32", std=0.7,
                                                 seed=seed, **kw))


def dense_mask(L, R, T, ts):
    kinds = ["H"] * L + ["R"] * R + ["T"] * T
    N = L + R + T
    M = np.zeros((N, N), dtype=bool)
    for j, kind in enumerate(kinds):
        for i in range(N):
            M[i, j] = True if kind == "H" else ((ts[i] > ts[j]) or i == j) if kind == "R" else i == j
    return M


def torch_dense(case, layer, norm):
    cfg = case.cfg
    r = cfg.Hq // cfg.Hkv
    q = torch.tensor(case.q, dtype=torch.float64, requires_grad=True)
    k = torch.tensor(case.k, dtype=torch.float64, requires_grad=True)
    v = torch.tensor(case.v, dtype=torch.float64, requires_grad=True)
    out = torch.zeros(case.q.shape, dtype=torch.float64)
    loss = 0.0
    for b in range(case.batch):
        L, T = int(case.hist_len[b]), int(case.n_targets[b])
        R = 0 if case.rt_len is None else int(case.rt_len[b])
        ks, ke = int(case.kv_offsets[b]), int(case.kv_offsets[b + 1])
        qs, qe = int(case.q_offsets[b]), int(case.q_offsets[b + 1])
        if qe == qs:
            continue
        ts = np.zeros(ke - ks, dtype=np.int64) if case.timestamps is None else case.timestamps[ks:ke]
        M = torch.tensor(dense_mask(L, R, T, ts))
        if layer == TARGET:
            M = M[L + R:]
        kb = k[ks:ke].repeat_interleave(r, dim=1)
        vb = v[ks:ke].repeat_interleave(r, dim=1)
        S = case.scale * torch.einsum("ihd,jhd->hij", q[qs:qe], kb)
        A = norm * torch.nn.functional.silu(S) * M[None]
        o = torch.einsum("hij,jhd->ihd", A, vb)
        out[qs:qe] = o.detach()
        loss = loss + (o * torch.tensor(case.dout[qs:qe], dtype=torch.float64)).sum()
    loss.backward()
    return out.numpy(), q.grad.numpy(), k.grad.numpy(), v.grad.numpy()


def run_oracle(case, layer, norm=NORM):
    rt = dict(rt_len=case.rt_len, timestamps=case.timestamps)
    out = O.forward_pointwise(case.q, case.k, case.v, case.q_offsets, case.kv_offsets, case.hist_len, case.n_targets,
                              case.scale, norm, layer, **rt)
    dq, dk, dv = O.backward_pointwise(case.dout, case.q, case.k, case.v, case.q_offsets, case.kv_offsets,
                                      case.hist_len, case.n_targets, case.scale, norm, layer, **rt)
    return out, dq, dk, dv


@pytest.mark.parametrize("layer", [FULL, TARGET])
@pytest.mark.parametrize("rt", [False, True])
def test_dense_brute_force_with_library_silu_and_autograd(layer, rt):
    case = small_case(layer, rt)
    got = run_oracle(case, layer)
    ref = torch_dense(case, layer, NORM)
    for name, g, r in zip(("out", "dq", "dk", "dv"), got, ref):
        assert np.allclose(g, r, rtol=1e-11, atol=1e-13), name


def test_one_history_key_closed_form():
    # one user, one history token, one target: the target row sees the history key and its own key
    case = inputs.make_case(inputs.custom_config("one", TARGET, [1], [1], 1, 1, 4, dtype="fp32", std=1.0, seed=3))
    out = O.forward_pointwise(case.q, case.k, case.v, case.q_offsets, case.kv_offsets, case.hist_len, case.n_targets,
                              0.5, 0.25, TARGET)
    silu = lambda x: x / (1.0 + math.exp(-x))
    q = case.q[0, 0].astype(np.float64)
    expect = sum(0.25 * silu(0.5 * float(q @ case.k[j, 0].astype(np.float64))) * case.v[j, 0].astype(np.float64)
                 for j in (0, 1))
    assert np.allclose(out[0, 0], expect, rtol=1e-13, atol=1e-15)


def test_zero_queries_give_zero_output_and_half_slope():
    # silu(0) = 0 and silu'(0) = 1/2: out = 0, dq_i = scale * norm / 2 * sum_j <dout_i, v_j> k_j, dv = 0
    case = small_case(FULL)
    case.q[:] = 0.0
    out, dq, dk, dv = run_oracle(case, FULL)
    assert not out.any() and not dv.any() and not dk.any()
    b, row, h = 0, 6, 1            # a target row of user 0 (5 history tokens): sees keys 0..4 and its own
    g = h // 2
    doi = case.dout[row, h].astype(np.float64)
    expect = np.zeros(8)
    for j in list(range(5)) + [row]:
        expect += case.scale * NORM * 0.5 * float(doi @ case.v[j, g].astype(np.float64)) * case.k[j, g].astype(np.float64)
    assert np.allclose(dq[row, h], expect, rtol=1e-12, atol=1e-15)


def test_output_is_linear_in_v_and_in_norm_and_rows_do_not_sum_to_one():
    case = small_case(FULL)
    out, *_ = run_oracle(case, FULL)
    out2 = O.forward_pointwise(case.q, case.k, 3.0 * case.v.astype(np.float64), case.q_offsets, case.kv_offsets,
                               case.hist_len, case.n_targets, case.scale, NORM, FULL)
    assert np.allclose(out2, 3.0 * out, rtol=1e-13)
    out3 = O.forward_pointwise(case.q, case.k, case.v, case.q_offsets, case.kv_offsets, case.hist_len, case.n_targets,
                               case.scale, 2.0 * NORM, FULL)
    assert np.allclose(out3, 2.0 * out, rtol=1e-13)
    # with v = 1 the output is the sum of the weights, which is not normalised and can be negative (silu >= -0.279)
    ones = np.ones_like(case.v)
    w = O.forward_pointwise(case.q, case.k, ones, case.q_offsets, case.kv_offsets, case.hist_len, case.n_targets,
                            case.scale, 1.0, FULL)[:, :, 0]
    assert not np.allclose(w, 1.0) and w.min() > -0.2785 * 13


def test_keys_do_not_compete():
    """Unlike a softmax, changing one key changes only that key's term: the outputs of rows that do not see the key
    stay put, and for rows that do the difference is exactly the difference of that one term."""
    case = small_case(FULL)
    out, *_ = run_oracle(case, FULL)
    k2 = case.k.astype(np.float64).copy()
    k2[2, 0] += 0.37                # history key 2 of user 0, kv head 0 (query heads 0, 1)
    out2 = O.forward_pointwise(case.q, k2, case.v, case.q_offsets, case.kv_offsets, case.hist_len, case.n_targets,
                               case.scale, NORM, FULL)
    assert np.array_equal(out2[8:], out[8:]) and np.array_equal(out2[:, 2:], out[:, 2:])
    silu = lambda x: x / (1.0 + np.exp(-x))
    q = case.q[3, 1].astype(np.float64)
    delta = NORM * (silu(case.scale * q @ k2[2, 0]) - silu(case.scale * q @ case.k[2, 0].astype(np.float64)))
    assert np.allclose(out2[3, 1] - out[3, 1], delta * case.v[2, 0].astype(np.float64), rtol=1e-9, atol=1e-15)


def test_target_layer_is_the_row_slice_of_the_full_layer():
    full = small_case(FULL, rt=True)
    tgt = small_case(TARGET, rt=True)
    out_f, *_ = run_oracle(full, FULL)
    out_t, *_ = run_oracle(tgt, TARGET)
    rows = np.concatenate([np.arange(full.kv_offsets[b] + full.hist_len[b] + full.rt_len[b], full.kv_offsets[b + 1])
                           for b in range(full.batch)])
    # the two cases draw their queries from the same stream but with different row counts: rebuild the slice
    q_t = full.q[rows]
    out_t2 = O.forward_pointwise(q_t, full.k, full.v, tgt.q_offsets, full.kv_offsets, full.hist_len, full.n_targets,
                                 full.scale, NORM, TARGET, rt_len=full.rt_len, timestamps=full.timestamps)
    assert np.array_equal(out_t2, out_f[rows]) and out_t.shape == out_t2.shape


def test_backward_equals_central_differences():
    case = inputs.make_case(inputs.custom_config("fd", FULL, [3, 0], [2, 1], 2, 1, 4, dtype="fp32", std=0.8, seed=8))
    out, dq, dk, dv = run_oracle(case, FULL)
    dout = case.dout.astype(np.float64)
    base = [case.q.astype(np.float64), case.k.astype(np.float64), case.v.astype(np.float64)]

    def loss(q, k, v):
        return float((O.forward_pointwise(q, k, v, case.q_offsets, case.kv_offsets, case.hist_len, case.n_targets,
                                          case.scale, NORM, FULL) * dout).sum())

    h = 1e-6
    for which, grad in enumerate((dq, dk, dv)):
        num = np.zeros_like(grad)
        for idx in np.ndindex(*grad.shape):
            hi = [a.copy() for a in base]
            lo = [a.copy() for a in base]
            hi[which][idx] += h
            lo[which][idx] -= h
            num[idx] = (loss(*hi) - loss(*lo)) / (2 * h)
        assert np.allclose(grad, num, rtol=1e-6, atol=1e-9)


def test_planted_mistakes_are_caught():
    """What the pins above would see if the derivative, the normaliser or the mask were wrong (mistakes planted in
    re-derivations here, on the CPU, never in the oracle)."""
    case = small_case(FULL)
    out, dq, dk, dv = run_oracle(case, FULL)
    ref_out, ref_dq, *_ = torch_dense(case, FULL, NORM)
    # sigmoid instead of silu' in the backward pass
    x = 0.3
    sg = 1 / (1 + math.exp(-x))
    assert abs(sg - sg * (1 + x * (1 - sg))) > 1e-2
    # a forgotten norm scales everything by 37
    assert not np.allclose(out * 37.0, ref_out)
    # a causal mask instead of the hybrid mask changes target rows (they would see earlier targets)
    L, T = 5, 3
    causal = np.tril(np.ones((L + T, L + T), dtype=bool))
    assert (causal != dense_mask(L, 0, T, np.zeros(L + T))).any()
