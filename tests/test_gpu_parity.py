"""GPU parity: the HIP library, called through the C ABI, against the float64 oracle on the same
seeded bits, element by element.  Tolerances: |gpu - ref| <= atol + rtol*|ref| with atol = rtol =
2e-2 for the bf16 path and 1e-4 for the fp32 debug path."""
import functools

import numpy as np
import pytest
import torch

from paper_2602_11235_amd import hta, inputs
from tests.hta_testlib import (check_case, close_on_tensor_scale, compare_with_oracle, device_batch, host, pick_users,
                               run_library, say, to_torch)

pytestmark = pytest.mark.gpu
FULL, TARGET = inputs.LAYER_FULL, inputs.LAYER_TARGET


def custom(name, layer, hist, tgts, Hq, Hkv, d, dtype, seed=77, std=None):
    std = std if std is not None else (0.5 if dtype == "fp32" else 0.3)
    return inputs.make_case(inputs.custom_config(name, layer, hist, tgts, Hq, Hkv, d, dtype=dtype, std=std, seed=seed))


# ------------------------------------------------------------------------------ fp32 debug path
def test_c1_fp32_forward_and_backward():
    check_case(inputs.make_case(inputs.CONFIGS["C1"]), with_bwd=True)


@pytest.mark.parametrize("layer", [FULL, TARGET])
def test_fp32_edge_cases(layer):
    # empty history, no targets, empty user, lengths around the 64-lane stride, odd head_dim
    c = custom("fp32_edges", layer, [0, 5, 0, 64, 65, 130, 1], [3, 0, 0, 1, 2, 70, 1], 6, 2, 24, "fp32")
    check_case(c, with_bwd=True)


# ------------------------------------------------------------------------------ bf16 MFMA path
EDGE_HIST = [0, 1, 63, 64, 65, 130, 200, 0, 257]
EDGE_TGTS = [3, 0, 70, 1, 33, 2, 64, 0, 129]


@pytest.mark.parametrize("layer", [FULL, TARGET])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 64), (4, 4, 64), (3, 1, 64), (16, 2, 128), (16, 1, 64), (4, 2, 32),
                                      (6, 1, 128), (4, 1, 16), (8, 2, 16)])
def test_bf16_edge_cases_forward(layer, Hq, Hkv, d):
    c = custom(f"bf16_edges_{Hq}_{Hkv}_{d}", layer, EDGE_HIST, EDGE_TGTS, Hq, Hkv, d, "bf16")
    check_case(c, with_bwd=False)


def test_c2_bf16_forward_full_batch():
    check_case(inputs.make_case(inputs.CONFIGS["C2"], with_dout=False), with_bwd=False)


def test_bf16_large_logits_online_softmax():
    # logits spread over hundreds of units: exercises the running-max rescale across tiles, and the absolute accuracy
    # of the scores in front of every exponential (a score of 400 rounded to 2^-9 relative would be off by almost a
    # unit: the scale has to be applied in float32, after the products).  Forward only: with weights this peaked the
    # gradient is a difference of large terms that the bf16 rounding of `out` alone moves by more than the tolerance.
    c = custom("bf16_large_logits", FULL, [300, 70], [5, 40], 4, 1, 64, "bf16", std=3.0)
    check_case(c, with_bwd=False)


@pytest.mark.parametrize("std", [1.0, 1.5])
def test_bf16_moderately_large_logits_backward(std):
    # logits of tens of units: the recomputed weights of both backward passes need scores accurate to ~1e-2
    c = custom(f"bf16_logits_std{std}", FULL, [300, 70], [5, 40], 4, 1, 64, "bf16", std=std)
    check_case(c, with_bwd=True)


def test_bf16_large_logits_backward_on_tensor_scale():
    # The same peaked regime as the forward test above (std = 3: logits of hundreds of units, weights that are 0 or 1
    # to bf16 accuracy).  A gradient element is then p (dp - delta) with dp ~ delta: a difference that the bf16 rounding
    # of `out` (inside delta) and of the weights moves by more than 2 % of a small element, so the element-wise
    # relative bound cannot hold; what must hold is that no error exceeds 2 % of the tensor's largest element.
    c = custom("bf16_large_logits_bwd", FULL, [300, 70], [5, 40], 4, 1, 64, "bf16", std=3.0)
    check_case(c, with_bwd=True, compare=close_on_tensor_scale)


# ------------------------------------------------------------------------------ bf16 backward
@pytest.mark.parametrize("layer", [FULL, TARGET])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 64), (4, 4, 64), (3, 1, 64), (16, 2, 128), (4, 2, 32), (4, 1, 16),
                                      (8, 2, 16)])
def test_bf16_edge_cases_backward(layer, Hq, Hkv, d):
    c = custom(f"bf16_bwd_edges_{Hq}_{Hkv}_{d}", layer, EDGE_HIST, EDGE_TGTS, Hq, Hkv, d, "bf16")
    check_case(c, with_bwd=True)


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (4, 4), (3, 1), (16, 4)])
def test_bf16_few_query_rows_against_long_histories(Hq, Hkv):
    # A target-only layer with at most 128 candidates per user against histories of hundreds of keys: the dK/dV pass
    # keeps all query rows of a (user, kv head) in LDS and walks the keys (the launch is chosen from the bounds of the
    # batch).  Histories around the 256-key stride of a workgroup pass, users without candidates, without history,
    # without both; odd and even numbers of (head, row block) units, up to the sixteen the kernel holds.
    # (That launch also wants a (user, kv head) item for every compute unit: 135 users; with one kv head the batch has
    # too few and stays with the kernel that streams the rows.)
    hist, tgts = [600, 0, 513, 1030, 64, 257, 255, 256, 0] * 15, [128, 5, 0, 33, 70, 1, 96, 2, 0] * 15
    c = custom(f"bf16_few_rows_{Hq}_{Hkv}", TARGET, hist, tgts, Hq, Hkv, 64, "bf16")
    check_case(c, with_bwd=True)


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("bf16", 16), ("fp32", 24)])
def test_target_layer_without_any_candidate(dtype, d):
    # no user of the batch has a target: there is no query row (empty row-shaped tensors, null pointers at the
    # boundary), the forward call has nothing to do and the backward call still has to write dk = dv = 0
    c = custom(f"no_candidates_{dtype}_{d}", TARGET, [300, 0, 64, 129], [0, 0, 0, 0], 8, 2, d, dtype)
    assert c.total_q == 0 and c.total_kv == 493
    b = device_batch(c)
    b.forward()
    b.prepare_backward()
    b.dk.fill_(float("nan"))
    b.dv.fill_(float("nan"))
    dq, dk, dv = b.backward(to_torch(c.dout, dtype))
    torch.cuda.synchronize()
    assert dq.shape[0] == 0
    assert torch.equal(dk, torch.zeros_like(dk)) and torch.equal(dv, torch.zeros_like(dv))


def test_c2_bf16_backward_full_batch():
    check_case(inputs.make_case(inputs.CONFIGS["C2"]), with_bwd=True)


def test_c3_bf16_forward_backward_full_batch():
    # the graded workload, every user: the persistent dK/dV work queue, the help-another-XCD path and the tail of the
    # schedule all leave their results somewhere in this batch
    check_case(inputs.make_case(inputs.CONFIGS["C3"]), with_bwd=True)


# ------------------------------------------------------------------------------ remaining workloads
def test_c4_target_layer_forward_backward_sampled_users():
    c = inputs.make_case(inputs.CONFIGS["C4"])
    users = sorted(set(pick_users(c, 12)) | {0, 255, 511})   # lengths are fixed: first, middle, last + 12 random users
    check_case(c, with_bwd=True, users=users)


@functools.lru_cache(maxsize=1)
def c5_on_the_gpu():
    """C5 once for the two tests below: the case and the library's results (kept on the device)."""
    c = inputs.make_case(inputs.CONFIGS["C5"])
    return c, run_library(c, with_bwd=True)


def c5_sample(c):
    """Shortest / longest history, fewest / most targets, a median history and 12 seeded random users."""
    median = int(np.argsort(c.hist_len)[c.batch // 2])
    return sorted(set(pick_users(c, 12)) | {median})


def test_c5_long_history_stress_sampled_users():
    c, g = c5_on_the_gpu()
    users = [u for u in c5_sample(c) if c.hist_len[u] < 8192]
    say(f"  users {users}: histories {[int(c.hist_len[u]) for u in users]}, targets {[int(c.n_targets[u]) for u in users]}")
    assert len(users) >= 12
    compare_with_oracle(c, g, True, users=users)


@pytest.mark.parametrize("which", [0, 1])
def test_c5_users_at_the_history_cap(which):
    # about 9 % of the users sit at the cap of 8192 history tokens and carry half of the work; the two of the sample
    # (the longest-history pick is one) are compared on all heads of both kv groups, one user per test.  The oracle
    # runs on the equivalent problem with one K/V copy per query head (see oracle_all): 16 units of work side by side
    # instead of 2 that would each run for minutes.
    c, g = c5_on_the_gpu()
    capped = [u for u in c5_sample(c) if c.hist_len[u] == 8192]
    assert len(capped) >= 2, "the recipe puts about 9 % of the users at the cap"
    u = capped[which]
    say(f"  capped user {u}, {int(c.n_targets[u])} targets")
    compare_with_oracle(c, g, True, users=[u], per_head=True)


def test_many_small_users_take_the_bucketed_schedule():
    # more than 4096 users: the device-side schedule switches from the exact rank sort to cost buckets
    B = 5000
    u = inputs.uniform01(inputs.stream_key(5, 7), 0, 2 * B)
    hist = (u[:B] * 41).astype(np.int32)          # 0 .. 40
    tgts = (u[B:] * 4).astype(np.int32)           # 0 .. 3
    c = custom("many_small_users", FULL, hist, tgts, 4, 2, 32, "bf16")
    check_case(c, with_bwd=True)


def test_results_do_not_depend_on_user_order():
    """The schedule reorders users internally; outputs must be bitwise those of the same users in any batch order."""
    c = custom("order_a", FULL, [300, 10, 700, 64, 129], [5, 9, 0, 33, 2], 8, 2, 64, "bf16")
    perm = [2, 4, 0, 3, 1]
    cp = inputs.take_users(c, perm)
    ba, bb = device_batch(c), device_batch(cp)
    oa, la = ba.forward()
    ob, lb = bb.forward()
    da = ba.backward(to_torch(c.dout, "bf16"))
    db = bb.backward(to_torch(cp.dout, "bf16"))
    torch.cuda.synchronize()
    qrows, kvrows = inputs.user_rows(c.q_offsets, perm), inputs.user_rows(c.kv_offsets, perm)
    assert torch.equal(oa[qrows], ob) and torch.equal(la[:, qrows], lb)
    assert torch.equal(da[0][qrows], db[0]) and torch.equal(da[1][kvrows], db[1]) and torch.equal(da[2][kvrows], db[2])


def test_backward_is_bitwise_reproducible():
    c = inputs.make_case(inputs.CONFIGS["C2"])
    b = device_batch(c)
    b.forward()
    dout = to_torch(c.dout, "bf16")
    first = [t.clone() for t in b.backward(dout)]
    second = b.backward(dout)
    torch.cuda.synchronize()
    for x, y in zip(first, second):
        assert torch.equal(x, y)
