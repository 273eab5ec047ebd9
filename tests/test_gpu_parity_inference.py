"""GPU parity at inference shapes: forward only, a handful of requests, so the library splits the keys of every
(user, kv head) group over several workgroups and merges the partial softmax results.  Same float64 oracle, same
tolerances (atol = rtol = 2e-2 for bf16) as the training shapes."""
import numpy as np
import pytest
import torch

from paper_2602_11235_amd import hta, inputs
from tests.hta_testlib import check_case, device_batch, host

pytestmark = pytest.mark.gpu
FULL, TARGET = inputs.LAYER_FULL, inputs.LAYER_TARGET


def is_split(case) -> bool:
    """The forward workspace holds partial results only when the keys are split."""
    b = device_batch(case)
    plain = 256 + 256 * ((4 * case.batch + 255) // 256)
    if case.rt_len is not None:
        plain += 256 * ((4 * case.total_q + 255) // 256)
    return b.fwd_workspace_bytes > plain


@pytest.mark.parametrize("name", ["I1", "I2", "I3", "I2_RT"])
def test_inference_workloads_forward(name):
    c = inputs.make_case(inputs.CONFIGS[name])
    assert is_split(c)
    check_case(c, with_bwd=False)


# Histories around the tile and split boundaries next to long ones (the split count follows the longest): no history
# at all (every split is empty, the own key alone), less than one tile, exactly two tiles, one key more than a tile.
EDGE_HIST = [2048, 0, 1, 63, 128, 65, 1000, 64]
EDGE_TGTS = [16, 5, 1, 33, 64, 2, 70, 0]


@pytest.mark.parametrize("layer", [TARGET, FULL])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 64), (2, 2, 64), (3, 1, 64), (16, 2, 128), (4, 2, 32), (6, 1, 128)])
def test_split_forward_edge_cases(layer, Hq, Hkv, d):
    hist, tg = (EDGE_HIST, EDGE_TGTS) if layer == TARGET else ([600, 63, 0], [16, 33, 5])  # full layer: few row tiles
    c = inputs.make_case(inputs.custom_config(f"split_{Hq}_{Hkv}_{d}", layer, hist, tg, Hq, Hkv, d, seed=31))
    assert is_split(c)
    check_case(c, with_bwd=(layer == FULL))   # the backward pass reads the merged out / lse


@pytest.mark.parametrize("layer", [TARGET, FULL])
def test_split_forward_with_real_time_tokens(layer):
    c = inputs.make_case(inputs.custom_config("split_rt", layer, [1500, 0, 63, 700], [16, 5, 33, 2], 8, 2, 64, seed=32,
                                              rt_len=[70, 5, 0, 130]))
    assert is_split(c)
    check_case(c, with_bwd=False)


def test_split_and_unsplit_forward_agree():
    """The same request alone (keys split) and as one of 300 copies (no split): two different summation orders of
    the same softmax, equal up to the bf16 rounding of the output."""
    one = inputs.make_case(inputs.custom_config("one", TARGET, [1800], [40], 8, 2, 64, seed=33))
    many = inputs.take_users(one, [0] * 300)
    assert is_split(one) and not is_split(many)
    a_out, a_lse = device_batch(one).forward()
    b_out, b_lse = device_batch(many).forward()
    torch.cuda.synchronize()
    n = one.total_q
    assert np.allclose(host(a_out), host(b_out)[:n], rtol=2e-2, atol=2e-3)
    # (the row sums are formed from bf16-rounded weights, so lse carries ~1e-3 of rounding in either order)
    assert np.allclose(host(a_lse), host(b_lse)[:, :n], rtol=2e-3, atol=2e-3)
