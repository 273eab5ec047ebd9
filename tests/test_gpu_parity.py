"""GPU parity: the HIP library, called through the C ABI, against the float64 oracle on the same
seeded bits, element by element.  Tolerances: |gpu - ref| <= atol + rtol*|ref| with atol = rtol =
2e-2 for the bf16 path and 1e-4 for the fp32 debug path."""
import numpy as np
import pytest
import torch

from paper_2602_11235_amd import hta, inputs
from tests.hta_testlib import check_case, device_batch, host, pick_users, say, to_torch

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
                                      (6, 1, 128)])
def test_bf16_edge_cases_forward(layer, Hq, Hkv, d):
    c = custom(f"bf16_edges_{Hq}_{Hkv}_{d}", layer, EDGE_HIST, EDGE_TGTS, Hq, Hkv, d, "bf16")
    check_case(c, with_bwd=False)


def test_c2_bf16_forward_full_batch():
    check_case(inputs.make_case(inputs.CONFIGS["C2"], with_dout=False), with_bwd=False)


def test_c3_bf16_forward_sampled_users():
    c = inputs.make_case(inputs.CONFIGS["C3"], with_dout=False)
    check_case(c, with_bwd=False, users=pick_users(c, 4))


def test_bf16_large_logits_online_softmax():
    # logits spread over hundreds of units: exercises the running-max rescale across tiles
    c = custom("bf16_large_logits", FULL, [300, 70], [5, 40], 4, 1, 64, "bf16", std=3.0)
    check_case(c, with_bwd=False)


# ------------------------------------------------------------------------------ bf16 backward
@pytest.mark.parametrize("layer", [FULL, TARGET])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 64), (4, 4, 64), (3, 1, 64), (16, 2, 128), (4, 2, 32)])
def test_bf16_edge_cases_backward(layer, Hq, Hkv, d):
    c = custom(f"bf16_bwd_edges_{Hq}_{Hkv}_{d}", layer, EDGE_HIST, EDGE_TGTS, Hq, Hkv, d, "bf16")
    check_case(c, with_bwd=True)


def test_c2_bf16_backward_full_batch():
    check_case(inputs.make_case(inputs.CONFIGS["C2"]), with_bwd=True)


def test_c3_bf16_forward_backward_sampled_users():
    c = inputs.make_case(inputs.CONFIGS["C3"])
    check_case(c, with_bwd=True, users=pick_users(c, 2))
