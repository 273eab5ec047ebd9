"""GPU parity for samples with real-time tokens (mask rule 2 of Section 3.2.2): the HIP library, called through the
C ABI (mtfm_hta_fwd_rt / mtfm_hta_bwd_rt), against the float64 oracle on the same seeded bits, element by element.
Tolerances as for the plain hybrid mask: atol = rtol = 2e-2 (bf16), 1e-4 (fp32)."""
import numpy as np
import pytest
import torch

from paper_2602_11235_amd import inputs
from tests.hta_testlib import check_case, device_batch, host, pick_users, to_torch

pytestmark = pytest.mark.gpu
FULL, TARGET = inputs.LAYER_FULL, inputs.LAYER_TARGET

# per user: history, real-time, targets.  Empty segments of every kind, real-time segments that straddle the 32-key
# sub-tiles, the 64-key tiles and the 128-key dK/dV tiles together with the end of the history, a real-time segment
# without history, users with nothing at all.
EDGE_HIST = [0, 1, 63, 64, 65, 130, 200, 0, 257, 96, 0, 40]
EDGE_RT = [5, 0, 3, 70, 31, 2, 140, 0, 33, 32, 64, 0]
EDGE_TGTS = [3, 0, 70, 1, 33, 2, 64, 0, 129, 0, 1, 7]


def custom(name, layer, Hq, Hkv, d, dtype, seed=78):
    std = 0.5 if dtype == "fp32" else 0.3
    return inputs.make_case(inputs.custom_config(name, layer, EDGE_HIST, EDGE_TGTS, Hq, Hkv, d, dtype=dtype, std=std,
                                                 seed=seed, rt_len=EDGE_RT))


@pytest.mark.parametrize("layer", [FULL, TARGET])
def test_fp32_realtime_edge_cases(layer):
    check_case(custom("fp32_rt_edges", layer, 6, 2, 24, "fp32"), with_bwd=True)


@pytest.mark.parametrize("layer", [FULL, TARGET])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 64), (4, 4, 64), (3, 1, 64), (16, 2, 128), (16, 1, 64), (4, 2, 32), (6, 1, 128),
                                      (4, 1, 16)])
def test_bf16_realtime_edge_cases(layer, Hq, Hkv, d):
    check_case(custom(f"bf16_rt_edges_{Hq}_{Hkv}_{d}", layer, Hq, Hkv, d, "bf16"), with_bwd=True)


def test_c2_rt_full_batch():
    check_case(inputs.make_case(inputs.CONFIGS["C2_RT"]), with_bwd=True)


def test_c3_rt_sampled_users():
    c = inputs.make_case(inputs.CONFIGS["C3_RT"])
    check_case(c, with_bwd=True, users=pick_users(c, 12))


def test_c4_rt_target_layer_sampled_users():
    c = inputs.make_case(inputs.CONFIGS["C4_RT"])
    check_case(c, with_bwd=True, users=sorted(set(pick_users(c, 12)) | {0, 63, 127}))


def test_zero_realtime_tokens_equal_the_plain_entry_points_bitwise():
    """rt_len = 0 for every user: the real-time entry points must return exactly what the plain ones return."""
    plain = inputs.make_case(inputs.custom_config("rt0", FULL, [200, 65, 0, 130], [7, 33, 2, 64], 8, 2, 64, seed=5))
    with_rt = inputs.make_case(inputs.custom_config("rt0", FULL, [200, 65, 0, 130], [7, 33, 2, 64], 8, 2, 64, seed=5,
                                                    rt_len=[0, 0, 0, 0]))
    assert np.array_equal(plain.q, with_rt.q) and np.array_equal(plain.kv_offsets, with_rt.kv_offsets)
    res = []
    for c in (plain, with_rt):
        b = device_batch(c)
        out, lse = b.forward()
        dq, dk, dv = b.backward(to_torch(c.dout, "bf16"))
        torch.cuda.synchronize()
        res.append([host(t) for t in (out, lse, dq, dk, dv)])
    for a, b in zip(*res):
        assert np.array_equal(a, b)
