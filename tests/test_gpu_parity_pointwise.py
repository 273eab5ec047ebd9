"""GPU parity of the pointwise variant (weights norm * silu(scale s) instead of a row softmax) against the float64
oracle, element by element through the C ABI.  Tolerances as for the softmax reading: atol = rtol = 2e-2 (bf16, where
the weights and dS are rounded to bf16 before their matrix products), 1e-4 (fp32)."""
import functools

import numpy as np
import pytest
import torch

from oracle import hta_oracle as O
from paper_2602_11235_amd import hta_pw, inputs
from tests.hta_testlib import assert_close, host, pick_users, say, sum_over_group, to_torch

pytestmark = pytest.mark.gpu
FULL, TARGET = inputs.LAYER_FULL, inputs.LAYER_TARGET


def norm_of(case):
    """HSTU divides the weights by the sequence length: the reciprocal of the longest sample of the batch."""
    rt = 0 if case.rt_len is None else case.rt_len
    n = int((case.hist_len + rt + case.n_targets).max()) if case.batch else 1
    return 1.0 / max(n, 1)


def device_batch(case, norm):
    dt = case.cfg.dtype
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to("cuda")
    rt = {}
    if case.rt_len is not None:
        rt = dict(rt_len=dev(case.rt_len), timestamps=dev(case.timestamps),
                  max_rt=int(case.rt_len.max()) if case.batch else 0)
    return hta_pw.PointwiseBatch(to_torch(case.q, dt), to_torch(case.k, dt), to_torch(case.v, dt), dev(case.q_offsets),
                                 dev(case.kv_offsets), dev(case.hist_len), dev(case.n_targets),
                                 int(case.hist_len.max()) if case.batch else 0,
                                 int(case.n_targets.max()) if case.batch else 0, case.scale, norm, case.cfg.layer, **rt)


def close_on_tensor_scale(name, got, ref, dtype):
    """For weights that are not normalised: an element is a sum of terms far larger than itself can be, and the bf16
    rounding of each term (2^-9 relative) is what the error is made of, so the bound is relative to the tensor."""
    rtol = 2e-2 if dtype == "bf16" else 1e-4
    assert np.isfinite(got).all(), f"{name}: non-finite values in GPU result"
    err = np.abs(got - ref).max()
    say(f"    {name}: max abs err {err:.3e}  ref absmax {np.abs(ref).max():.3e}")
    assert err <= rtol * np.abs(ref).max(), f"{name}: max abs err {err:.3e} exceeds {rtol:g} x max|ref|"


def run_gpu(case, norm):
    b = device_batch(case, norm)
    out = b.forward()
    dq, dk, dv = b.backward(to_torch(case.dout, case.cfg.dtype))
    torch.cuda.synchronize()
    return dict(out=out, dq=dq, dk=dk, dv=dv)


def check(case, users=None, norm=None, kv_group=None, compare=assert_close, gpu=None, per_head=False):
    dt = case.cfg.dtype
    norm = norm_of(case) if norm is None else norm
    say(f"  pointwise {case.cfg.name}: layer={case.cfg.layer} B={case.batch} total_q={case.total_q} Hq={case.cfg.Hq} "
        f"Hkv={case.cfg.Hkv} d={case.cfg.head_dim} {dt} norm={norm:.3e}")
    g = gpu if gpu is not None else run_gpu(case, norm)   # kept on the device; the compared rows are taken there
    ref_case, qrows, kvrows = case, None, None
    if users is not None:
        ref_case = inputs.take_users(case, users)
        qrows = torch.from_numpy(inputs.user_rows(case.q_offsets, users)).to("cuda")
        kvrows = torch.from_numpy(inputs.user_rows(case.kv_offsets, users)).to("cuda")
    hs, gs = slice(None), slice(None)
    if kv_group is not None:   # one kv head and its query heads (heads of different kv heads are independent)
        r = case.cfg.Hq // case.cfg.Hkv
        hs, gs = slice(kv_group * r, (kv_group + 1) * r), slice(kv_group, kv_group + 1)
        ref_case = inputs.take_kv_group(ref_case, kv_group)
    # per_head: the oracle on the equivalent problem with one K/V copy per query head (tests/hta_testlib.oracle_all)
    c = inputs.repeat_kv_heads(ref_case) if per_head else ref_case
    rt = dict(rt_len=c.rt_len, timestamps=c.timestamps)
    r_out = O.forward_pointwise(c.q, c.k, c.v, c.q_offsets, c.kv_offsets, c.hist_len, c.n_targets, c.scale, norm,
                                c.cfg.layer, **rt)
    r_dq, r_dk, r_dv = O.backward_pointwise(c.dout, c.q, c.k, c.v, c.q_offsets, c.kv_offsets, c.hist_len, c.n_targets,
                                            c.scale, norm, c.cfg.layer, **rt)
    if per_head:
        r_dk, r_dv = sum_over_group(r_dk, ref_case.cfg.Hkv), sum_over_group(r_dv, ref_case.cfg.Hkv)

    def rows_of(t, rows, heads):
        return host((t if rows is None else t.index_select(0, rows))[:, heads])

    compare("out", rows_of(g["out"], qrows, hs), r_out, dt)
    compare("dq", rows_of(g["dq"], qrows, hs), r_dq, dt)
    compare("dk", rows_of(g["dk"], kvrows, gs), r_dk, dt)
    compare("dv", rows_of(g["dv"], kvrows, gs), r_dv, dt)


# histories around the 32 / 64 / 128-key boundaries, users without history, without targets, with nothing
EDGE_HIST = [0, 1, 63, 64, 65, 130, 200, 0, 257, 96, 0, 40]
EDGE_TGTS = [3, 0, 70, 1, 33, 2, 64, 0, 129, 0, 1, 7]


@pytest.mark.parametrize("layer", [FULL, TARGET])
def test_fp32_edge_cases(layer):
    check(inputs.make_case(inputs.custom_config("pw_fp32", layer, EDGE_HIST, EDGE_TGTS, 6, 2, 24, dtype="fp32", std=0.5,
                                                seed=51)))


@pytest.mark.parametrize("layer", [FULL, TARGET])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 64), (4, 4, 64), (3, 1, 64), (16, 2, 128), (16, 1, 64), (4, 2, 32), (6, 1, 128),
                                      (4, 1, 16)])
def test_bf16_edge_cases(layer, Hq, Hkv, d):
    check(inputs.make_case(inputs.custom_config(f"pw_{Hq}_{Hkv}_{d}", layer, EDGE_HIST, EDGE_TGTS, Hq, Hkv, d, seed=52)))


# with real-time tokens (mask rule 2): the segment lengths of the softmax edge tests
RT_HIST = [0, 1, 63, 64, 65, 130, 200, 0, 257, 96, 0, 40]
RT_RT = [5, 0, 3, 70, 31, 2, 140, 0, 33, 32, 64, 0]
RT_TGTS = [3, 0, 70, 1, 33, 2, 64, 0, 129, 0, 1, 7]


@pytest.mark.parametrize("layer", [FULL, TARGET])
def test_fp32_realtime_edge_cases(layer):
    check(inputs.make_case(inputs.custom_config("pw_rt_fp32", layer, RT_HIST, RT_TGTS, 6, 2, 24, dtype="fp32", std=0.5,
                                                seed=54, rt_len=RT_RT)))


@pytest.mark.parametrize("layer", [FULL, TARGET])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 64), (3, 1, 64), (16, 2, 128), (4, 2, 32), (4, 1, 16)])
def test_bf16_realtime_edge_cases(layer, Hq, Hkv, d):
    check(inputs.make_case(inputs.custom_config(f"pw_rt_{Hq}_{Hkv}_{d}", layer, RT_HIST, RT_TGTS, Hq, Hkv, d, seed=55,
                                                rt_len=RT_RT)))


def test_c2_rt_whole_and_c3_rt_sampled_users():
    check(inputs.make_case(inputs.CONFIGS["C2_RT"]))
    c = inputs.make_case(inputs.CONFIGS["C3_RT"])
    check(c, users=pick_users(c, 12))


def test_c1_and_c2_whole():
    check(inputs.make_case(inputs.CONFIGS["C1"]))
    check(inputs.make_case(inputs.CONFIGS["C2"]))


def test_c3_sampled_users():
    c = inputs.make_case(inputs.CONFIGS["C3"])
    check(c, users=pick_users(c, 12))


def test_c4_target_layer_sampled_users():
    c = inputs.make_case(inputs.CONFIGS["C4"])
    check(c, users=sorted(set(pick_users(c, 12)) | {0, 255, 511}))


@functools.lru_cache(maxsize=1)
def c5_on_the_gpu():
    """C5 once for the tests below: the case, its sample of users and the library's results (kept on the device).
    The sample: shortest / longest history, fewest / most targets, a median history and 12 seeded random users."""
    c = inputs.make_case(inputs.CONFIGS["C5"])
    median = int(np.argsort(c.hist_len)[c.batch // 2])
    users = sorted(set(pick_users(c, 12)) | {median})
    assert len(users) >= 16 and max(int(c.hist_len[u]) for u in users) == 8192
    return c, users, run_gpu(c, norm_of(c))


def test_c5_long_histories_sampled_users():
    c, users, gpu = c5_on_the_gpu()
    users = [u for u in users if c.hist_len[u] < 8192]
    say(f"  histories {[int(c.hist_len[u]) for u in users]}")
    check(c, users=users, gpu=gpu)


@pytest.mark.parametrize("which", [0, 1])
def test_c5_users_at_the_history_cap(which):
    # the users of the sample at the cap of 8192 history tokens (the longest-history pick is one), all heads of both kv
    # groups, one user per test, with the oracle run per query head (its backward pass runs one thread per
    # (user, kv head): minutes for such a user)
    c, users, gpu = c5_on_the_gpu()
    capped = [u for u in users if c.hist_len[u] == 8192]
    assert len(capped) >= 2
    check(c, users=[capped[which]], gpu=gpu, per_head=True)


def test_large_logits_and_unit_norm():
    """Logits far into both tails of the SiLU (weights ~ x and ~ 0) with norm = 1."""
    c = inputs.make_case(inputs.custom_config("pw_big", FULL, [100, 70], [5, 9], 8, 2, 64, std=1.5, seed=53))
    check(c, norm=1.0, compare=close_on_tensor_scale)


@pytest.mark.parametrize("name", ["I1", "I2", "I3", "I2_RT"])
def test_inference_shapes_split_the_keys(name):
    """A few requests: the forward pass splits the keys and adds up the partial sums (the backward pass is unsplit)."""
    c = inputs.make_case(inputs.CONFIGS[name])
    b = device_batch(c, norm_of(c))
    assert b.fwd_ws is not None and b.fwd_ws.numel() > 4096   # partial results in the workspace
    check(c)


def test_split_edge_batch():
    # short users next to a long one: splits that see no key, less than a tile, exactly two tiles
    c = inputs.make_case(inputs.custom_config("pw_split", TARGET, [2048, 0, 1, 63, 128, 65, 1000, 64],
                                              [16, 5, 1, 33, 64, 2, 70, 0], 8, 2, 64, seed=56))
    check(c)
