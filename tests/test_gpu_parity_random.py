"""GPU parity on seeded random batch shapes: head layouts, head widths, layers, batch sizes and length mixes drawn per
seed (lengths include empty histories, users without targets, empty users, lengths around the 32 / 64 / 128 tile
edges and a few long histories), with and without real-time tokens; forward and backward against the float64 oracle,
element by element.  The fixed edge batches pin the cases that were thought of; this sweep is for the combinations
that were not.  Tolerance: atol + rtol x the scale of the element's own (token, head) row (close_on_row_scale): the
draws contain users with two or three history tokens and a hundred candidates, whose dk/dv rows are sums of hundreds
of terms of order one."""
import numpy as np
import pytest

from paper_2602_11235_amd import inputs
from tests.hta_testlib import check_case, close_on_row_scale, say
from tests.test_gpu_parity_pointwise import check as check_pointwise

pytestmark = pytest.mark.gpu
FULL, TARGET = inputs.LAYER_FULL, inputs.LAYER_TARGET

HEADS = [(8, 2), (4, 4), (3, 1), (16, 2), (6, 2), (16, 4), (1, 1), (12, 4), (2, 1), (8, 1)]
WIDTHS = [16, 32, 64, 64, 64, 128]
EDGES = [0, 0, 1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257]


def draw_shape(seed: int, realtime: bool):
    """Lengths and head layout of one random batch (shapes only: the tensors come from the seeded input generator)."""
    rng = np.random.default_rng(1000 + seed)
    Hq, Hkv = HEADS[rng.integers(len(HEADS))]
    d = WIDTHS[(seed // 2) % len(WIDTHS)]   # every width and both layers turn up whatever the draws are
    layer = FULL if seed % 2 == 0 else TARGET
    B = int(rng.integers(1, 41))
    # a third of the users at a tile edge, the rest uniform; one batch in four has a few long histories
    hist = np.where(rng.random(B) < 0.33, rng.choice(EDGES, B), rng.integers(0, 400, B))
    if seed % 4 == 0:
        hist[rng.integers(B, size=max(1, B // 8))] = rng.integers(600, 1400, max(1, B // 8))
    tgts = np.where(rng.random(B) < 0.33, rng.choice(EDGES[:10], B), rng.integers(0, 150, B))
    rt = None
    if realtime:
        rt = np.where(rng.random(B) < 0.4, 0, rng.integers(1, 150, B))
    return layer, hist.astype(int), tgts.astype(int), Hq, Hkv, d, rt


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes(seed):
    layer, hist, tgts, Hq, Hkv, d, _ = draw_shape(seed, False)
    say(f"  seed {seed}: layer {layer} heads {Hq}/{Hkv} d {d} hist {list(hist)} targets {list(tgts)}")
    cfg = inputs.custom_config(f"random_{seed}", layer, hist, tgts, Hq, Hkv, d, dtype="bf16", std=0.3, seed=500 + seed)
    check_case(inputs.make_case(cfg), with_bwd=True, compare=close_on_row_scale)


@pytest.mark.parametrize("seed", range(8))
def test_random_shapes_with_realtime_tokens(seed):
    layer, hist, tgts, Hq, Hkv, d, rt = draw_shape(100 + seed, True)
    say(f"  seed {seed}: layer {layer} heads {Hq}/{Hkv} d {d} hist {list(hist)} rt {list(rt)} targets {list(tgts)}")
    cfg = inputs.custom_config(f"random_rt_{seed}", layer, hist, tgts, Hq, Hkv, d, dtype="bf16", std=0.3,
                               seed=700 + seed, rt_len=rt)
    check_case(inputs.make_case(cfg), with_bwd=True, compare=close_on_row_scale)


@pytest.mark.parametrize("seed", range(8))
def test_random_shapes_with_pointwise_weights(seed):
    # even seeds without, odd seeds with real-time tokens; norm = 1, so that the results are of order one or larger and
    # the relative part of the bound is the one that binds
    layer, hist, tgts, Hq, Hkv, d, rt = draw_shape(200 + seed, seed % 2 == 1)
    say(f"  seed {seed}: layer {layer} heads {Hq}/{Hkv} d {d} hist {list(hist)} rt {rt} targets {list(tgts)}")
    cfg = inputs.custom_config(f"random_pw_{seed}", layer, hist, tgts, Hq, Hkv, d, dtype="bf16", std=0.3,
                               seed=800 + seed, rt_len=rt)
    check_pointwise(inputs.make_case(cfg), norm=1.0, compare=close_on_row_scale)


def test_random_fp32_shape():
    layer, hist, tgts, Hq, Hkv, _, _ = draw_shape(50, False)
    cfg = inputs.custom_config("random_fp32", layer, hist[:12], tgts[:12], Hq, Hkv, 40, dtype="fp32", std=0.5, seed=900)
    check_case(inputs.make_case(cfg), with_bwd=True, compare=close_on_row_scale)
