"""The seeded generators: reproducible, independent of chunking, with the advertised shapes."""
import numpy as np

import bench
from paper_2602_11235_amd import inputs


def test_splitmix64_published_vector():
    # first outputs of the splitmix64 sequence started at state 0 (reference vector of the algorithm)
    got = inputs.raw_bits(np.uint64(0), 0, 3)
    assert int(got[0]) == 0xE220A8397B1DCDAF
    assert int(got[1]) == 0x6E789E6AA1B965F4
    assert int(got[2]) == 0x06C45D188009454F


def test_normal_is_chunk_independent_and_standard():
    key = inputs.stream_key(7, 3)
    a = inputs.normal(key, 200001)
    b = inputs.normal(key, 200001, chunk=4097)
    assert np.array_equal(a, b)
    assert abs(a.mean()) < 0.01 and abs(a.std() - 1.0) < 0.01
    assert not np.array_equal(a, inputs.normal(inputs.stream_key(7, 4), 200001))


def test_bf16_round_trip_is_rne():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e-5, 1.0 + 2 ** -8 + 2 ** -20], dtype=np.float32)
    bits = inputs.f32_to_bf16_bits(x)
    back = inputs.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties to 1 + 2^-6
    assert back[1] == 1.0 and back[2] == 1.015625 and back[0] == 1.0 and back[3] == -2.5
    assert back[5] == 1.0078125
    assert np.array_equal(inputs.f32_to_bf16_bits(back), bits)


def test_c1_shapes_and_offsets():
    c = inputs.make_case(inputs.CONFIGS["C1"])
    assert c.hist_len.tolist() == [40, 64] and c.n_targets.tolist() == [8, 8]
    assert c.kv_offsets.tolist() == [0, 48, 120] and c.q_offsets.tolist() == [0, 48, 120]
    assert c.q.shape == (120, 4, 16) and c.k.shape == (120, 1, 16) and c.dout.shape == c.q.shape
    c2 = inputs.make_case(inputs.CONFIGS["C1"])
    assert np.array_equal(c.q, c2.q) and np.array_equal(c.v, c2.v)


def test_length_recipes():
    c2 = inputs.CONFIGS["C2"]
    L = inputs._draw_lengths(c2.hist, inputs.stream_key(c2.seed, 0), c2.batch)
    assert L.min() >= 128 and L.max() <= 512 and len(set(L.tolist())) > 32
    c5 = inputs.CONFIGS["C5"]
    L5 = inputs._draw_lengths(c5.hist, inputs.stream_key(c5.seed, 0), 100000)
    assert L5.max() == 8192 and L5.min() >= 750
    assert 1400 < np.median(L5) < 1600          # Pareto(alpha=1, scale 750): median 1500
    assert 0.08 < (L5 == 8192).mean() < 0.10    # 750/8192 = 9.2 % of users sit at the cap


def test_target_layer_offsets_and_subset():
    cfg = inputs.custom_config("t", inputs.LAYER_TARGET, [5, 0, 9], [3, 2, 0], 4, 2, 16)
    c = inputs.make_case(cfg)
    assert c.q_offsets.tolist() == [0, 3, 5, 5] and c.kv_offsets.tolist() == [0, 8, 10, 19]
    s = inputs.take_users(c, [2, 0])
    assert s.hist_len.tolist() == [9, 5] and s.q_offsets.tolist() == [0, 0, 3]
    assert np.array_equal(s.k[:9], c.k[10:19]) and np.array_equal(s.q, c.q[0:3])


def test_visible_pairs_formula():
    hl = np.array([40, 64], np.int32)
    nt = np.array([8, 8], np.int32)
    assert bench.visible_pairs(hl, nt, 4, inputs.LAYER_FULL) == 26176
    assert bench.visible_pairs(hl, nt, 4, inputs.LAYER_TARGET) == 4 * (328 + 520)


def test_gln_case_is_reproducible_and_groups_differ_in_distribution():
    a = inputs.make_gln_case("g", 4000, 64, 4, dtype="bf16", gated=True, seed=3)
    b = inputs.make_gln_case("g", 4000, 64, 4, dtype="bf16", gated=True, seed=3)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.group_id, b.group_id) and np.array_equal(a.gamma, b.gamma)
    assert a.x.shape == (4000, 64) and a.gate.shape == a.x.shape and a.gamma.shape == (4, 64)
    assert a.group_id.dtype == np.int32 and a.group_id.min() == 0 and a.group_id.max() == 3
    counts = np.bincount(a.group_id, minlength=4)
    assert counts.min() > 800                                   # uniform over the groups
    # every value survives a bf16 round trip, and the groups' feature means / spreads differ (what the groups are for)
    assert np.array_equal(inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(a.x)).reshape(a.x.shape), a.x)
    means = np.array([a.x[a.group_id == g].mean() for g in range(4)])
    stds = np.array([a.x[a.group_id == g].std() for g in range(4)])
    assert np.ptp(means) > 0.2 and np.ptp(stds) > 0.2
    assert inputs.make_gln_case("g", 10, 8, 2, gated=False).gate is None


def test_inference_configs_are_small_target_layer_batches():
    for name in ("I1", "I2", "I3", "I2_RT"):
        cfg = inputs.CONFIGS[name]
        assert cfg.layer == inputs.LAYER_TARGET and cfg.batch <= 8 and cfg.dtype == "bf16"
    c = inputs.make_case(inputs.CONFIGS["I2_RT"])
    assert c.total_q == int(c.n_targets.sum()) and c.rt_len is not None
    assert c.total_kv == int((c.hist_len + c.rt_len + c.n_targets).sum())
