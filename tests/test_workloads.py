"""The seeded generators: reproducible, right shapes, right distributions."""
import numpy as np

import tmac_workloads as wl


def test_seed_rule_and_reproducibility():
    assert wl.seed_for(2, 1) == 20240700 + 201
    a, b = wl.config1(), wl.config1()
    assert np.array_equal(a.q, b.q) and np.array_equal(a.act, b.act)
    assert np.array_equal(a.scales, b.scales) and np.array_equal(a.zeros, b.zeros)


def test_config1_recipe():
    p = wl.config1()
    assert (p.N, p.M, p.K, p.bits, p.group) == (1, 256, 256, 2, 32)
    assert p.q.dtype == np.uint8 and p.q.min() == 0 and p.q.max() == 3
    assert p.scales.dtype == np.float16 and p.scales.shape == (256, 8)
    assert 0.0099 <= float(p.scales.min()) and float(p.scales.max()) <= 0.1001
    assert 0.0 <= float(p.zeros.min()) and float(p.zeros.max()) <= 3.0
    assert p.act.dtype == np.float16 and p.act.shape == (1, 256)
    assert abs(float(p.act.astype(np.float64).std()) - 1.0) < 0.15


def test_ternary_recipe():
    p = wl.make_ternary(4, 0, 2, 64, 512)
    assert p.bits == 2 and p.group == 0 and p.zero_point == 1.0
    assert set(np.unique(p.q)) <= {0, 1, 2}
    frac0 = float((p.q == 1).mean())
    assert 0.45 < frac0 < 0.55
    assert p.act_q.dtype == np.int8 and np.abs(p.act_q.astype(np.int32)).max() == 127
    assert p.act_scale.dtype == np.float32 and p.act_scale.shape == (2,)


def test_absmax_int8_is_round_to_nearest_even():
    a = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5]], dtype=np.float16)
    a_q, s = wl.absmax_int8(a)
    assert s[0] == np.float32(1.0)
    assert a_q.tolist() == [[127, 0, 2, 2, 0, -2]]


def test_shapes_listed():
    assert wl.LLAMA7B_SHAPES == [(4096, 4096), (11008, 4096), (4096, 11008)]
    assert wl.BITNET3B_SHAPES == [(3200, 3200), (8640, 3200), (3200, 8640)]
    assert wl.LLAMA13B_SHAPES == [(5120, 5120), (13824, 5120), (5120, 13824)]
