"""Pins of the kernel-rounding models in tests/rounding_models.py (CPU only)."""
import numpy as np

import tmac_workloads as wl
from oracle import tmac_oracle as orc
import rounding_models as rm

# ---------------------------------------------- narrow running sums (fp16) ----

def test_narrow_sum_is_exact_on_small_integers_and_bounded_on_gaussian_data():
    """fp16 pairwise sums of eight table entries (the batched kernel's aggregation, Section 3.3 /
    Section 4 "fast aggregation" read for fp16 tables): exact whenever every partial sum is an
    integer below 2048 (then the route must equal the definition bit for bit), and on Gaussian
    activations an error of a few 1e-4, between the error of fp16 tables alone and the 2e-3 bar."""
    rng = np.random.default_rng(77)
    N, M, K, G, b = 2, 24, 512, 128, 4
    q = rng.integers(0, 16, size=(M, K), dtype=np.uint8)
    ones = np.ones((M, K // G), np.float16)
    zer = np.zeros((M, K // G), np.float16)
    ai = rng.integers(-30, 31, size=(N, K)).astype(np.float16)      # |entry| <= 120, |sum of 8| <= 960
    exact = (ai.astype(np.int64) @ q.astype(np.int64).T).astype(np.float64)
    assert np.array_equal(rm.lut_mpgemm_narrow(ai, q, b, ones, zer, G), exact)
    p = wl.make_grouped(5, 40, 4, 96, 5120, 4, 128)
    ref = orc.mpgemm_definition(p.act, p.q, p.scales, p.zeros, p.group)
    e_tab = orc.rel_frobenius(orc.lut_mpgemm(p.act, p.q, 4, p.scales, p.zeros, p.group, table_dtype=np.float16), ref)
    e_nar = orc.rel_frobenius(rm.lut_mpgemm_narrow(p.act, p.q, 4, p.scales, p.zeros, p.group), ref)
    assert 5e-5 < e_tab < e_nar < 8e-4
    # sums of two entries only: closer to the tables' own error
    e_2 = orc.rel_frobenius(rm.lut_mpgemm_narrow(p.act, p.q, 4, p.scales, p.zeros, p.group, tables_per_sum=2), ref)
    assert e_tab < e_2 < e_nar


# ------------------------------------------------ tables built by fp16 additions ----

def test_fp16_tree_tables_worked_example_and_special_cases():
    """Tables built with fp16 additions, pair sums first.  Worked by hand for a = (2048, 1, 1, 0),
    where fp16 has a spacing of 2 above 2048: +a0+a1 = 2049 is a tie and goes to the even 2048,
    +a2+a3 = 1, and 2048 + 1 is a tie again -> 2048, whereas the exact sum 2050 is representable;
    with -a1 every partial sum is exact.  The negated index mirrors exactly; one addition (g = 2)
    equals the once-rounded exact sum; small integers are exact at every g."""
    a = np.array([[2048, 1, 1, 0]], dtype=np.float16)
    t = rm.precompute_lut_fp16_tree(a, 4)[0, 0].astype(np.float64)
    once = orc.precompute_lut(a, 4, dtype=np.float16)[0, 0].astype(np.float64)
    assert t[15] == 2048.0 and once[15] == 2050.0
    assert t[0] == -2048.0 and once[0] == -2050.0
    assert t[0b1101] == 2048.0 == once[0b1101]          # 2048 - 1 = 2047, + 1 = 2048: no rounding anywhere
    assert t[0b0111] == 2048.0 and once[0b0111] == 2050.0   # a3 = 0: its sign does not matter
    rng = np.random.default_rng(91)
    A = (rng.standard_normal((3, 64)) * 50).astype(np.float16)
    for g in (2, 4, 8):
        T = rm.precompute_lut_fp16_tree(A, g)
        assert T.dtype == np.float16 and T.shape == (3, 64 // g, 1 << g)
        assert np.array_equal(T.astype(np.float64), -T[..., ::-1].astype(np.float64))
        exact = orc.precompute_lut(A, g)
        # each of the g - 1 additions is off by at most half a spacing of its result, and no partial
        # sum exceeds sum |a_j|
        top = np.abs(A.astype(np.float64)).reshape(3, -1, g).sum(-1).astype(np.float16)
        bound = 0.5 * (g - 1) * np.spacing(top).astype(np.float64)
        assert np.all(np.abs(T.astype(np.float64) - exact) <= bound[..., None])
    assert np.array_equal(rm.precompute_lut_fp16_tree(A, 2).view(np.uint16),
                          orc.precompute_lut(A, 2, dtype=np.float16).view(np.uint16))
    Ai = rng.integers(-100, 101, size=(2, 32)).astype(np.float16)
    for g in (2, 4, 8):
        assert np.array_equal(rm.precompute_lut_fp16_tree(Ai, g).astype(np.float64), orc.precompute_lut(Ai, g))


def test_fp16_tree_tables_route_error():
    """End to end the extra roundings of the partial sums cost little: on Gaussian activations the
    route with tree-built tables errs more than the once-rounded tables and stays far inside the
    2e-3 bar."""
    p = wl.make_grouped(5, 41, 2, 96, 5120, 4, 128)
    ref = orc.mpgemm_definition(p.act, p.q, p.scales, p.zeros, p.group)
    e_once = orc.rel_frobenius(orc.lut_mpgemm(p.act, p.q, 4, p.scales, p.zeros, p.group, table_dtype=np.float16), ref)
    e_tree = orc.rel_frobenius(rm.lut_mpgemm_fp16_tree(p.act, p.q, 4, p.scales, p.zeros, p.group), ref)
    print(f"fp16 tables: once-rounded {e_once:.2e}, built by fp16 additions {e_tree:.2e}")
    assert 5e-5 < e_once < e_tree < 6e-4


def test_fp16_routes_keep_their_error_on_heavy_tailed_activations():
    """The roundings of the fp16 routes (tables built by fp16 additions, narrow chunk sums) scale with
    the entries themselves: outlier channels 50 or 300 times the rest, Student-t tails or an all-positive
    offset leave the relative error where it is on Gaussian data, a fifth of the 2e-3 bar."""
    rng = np.random.default_rng(95)
    M, K, G, b = 32, 2048, 128, 4
    q = rng.integers(0, 16, size=(M, K), dtype=np.uint8)
    s = rng.uniform(0.01, 0.1, size=(M, K // G)).astype(np.float16)
    z = rng.uniform(0, 15, size=(M, K // G)).astype(np.float16)
    base = rng.standard_normal((2, K))
    cases = {
        "gauss": base,
        "1% x50": base * np.where(rng.random((2, K)) < 0.01, 50.0, 1.0),
        "0.2% x300": base * np.where(rng.random((2, K)) < 0.002, 300.0, 1.0),
        "student t3": rng.standard_t(3, size=(2, K)),
        "positive": np.abs(base) + 3.0,
    }
    for name, a in cases.items():
        a = a.astype(np.float16)
        ref = orc.mpgemm_definition(a, q, s, z, group=G)
        e_tree = orc.rel_frobenius(rm.lut_mpgemm_fp16_tree(a, q, b, s, z, group=G), ref)
        e_narrow = orc.rel_frobenius(rm.lut_mpgemm_narrow(a, q, b, s, z, G), ref)
        assert e_tree < 5e-4 and e_narrow < 7e-4, (name, e_tree, e_narrow)
