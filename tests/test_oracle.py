"""Pins for the CPU oracle: every function is checked against something other
than itself -- the paper's worked example, closed forms, exact rational brute
force, integer matmul -- chosen so that a dropped term, a wrong sign or index,
or a transposed operand fails at least one of them."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import tmac_workloads as wl
from oracle import tmac_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- tables ----

def _read_worked_example():
    rows = []
    with open(os.path.join(GOLDEN, "worked_example_g4.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, signs = line.split(":")
            rows.append(([int(b) for b in bits.split()],
                         [1 if s == "+" else -1 for s in signs.split()]))
    return rows


@pytest.mark.parametrize("A", [(1.0, 2.0, 4.0, 8.0), (0.5, -3.0, 7.25, 11.0), (-1.0, -1.0, 2.0, 100.0)])
def test_worked_example_section_3_1(A):
    """Section 3.1 example: 0000 -> -A1-A2-A3-A4, 0101 -> -A1+A2-A3+A4, table of 16."""
    rows = _read_worked_example()
    assert len(rows) == 3
    lut = orc.precompute_lut(np.array([A]), g=4)
    assert lut.shape == (1, 1, 16)
    for wbits, signs in rows:
        idx = orc.group_indices(np.array([wbits], dtype=np.uint8), g=4)
        assert idx.shape == (1, 1)
        expect = sum(s * a for s, a in zip(signs, A))
        assert lut[0, 0, idx[0, 0]] == expect
    # the table runs from -sum(A) to +sum(A)
    assert lut[0, 0, 0] == -sum(A) and lut[0, 0, 15] == sum(A)


def test_index_bit_order_lowest_k_is_lsb():
    """Algorithm 1, PreprocessWeights: element k contributes at bit k % g."""
    assert orc.group_indices(np.array([[1, 0, 0, 0]]), 4)[0, 0] == 1
    assert orc.group_indices(np.array([[0, 0, 0, 1]]), 4)[0, 0] == 8
    assert orc.group_indices(np.array([[0, 1, 0, 1]]), 4)[0, 0] == 10
    two = orc.group_indices(np.array([[1, 0, 0, 0, 0, 1, 1, 0]]), 4)
    assert two.tolist() == [[1, 6]]


def test_table_closed_forms():
    """Mirror symmetry T[p] = -T[~p] (Section 3.3), zero column sum, T[2^g-1] = sum(A),
    table size 2^g per g activations (Section 3.1: four times the activations at g=4)."""
    rng = np.random.default_rng(1)
    A = rng.standard_normal((3, 32))
    lut = orc.precompute_lut(A, 4)
    assert lut.shape == (3, 8, 16)
    assert lut.size == 4 * A.size
    assert np.array_equal(lut + lut[..., ::-1], np.zeros_like(lut))
    assert np.allclose(lut.sum(axis=-1), 0.0, atol=1e-12)
    assert np.allclose(lut[..., 15], A.reshape(3, 8, 4).sum(-1), atol=1e-12)
    # every entry is a signed sum: brute force over all 16 patterns of one group
    a = A[0, :4]
    for p in range(16):
        expect = sum((a[j] if (p >> j) & 1 else -a[j]) for j in range(4))
        assert abs(lut[0, 0, p] - expect) < 1e-12
    # other g
    lut2 = orc.precompute_lut(A, 2)
    assert lut2.shape == (3, 16, 4)
    assert np.allclose(lut2[0, 0], [-A[0, 0] - A[0, 1], A[0, 0] - A[0, 1], -A[0, 0] + A[0, 1], A[0, 0] + A[0, 1]])


def test_mirror_roundtrip():
    rng = np.random.default_rng(2)
    lut = orc.precompute_lut(rng.integers(-127, 128, size=(2, 16)), 4)
    half = orc.mirror_half(lut)
    assert half.shape[-1] == 8
    assert np.array_equal(orc.expand_mirror(half), lut)


def test_int_tables_are_exact_and_bounded():
    a = np.array([[127, -127, 127, 127, -128 + 1, 0, 5, -9]], dtype=np.int8)
    lut = orc.precompute_lut(a, 4)
    assert lut.dtype == np.int64
    assert lut.max() == 508 and lut.min() == -508
    # all entries of one table share the parity of the group's sum
    assert np.all((lut[0, 0] - lut[0, 0, 15]) % 2 == 0)


# ---------------------------------------------------------- bit planes ----

@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_bit_planes_reconstruct(bits):
    """Eq. 1: W = sum_i 2^i W_i, exhaustively over all codes."""
    q = np.arange(1 << bits, dtype=np.uint8).reshape(1, -1)
    q = np.repeat(q, 4 // q.shape[1] + 1, axis=1)[:, : max(4, q.shape[1])]
    planes = orc.bit_planes(q, bits)
    assert len(planes) == bits
    rec = sum((p.astype(np.int64) << i) for i, p in enumerate(planes))
    assert np.array_equal(rec, q)
    for p in planes:
        assert set(np.unique(p)) <= {0, 1}


def test_eq1_bit_serial_identity():
    """Eq. 1: A x W = sum_i 2^i A x W_i with integer data (exact)."""
    rng = np.random.default_rng(3)
    A = rng.integers(-50, 50, size=(3, 24))
    q = rng.integers(0, 16, size=(5, 24))
    planes = orc.bit_planes(q, 4)
    lhs = A @ q.T
    rhs = sum((1 << i) * (A @ p.astype(np.int64).T) for i, p in enumerate(planes))
    assert np.array_equal(lhs, rhs)


# ---------------------------------------------------- the definition ----

def test_dequantize_hand_example():
    """w = s*(q-z): q=[3,0,1,2], s=0.5, z=1 -> [1,-0.5,0,0.5]; a=[1,2,3,4] -> 2."""
    q = np.array([[3, 0, 1, 2]], dtype=np.uint8)
    s = np.array([[0.5]], dtype=np.float16)
    z = np.array([[1.0]], dtype=np.float16)
    W = orc.dequantize(q, s, z, group=4)
    assert W.tolist() == [[1.0, -0.5, 0.0, 0.5]]
    R = orc.mpgemm_definition(np.array([[1, 2, 3, 4]], dtype=np.float16), q, s, z, group=4)
    assert R.shape == (1, 1) and R[0, 0] == 2.0
    # per-tensor form
    Wt = orc.dequantize(q, group=0, weight_scale=0.5, zero_point=1.0)
    assert np.array_equal(Wt, W)


def test_definition_group_boundaries_and_orientation():
    """Two groups with different scale/zero, N != M, exact rational brute force."""
    rng = np.random.default_rng(4)
    N, M, K, G, b = 2, 3, 8, 4, 3
    q = rng.integers(0, 1 << b, size=(M, K), dtype=np.uint8)
    s = rng.uniform(0.01, 0.1, size=(M, K // G)).astype(np.float16)
    z = rng.uniform(0, 7, size=(M, K // G)).astype(np.float16)
    a = rng.standard_normal((N, K)).astype(np.float16)
    R = orc.mpgemm_definition(a, q, s, z, group=G)
    assert R.shape == (N, M)
    for n in range(N):
        for m in range(M):
            acc = Fraction(0)
            for k in range(K):
                w = Fraction(float(s[m, k // G])) * (int(q[m, k]) - Fraction(float(z[m, k // G])))
                acc += Fraction(float(a[n, k])) * w
            assert abs(R[n, m] - float(acc)) <= 1e-12 * max(1.0, abs(float(acc)))


def test_definition_closed_forms_bias_term():
    """All-zero codes: R = -sum_G s z S.  All-max codes: R = sum_G s (2^b-1-z) S."""
    rng = np.random.default_rng(5)
    N, M, K, G, b = 2, 4, 64, 16, 4
    s = rng.uniform(0.01, 0.1, size=(M, K // G)).astype(np.float16)
    z = rng.uniform(0, 15, size=(M, K // G)).astype(np.float16)
    a = rng.standard_normal((N, K)).astype(np.float16)
    S = a.astype(np.float64).reshape(N, K // G, G).sum(-1)
    s64, z64 = s.astype(np.float64), z.astype(np.float64)
    for code, coef in ((0, -z64), (15, 15.0 - z64)):
        q = np.full((M, K), code, dtype=np.uint8)
        expect = np.einsum("ng,mg->nm", S, s64 * coef)
        for fn in (orc.mpgemm_definition,
                   lambda *args, **kw: orc.lut_mpgemm(args[0], args[1], b, *args[2:], **kw)):
            R = fn(a, q, s, z, group=G)
            assert np.allclose(R, expect, rtol=1e-12, atol=1e-12)


# ------------------------------------- LUT formulation == definition ----

@pytest.mark.parametrize("bits", [1, 2])
def test_lut_route_exhaustive_one_group(bits):
    """Every combination of codes of one group of g=4 weights, integer activations,
    s=1, z=0: the LUT route must equal numpy's integer matmul exactly."""
    codes = list(itertools.product(range(1 << bits), repeat=4))
    q = np.array(codes, dtype=np.uint8)                    # [M = (2^b)^4, K = 4]
    a = np.array([[3, -5, 7, 11], [1, 1, -2, 0]], dtype=np.float64)
    ref = a.astype(np.int64) @ q.astype(np.int64).T
    R = orc.lut_mpgemm(a, q, bits, group=0, weight_scale=1.0, zero_point=0.0)
    assert np.array_equal(R, ref.astype(np.float64))
    R1 = orc.algorithm1_unscaled(a, q, bits)
    assert np.array_equal(R1, ref.astype(np.float64))


@pytest.mark.parametrize("bits,K,G", [(3, 8, 4), (4, 32, 8), (4, 32, 32), (2, 64, 16), (1, 16, 4)])
def test_lut_route_random_matches_definition(bits, K, G):
    rng = np.random.default_rng(100 + bits + K)
    N, M = 2, 8
    q = rng.integers(0, 1 << bits, size=(M, K), dtype=np.uint8)
    s = rng.uniform(0.01, 0.1, size=(M, K // G)).astype(np.float16)
    z = rng.uniform(0, (1 << bits) - 1, size=(M, K // G)).astype(np.float16)
    a = rng.standard_normal((N, K)).astype(np.float16)
    ref = orc.mpgemm_definition(a, q, s, z, group=G)
    R = orc.lut_mpgemm(a, q, bits, s, z, group=G)
    assert np.allclose(R, ref, rtol=1e-11, atol=1e-12)
    # integer data, unit scale: exact
    ai = rng.integers(-20, 20, size=(N, K)).astype(np.float64)
    ones = np.ones((M, K // G), dtype=np.float16)
    zer = np.zeros((M, K // G), dtype=np.float16)
    Ri = orc.lut_mpgemm(ai, q, bits, ones, zer, group=G)
    assert np.array_equal(Ri, (ai.astype(np.int64) @ q.astype(np.int64).T).astype(np.float64))


@pytest.mark.parametrize("g", [2, 8])
def test_lut_route_other_group_sizes(g):
    """LUT group sizes 2 and 8 (Section 4 on the choice of g): table shape and closed forms, every
    entry against the signed sum it stands for, exhaustive codes of one group at 1 bit (g = 8:
    all 256 patterns) and 2 bit (g = 2: all 16 pairs) against numpy's integer matmul, and random
    grouped data against the definition."""
    rng = np.random.default_rng(300 + g)
    A = rng.integers(-50, 50, size=(2, 16)).astype(np.float64)
    lut = orc.precompute_lut(A, g)
    assert lut.shape == (2, 16 // g, 1 << g)
    assert np.array_equal(lut + lut[..., ::-1], np.zeros_like(lut))
    assert np.array_equal(lut[..., -1], A.reshape(2, 16 // g, g).sum(-1))
    for p in range(1 << g):
        expect = sum((A[1, g + j] if (p >> j) & 1 else -A[1, g + j]) for j in range(g))
        assert lut[1, 1, p] == expect
    bits = 1 if g == 8 else 2
    q = np.array(list(itertools.product(range(1 << bits), repeat=g)), dtype=np.uint8)   # [(2^b)^g, g]
    a = A[:, :g]
    ref = (a.astype(np.int64) @ q.astype(np.int64).T).astype(np.float64)
    assert np.array_equal(orc.lut_mpgemm(a, q, bits, group=0, g=g), ref)
    assert np.array_equal(orc.algorithm1_unscaled(a, q, bits, g=g), ref)
    N, M, K, G, b = 2, 8, 64, 32, 3
    q = rng.integers(0, 1 << b, size=(M, K), dtype=np.uint8)
    sc = rng.uniform(0.01, 0.1, size=(M, K // G)).astype(np.float16)
    z = rng.uniform(0, 7, size=(M, K // G)).astype(np.float16)
    act = rng.standard_normal((N, K)).astype(np.float16)
    assert np.allclose(orc.lut_mpgemm(act, q, b, sc, z, group=G, g=g), orc.mpgemm_definition(act, q, sc, z, group=G),
                       rtol=1e-11, atol=1e-12)
    aq = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    t = rng.integers(0, 3, size=(M, K), dtype=np.uint8)
    assert np.array_equal(orc.lut_int_matmul(aq, t, 2, 1, g=g)[0], orc.ternary_int_matmul(aq, t, 1))


def test_bias_vanishes_at_mid_zero_point():
    """z = (2^b-1)/2 leaves only the look-up term: R = sum_G s * 1/2 * sum_i 2^i L_i."""
    rng = np.random.default_rng(6)
    N, M, K, G, b = 1, 4, 32, 16, 2
    q = rng.integers(0, 4, size=(M, K), dtype=np.uint8)
    s = rng.uniform(0.01, 0.1, size=(M, K // G)).astype(np.float16)
    z = np.full((M, K // G), 1.5, dtype=np.float16)
    a = rng.standard_normal((N, K)).astype(np.float16)
    lut = orc.precompute_lut(a, 4)
    L = sum((1 << i) * orc.lookup_sum(lut, orc.group_indices(p, 4), G // 4)
            for i, p in enumerate(orc.bit_planes(q, b)))
    expect = (0.5 * L * s.astype(np.float64)[None]).sum(-1)
    assert np.allclose(orc.mpgemm_definition(a, q, s, z, group=G), expect, rtol=1e-11, atol=1e-13)


def test_sign_symmetries():
    rng = np.random.default_rng(7)
    N, M, K = 2, 6, 32
    a = rng.standard_normal((N, K)).astype(np.float16)
    # 1-bit sign weights, z = 1/2: flipping every bit negates R exactly
    q = rng.integers(0, 2, size=(M, K), dtype=np.uint8)
    R = orc.lut_mpgemm(a, q, 1, group=0, weight_scale=0.25, zero_point=0.5)
    Rf = orc.lut_mpgemm(a, 1 - q, 1, group=0, weight_scale=0.25, zero_point=0.5)
    assert np.array_equal(R, -Rf)
    assert np.array_equal(orc.mpgemm_definition(a, q, group=0, weight_scale=0.25, zero_point=0.5),
                          -orc.mpgemm_definition(a, 1 - q, group=0, weight_scale=0.25, zero_point=0.5))
    # ternary: t -> -t is q -> 2-q
    aq = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    qt = rng.integers(0, 3, size=(M, K), dtype=np.uint8)
    Ri, _ = orc.lut_int_matmul(aq, qt, 2, 1)
    Rn, _ = orc.lut_int_matmul(aq, 2 - qt, 2, 1)
    assert np.array_equal(Ri, -Rn)
    # a -> -a
    Ra, _ = orc.lut_int_matmul(-aq, qt, 2, 1)
    assert np.array_equal(Ri, -Ra)


# ------------------------------------------------------- integer path ----

def test_int_path_matches_bruteforce_and_numerator_even():
    rng = np.random.default_rng(8)
    N, M, K = 2, 5, 24
    aq = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    q = rng.integers(0, 3, size=(M, K), dtype=np.uint8)
    ref = orc.ternary_int_matmul(aq, q, 1)
    for n in range(N):
        for m in range(M):
            assert ref[n, m] == sum(int(aq[n, k]) * (int(q[m, k]) - 1) for k in range(K))
    R, numer = orc.lut_int_matmul(aq, q, 2, 1)
    assert np.array_equal(R, ref)
    assert np.all(numer % 2 == 0)
    # code 3 is accepted and means +2
    q3 = q.copy()
    q3[0, 0] = 3
    R3, _ = orc.lut_int_matmul(aq, q3, 2, 1)
    assert np.array_equal(R3, orc.ternary_int_matmul(aq, q3, 1))


def test_int_path_f32_output_two_roundings():
    """fl(fl(R*s_a)*s_w): products of two fp32 are exact in fp64, so a correctly
    rounded reference is obtained by rounding the exact fp64 product twice."""
    rng = np.random.default_rng(9)
    r = rng.integers(-(1 << 20), 1 << 20, size=(3, 50))
    s_a = rng.uniform(0.001, 0.1, size=3).astype(np.float32)
    s_w = np.float32(0.0213)
    out = orc.int_path_output_f32(r, s_a, s_w)
    assert out.dtype == np.float32
    for n in range(3):
        for m in range(50):
            f1 = np.float32(float(r[n, m]) * float(s_a[n]))
            f2 = np.float32(float(f1) * float(s_w))
            assert out[n, m] == f2
    assert orc.int_path_output_f32(np.array([[3]]), np.array([0.5], np.float32), 0.25)[0, 0] == 0.375


# ------------------------------------------- fp16 tables, quantised tables ----

def test_fp16_table_route_error_is_far_below_tolerance():
    """Rounding every table entry to fp16 once costs a few 1e-4 relative
    Frobenius error at Llama-like K: well inside the 2e-3 bar, so a measured
    error near the bar signals a bug rather than rounding."""
    rng = np.random.default_rng(10)
    N, M, K, G, b = 1, 128, 1024, 128, 4
    q = rng.integers(0, 16, size=(M, K), dtype=np.uint8)
    s = rng.uniform(0.01, 0.1, size=(M, K // G)).astype(np.float16)
    z = rng.uniform(0, 15, size=(M, K // G)).astype(np.float16)
    a = rng.standard_normal((N, K)).astype(np.float16)
    ref = orc.mpgemm_definition(a, q, s, z, group=G)
    R16 = orc.lut_mpgemm(a, q, b, s, z, group=G, table_dtype=np.float16)
    err = orc.rel_frobenius(R16, ref)
    assert 1e-5 < err < 8e-4


def test_table_quantisation_per_unit_properties():
    """Section 3.3 table quantisation, one scale per 16 activations: entries are integers in
    [-127, 127], the largest magnitude of every non-zero unit is exactly 127, the mirror
    symmetry survives rounding, an all-zero unit quantises to zeros with scale 0, and
    de-quantised entries are within half a step of the exact ones."""
    rng = np.random.default_rng(77)
    A = rng.standard_normal((3, 64)).astype(np.float16)
    A[1, 16:32] = 0
    lut = orc.precompute_lut(A, 4)
    qt, sc = orc.quantize_tables_int8_per_unit(lut, 4)
    assert qt.shape == lut.shape and sc.shape == (3, 4)
    assert qt.min() >= -127 and qt.max() <= 127
    assert np.array_equal(qt, -qt[..., ::-1])
    units = np.abs(qt).reshape(3, 4, 64).max(axis=2)
    assert units[1, 1] == 0 and sc[1, 1] == 0
    assert np.all(np.delete(units.ravel(), 5) == 127)
    deq = qt * np.repeat(sc, 4, axis=1)[:, :, None]
    step = np.repeat(sc, 4, axis=1)[:, :, None]
    assert np.all(np.abs(deq - lut) <= 0.5 * step + 1e-12)
    # scale of a unit = largest sum of magnitudes among its four tables / 127
    amax = np.abs(A.astype(np.float64)).reshape(3, 4, 4, 4).sum(axis=3).max(axis=2)
    assert np.allclose(sc, amax / 127.0, rtol=0, atol=1e-15)


def test_table_quantisation_route_small_exact_cases():
    """A unit with a single non-zero activation a has entries +-a and step |a|/127: every entry
    is representable, so the quantised route equals the definition."""
    M, K = 6, 32
    rng = np.random.default_rng(78)
    A = np.zeros((2, K), dtype=np.float16)
    A[0, ::16] = [1.5, -2.25]
    A[1, 3::16] = [0.75, 3.0]
    q = rng.integers(0, 16, size=(M, K), dtype=np.uint8)
    s = rng.uniform(0.01, 0.1, size=(M, 2)).astype(np.float16)
    z = rng.uniform(0, 15, size=(M, 2)).astype(np.float16)
    ref = orc.mpgemm_definition(A, q, s, z, 16)
    got = orc.lut_mpgemm_tq(A, q, 4, s, z, 16)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_table_quantisation_route_error_matches_the_papers_magnitude():
    """Table 3 prints an NMSE increase of about 2e-5 for the table-quantised kernel on Gaussian
    4-bit GEMV (3.33e-3 -> 3.35e-3), i.e. a relative error of about 4.5e-3 against the result
    with exact tables; the per-unit reading lands in the same range, and far above the fp16
    tables' error."""
    p = wl.make_grouped(0, 900, 1, 256, 2048, 4, 128)
    ref = orc.mpgemm_definition(p.act, p.q, p.scales, p.zeros, p.group)
    tq = orc.lut_mpgemm_tq(p.act, p.q, 4, p.scales, p.zeros, p.group)
    err = orc.rel_frobenius(tq, ref)
    assert 1.5e-3 < err < 8e-3, err
    assert 2e-6 < orc.nmse(tq, ref) < 6e-5
    # unpadded K that is not a multiple of 16 goes through the zero padding
    p2 = wl.make_grouped(0, 901, 2, 24, 24, 2, 8)
    err2 = orc.rel_frobenius(orc.lut_mpgemm_tq(p2.act, p2.q, 2, p2.scales, p2.zeros, 8),
                             orc.mpgemm_definition(p2.act, p2.q, p2.scales, p2.zeros, 8))
    assert err2 < 2e-2


# ------------------------------------------------------------ error measures ----

def test_error_measures_hand_values():
    """The yardsticks of every floating-point assertion, on numbers worked by hand:
    x = (3, 4), ref = (0, 5): x - ref = (3, -1), ||x - ref|| = sqrt(10), ||ref|| = 5, so the relative
    Frobenius error is sqrt(10)/5 and the NMSE 10/25; a matrix argument is taken as one long vector
    (Frobenius norm); the measure is not symmetric in its arguments; identical inputs give 0; a zero
    reference falls back to the absolute norm."""
    assert orc.rel_frobenius([3.0, 4.0], [0.0, 5.0]) == pytest.approx(10 ** 0.5 / 5, rel=1e-15)
    assert orc.nmse([3.0, 4.0], [0.0, 5.0]) == pytest.approx(0.4, rel=1e-15)
    # 2 x 2: x - ref = [[1, -2], [0, 2]] -> 3; ||ref||_F = ||[[2, 2], [4, 5]]|| = 7
    x = np.array([[3.0, 0.0], [4.0, 7.0]])
    ref = np.array([[2.0, 2.0], [4.0, 5.0]])
    assert orc.rel_frobenius(x, ref) == pytest.approx(3.0 / 7.0, rel=1e-15)
    assert orc.nmse(x, ref) == pytest.approx(9.0 / 49.0, rel=1e-15)
    assert orc.rel_frobenius(ref, x) == pytest.approx(3.0 / np.sqrt(74.0), rel=1e-15)
    assert orc.rel_frobenius(ref, ref) == 0.0 and orc.nmse(ref, ref) == 0.0
    assert orc.rel_frobenius([3.0, 4.0], [0.0, 0.0]) == 5.0
    # float32 inputs are widened before the subtraction: 1 + 2^-24 is not representable in fp32
    assert orc.rel_frobenius(np.array([1.0], np.float32), np.array([1.0 + 2.0 ** -24])) == pytest.approx(2.0 ** -24, rel=1e-6)
