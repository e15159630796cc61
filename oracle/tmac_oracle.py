"""CPU oracle for LUT-based mixed-precision GEMV/GEMM (T-MAC, arxiv 2407.00088).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP
path is checked against.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import it; the product package never does, and this
file imports nothing from the product package.

Two independent routes to the same result are given:

* the *definition* (Section 1/3: the method computes the ordinary product of
  the activations with the de-quantised weights, only without de-quantising):
  ``dequantize`` + ``mpgemm_definition`` / ``ternary_int_matmul``;
* the *LUT formulation*, step by step in the order of Algorithm 1 and Eq. 1:
  ``bit_planes`` -> ``group_indices`` -> ``precompute_lut`` -> ``lookup_sum``
  -> ``lut_mpgemm`` (with the +-1 bit transform of Section 4, "Bit-serial
  linear transformation").

Floating point is fp64 throughout unless a dtype is asked for explicitly;
integer work is int64.

Readings taken where the paper is silent or garbled (also listed in the design
notes): de-quantisation is ``w = s*(q - z)`` with a real-valued zero point in
code units; bit planes are numbered from 0 and plane i carries weight 2^i
(Eq. 1); inside a g-bit index the element with the lowest k is the least
significant bit (Algorithm 1, PreprocessWeights: shift by ``k % g``); the
Precompute loops of Algorithm 1 are read as "for every group of g activations,
for every bit pattern p, add the activation when its bit is set and subtract it
otherwise" (Section 3.1 example); ternary weights t map to 2-bit codes q=t+1
with zero point 1 (Section 5.1).
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------
# Route 1: the definition
# ----------------------------------------------------------------------------


def dequantize(q, scales=None, zeros=None, group=0, weight_scale=1.0, zero_point=0.0):
    """w[m,k] = s[m, k//G] * (q[m,k] - z[m, k//G]) in fp64.

    ``group == 0``: one scale and one zero for the whole tensor.
    ``zeros is None`` with group scales means z = (2^b-1)/2 is NOT assumed here;
    the caller must pass zeros explicitly (the oracle takes no defaults).
    """
    q = np.asarray(q)
    M, K = q.shape
    q64 = q.astype(np.float64)
    if group == 0:
        return np.float64(weight_scale) * (q64 - np.float64(zero_point))
    assert K % group == 0
    s = np.asarray(scales).astype(np.float64)
    z = np.asarray(zeros).astype(np.float64)
    assert s.shape == (M, K // group) and z.shape == s.shape
    s_full = np.repeat(s, group, axis=1)
    z_full = np.repeat(z, group, axis=1)
    return s_full * (q64 - z_full)


def mpgemm_definition(act, q, scales=None, zeros=None, group=0, weight_scale=1.0, zero_point=0.0):
    """R[n,m] = sum_k a[n,k] * w[m,k], all operands widened exactly to fp64
    (Algorithm 1: A is [N,K], W is [M,K], R is [N,M])."""
    W = dequantize(q, scales, zeros, group, weight_scale, zero_point)
    A = np.asarray(act).astype(np.float64)
    return A @ W.T


def ternary_int_matmul(act_q, q, zero_point=1):
    """Integer route for int8 activations and small integer weights:
    R_int[n,m] = sum_k a_q[n,k] * (q[m,k] - zero_point), exact in int64."""
    a = np.asarray(act_q).astype(np.int64)
    t = np.asarray(q).astype(np.int64) - int(zero_point)
    return a @ t.T


def int_path_output_f32(r_int, act_scale, weight_scale):
    """fp32 output of the integer path: two fp32 multiplies, left to right,
    fl(fl(float(R_int) * s_a[n]) * s_w).  float(R_int) is exact for |R_int| < 2^24."""
    r = np.asarray(r_int)
    assert np.abs(r).max(initial=0) < (1 << 24)
    f = r.astype(np.float32)
    f = (f * np.asarray(act_scale, dtype=np.float32)[:, None]).astype(np.float32)
    return (f * np.float32(weight_scale)).astype(np.float32)


def rel_frobenius(x, ref):
    """||x - ref||_F / ||ref||_F in fp64."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / den) if den > 0 else float(np.linalg.norm(x - ref))


def nmse(x, ref):
    """Normalised mean squared error ||x-ref||^2 / ||ref||^2 (the paper prints
    NMSE values in Table 3 without a formula; this is the reading used)."""
    return rel_frobenius(x, ref) ** 2


# ----------------------------------------------------------------------------
# Route 2: the LUT formulation, in the order of Algorithm 1
# ----------------------------------------------------------------------------


def bit_planes(q, bits):
    """PreprocessWeights, first half: W_i = (W >> i) & 1 for i = 0..b-1 (Eq. 1:
    W = sum_i 2^i W_i)."""
    q = np.asarray(q).astype(np.int64)
    assert q.min(initial=0) >= 0 and q.max(initial=0) < (1 << bits)
    return [((q >> i) & 1).astype(np.uint8) for i in range(bits)]


def group_indices(plane, g=4):
    """PreprocessWeights, second half: every g consecutive bits along K become
    one g-bit index, the bit of element k sits at position k % g."""
    plane = np.asarray(plane).astype(np.int64)
    M, K = plane.shape
    assert K % g == 0
    p = plane.reshape(M, K // g, g)
    idx = np.zeros((M, K // g), dtype=np.int64)
    for j in range(g):
        idx += p[:, :, j] << j
    return idx


def precompute_lut(act, g=4, dtype=np.float64):
    """Precompute: LUT[n, kg, p] = sum_j (+a[n, g*kg+j] if bit j of p else -a[...]).
    Shape (N, K/g, 2^g) (Section 3.1; Section 4 "Register swizzling": only adds
    and subtracts).  ``dtype`` is the accumulation/storage type of the entries."""
    A = np.asarray(act)
    A = A.astype(np.int64) if np.issubdtype(A.dtype, np.integer) else A.astype(np.float64)
    N, K = A.shape
    assert K % g == 0
    Ag = A.reshape(N, K // g, g)
    lut = np.zeros((N, K // g, 1 << g), dtype=A.dtype)
    for p in range(1 << g):
        for j in range(g):
            if (p >> j) & 1:
                lut[:, :, p] += Ag[:, :, j]
            else:
                lut[:, :, p] -= Ag[:, :, j]
    if np.issubdtype(A.dtype, np.integer):
        return lut
    return lut.astype(dtype)


def mirror_half(lut):
    """Mirror consolidation (Section 3.3): keep entries 0..2^(g-1)-1 only."""
    return lut[..., : lut.shape[-1] // 2]


def expand_mirror(half):
    """Rebuild the full table from the stored half: T[2^g-1-p] = -T[p]."""
    return np.concatenate([half, -half[..., ::-1]], axis=-1)


def lookup_sum(lut, idx, lut_groups_per_qgroup):
    """Look-up + aggregation for one bit plane (Algorithm 1, main loop):
    L[n, m, G] = sum over the LUT groups kg inside quantisation group G of
    LUT[n, kg, idx[m, kg]]."""
    N, KG, _ = lut.shape
    M, KG2 = idx.shape
    assert KG == KG2 and KG % lut_groups_per_qgroup == 0
    nq = KG // lut_groups_per_qgroup
    out = np.zeros((N, M, nq), dtype=lut.dtype if lut.dtype != np.float16 else np.float64)
    kg_range = np.arange(KG)
    for n in range(N):
        looked = lut[n][kg_range[None, :], idx]            # [M, KG]
        looked = looked.astype(out.dtype)
        out[n] = looked.reshape(M, nq, lut_groups_per_qgroup).sum(axis=2)
    return out


def group_sums(act, group):
    """S[n, G] = sum of the activations of quantisation group G (the product of
    A with the all-ones matrix J of Section 4, per group)."""
    A = np.asarray(act)
    A = A.astype(np.int64) if np.issubdtype(A.dtype, np.integer) else A.astype(np.float64)
    N, K = A.shape
    return A.reshape(N, K // group, group).sum(axis=2)


def lut_mpgemm(act, q, bits, scales=None, zeros=None, group=0, weight_scale=1.0,
               zero_point=0.0, g=4, table_dtype=np.float64):
    """Whole LUT route for float activations.

    With the bit transform f(v) = 2v-1 (s0=-1, s1=+1) each bit is
    v = (f(v)+1)/2, so alpha_i = 1/2 and beta_i = 1/2 (Section 4) and

      R[n,m] = sum_G s[m,G] * ( 1/2 * sum_i 2^i L_i[n,m,G]
                                + ((2^b-1)/2 - z[m,G]) * S[n,G] ).

    The first term is Algorithm 1's sum_i alpha_i R_i, the second is its R_beta
    with the zero point folded into the constant matrix B.
    ``table_dtype=np.float16`` rounds every table entry to fp16 once; the sums
    over looked-up entries stay in fp64.
    """
    q = np.asarray(q)
    M, K = q.shape
    G = K if group == 0 else group
    assert K % G == 0 and G % g == 0
    nq = K // G
    if group == 0:
        s = np.full((M, 1), np.float64(weight_scale))
        z = np.full((M, 1), np.float64(zero_point))
    else:
        s = np.asarray(scales).astype(np.float64)
        z = np.asarray(zeros).astype(np.float64)
    lut = precompute_lut(act, g, dtype=table_dtype)
    S = group_sums(act, G).astype(np.float64)                     # [N, nq]
    mid = (2.0 ** bits - 1.0) / 2.0
    N = lut.shape[0]
    Lsum = np.zeros((N, M, nq), dtype=np.float64)
    for i, plane in enumerate(bit_planes(q, bits)):
        idx = group_indices(plane, g)
        Lsum += (2.0 ** i) * lookup_sum(lut, idx, G // g).astype(np.float64)
    R = np.zeros((N, M), dtype=np.float64)
    for gq in range(nq):
        R += s[None, :, gq] * (0.5 * Lsum[:, :, gq] + (mid - z[None, :, gq]) * S[:, gq][:, None])
    return R


def lut_int_matmul(act_q, q, bits, zero_point, g=4):
    """Whole LUT route in exact integers for integer activations and an integer
    zero point: R_int = sum_k a_q * (q - z).  Returns (R_int, numerator) where
    numerator = sum_i 2^i L_i + (2^b - 1 - 2z) * S is always even."""
    q = np.asarray(q)
    M, K = q.shape
    lut = precompute_lut(act_q, g)                                 # int64
    S = group_sums(act_q, K)[:, 0]                                 # [N]
    N = lut.shape[0]
    Lsum = np.zeros((N, M), dtype=np.int64)
    for i, plane in enumerate(bit_planes(q, bits)):
        idx = group_indices(plane, g)
        Lsum += (1 << i) * lookup_sum(lut, idx, K // g)[:, :, 0]
    numer = Lsum + ((1 << bits) - 1 - 2 * int(zero_point)) * S[:, None]
    assert np.all(numer % 2 == 0)
    return numer // 2, numer


def algorithm1_unscaled(act, q, bits, g=4):
    """Algorithm 1 literally, for plain unsigned integer weights without scales:
    R = sum_i alpha_i R_i + R_beta with alpha_i = 2^i / 2 and
    beta = sum_i 2^i / 2 (every element of B), R_beta = A . B^T."""
    q = np.asarray(q)
    M, K = q.shape
    A = np.asarray(act).astype(np.float64)
    lut = precompute_lut(A, g)
    R = np.zeros((A.shape[0], M))
    for i, plane in enumerate(bit_planes(q, bits)):
        R_i = lookup_sum(lut, group_indices(plane, g), K // g)[:, :, 0]
        R += 0.5 * (2.0 ** i) * R_i
    beta = sum(0.5 * (2.0 ** i) for i in range(bits))
    B = np.full((M, K), beta)
    return R + A @ B.T


# ----------------------------------------------------------------------------
# Table quantisation (Section 3.3) -- reading: one scale per unit of four tables
# (16 activations), shared by the tables whose look-ups are added as integers
# before the single conversion
# ----------------------------------------------------------------------------


def quantize_tables_int8_per_unit(lut, tables_per_unit=4):
    """int8 table quantisation with one dynamic scale per unit of ``tables_per_unit``
    consecutive tables (16 activations for g = 4): scale = max|T| / 127 over the unit,
    entries rint(T / scale) clipped to +-127 (Section 3.3 "table quantization": fine-grained,
    dynamic; the granularity and the rounding are this build's reading).  The tables of a
    unit share a scale so that their looked-up entries can be added as integers.
    Returns (int8 tables as int64 [N, KG, P], scales fp64 [N, KG / tables_per_unit]);
    K/g must be a multiple of tables_per_unit (pad the activations with zeros first)."""
    N, KG, P = lut.shape
    assert KG % tables_per_unit == 0
    nu = KG // tables_per_unit
    t = lut.astype(np.float64).reshape(N, nu, tables_per_unit * P)
    amax = np.abs(t).max(axis=2)
    scale = amax / 127.0
    safe = np.where(amax > 0, scale, 1.0)
    qt = np.clip(np.rint(t / safe[:, :, None]), -127, 127).astype(np.int64)
    return qt.reshape(N, KG, P), scale


def lut_mpgemm_tq(act, q, bits, scales=None, zeros=None, group=0, weight_scale=1.0,
                  zero_point=0.0, g=4, tables_per_unit=4):
    """LUT route with int8-quantised tables (Section 3.3): as ``lut_mpgemm`` but every table
    entry is replaced by scale_unit * rint(T / scale_unit); the bias term keeps the exact
    activation sums.  Look-ups of one unit are added as integers, converted once and
    multiplied by the unit's scale."""
    q = np.asarray(q)
    M, K = q.shape
    A = np.asarray(act).astype(np.float64)
    unit = g * tables_per_unit
    Kp = (K + unit - 1) // unit * unit
    if Kp != K:                      # zero activations and zero codes: contribute nothing
        A = np.concatenate([A, np.zeros((A.shape[0], Kp - K))], axis=1)
        q = np.concatenate([q, np.zeros((M, Kp - K), dtype=q.dtype)], axis=1)
    G = K if group == 0 else group
    assert K % G == 0 and G % g == 0
    nq = K // G
    if group == 0:
        s = np.full((M, 1), np.float64(weight_scale))
        z = np.full((M, 1), np.float64(zero_point))
    else:
        s = np.asarray(scales).astype(np.float64)
        z = np.asarray(zeros).astype(np.float64)
    lut = precompute_lut(A, g)                                     # exact, fp64
    qt, usc = quantize_tables_int8_per_unit(lut, tables_per_unit)
    deq = qt.astype(np.float64) * np.repeat(usc, tables_per_unit, axis=1)[:, :, None]
    S = group_sums(A[:, :K], G).astype(np.float64)
    mid = (2.0 ** bits - 1.0) / 2.0
    N = A.shape[0]
    # per-LUT-group partial results, then summed per quantisation group (a unit never straddles
    # a quantisation group when G is a multiple of g * tables_per_unit; otherwise the tables of a
    # unit are still looked up one by one, so the split is by table)
    KG = Kp // g
    contrib = np.zeros((N, M, KG), dtype=np.float64)
    kg_range = np.arange(KG)
    for i, plane in enumerate(bit_planes(q, bits)):
        idx = group_indices(plane, g)                              # [M, KG]
        for n in range(N):
            contrib[n] += (2.0 ** i) * deq[n][kg_range[None, :], idx]
    R = np.zeros((N, M), dtype=np.float64)
    for gq in range(nq):
        k0, k1 = gq * G // g, (gq + 1) * G // g
        L = contrib[:, :, k0:k1].sum(axis=2)
        R += s[None, :, gq] * (0.5 * L + (mid - z[None, :, gq]) * S[:, gq][:, None])
    return R
