"""Models of the roundings the HIP kernels take on the fp16 path (test helpers, not the oracle).

The oracle (``oracle/tmac_oracle.py``) holds what the paper defines: the exact product and the
LUT formulation of Algorithm 1 in fp64.  The kernels round in two places of their own choosing,
and these functions replay exactly those roundings on the CPU so that a GPU test can tell "the
kernel does the arithmetic it says it does" (agreement to a few 1e-8) from "the result is inside
the 2e-3 bar" (which a wrong kernel could also be):

* ``precompute_lut_fp16_tree``: tables of fp16 activations built with fp16 additions, pair sums
  first (the library's reading of Section 3.1 / Section 4, where the table build is said to take
  additions and subtractions only, for 16-bit activations);
* ``lookup_sum_narrow`` / ``lut_mpgemm_narrow``: the batched kernels add the eight entries that a
  32-k chunk gives one bit plane in fp16 before widening.  This is the library's own choice and it
  is lossy; the paper's "fast 8-bit aggregation" (Section 4) is a different, integer technique.

They build on the oracle's exact steps (bit planes, indices, group sums) and are pinned by
``tests/test_rounding_models.py``.
"""
from __future__ import annotations

import numpy as np

from oracle import tmac_oracle as orc


def precompute_lut_fp16_tree(act, g=4):
    """Tables in the activations' own precision: the g signed terms +-a_j are added pairwise,
    ((+-a0 +- a1) + (+-a2 +- a3)) + ..., and every addition is rounded to fp16 (round to nearest
    even).  Returns a float16 array of shape (N, K/g, 2^g).  With g = 2 there is one addition and
    the result equals the once-rounded exact sum; from g = 4 on entries can differ from it by the
    roundings of the partial sums."""
    A = np.asarray(act)
    assert A.dtype == np.float16 and g & (g - 1) == 0
    N, K = A.shape
    assert K % g == 0
    Ag = A.reshape(N, K // g, g).astype(np.float64)
    lut = np.zeros((N, K // g, 1 << g), dtype=np.float16)
    for p in range(1 << g):
        terms = [Ag[:, :, j] if (p >> j) & 1 else -Ag[:, :, j] for j in range(g)]
        while len(terms) > 1:
            # the fp64 sum of two fp16 numbers is exact, so this is one rounding per addition
            terms = [(terms[i] + terms[i + 1]).astype(np.float16).astype(np.float64)
                     for i in range(0, len(terms), 2)]
        lut[:, :, p] = terms[0].astype(np.float16)
    return lut


def lookup_sum_narrow(lut16, idx, lut_groups_per_qgroup, tables_per_sum=8):
    """Look-up + aggregation for one bit plane with a narrow running sum: the entries of
    ``tables_per_sum`` consecutive LUT groups are added pairwise in fp16,
    ((e0+e1)+(e2+e3))+((e4+e5)+(e6+e7)), every add rounded to fp16; these short sums are then
    added in fp64.  ``lut16`` must be a float16 table."""
    assert lut16.dtype == np.float16
    N, KG, _ = lut16.shape
    M, KG2 = idx.shape
    T = tables_per_sum
    assert KG == KG2 and KG % lut_groups_per_qgroup == 0 and lut_groups_per_qgroup % T == 0
    assert T & (T - 1) == 0
    nq = KG // lut_groups_per_qgroup
    out = np.zeros((N, M, nq), dtype=np.float64)
    kg_range = np.arange(KG)
    for n in range(N):
        v = lut16[n][kg_range[None, :], idx].reshape(M, KG // T, T)      # fp16
        while v.shape[-1] > 1:
            v = (v[..., 0::2] + v[..., 1::2]).astype(np.float16)          # one rounding per add
        short = v[..., 0].astype(np.float64)                              # [M, KG/T]
        out[n] = short.reshape(M, nq, lut_groups_per_qgroup // T).sum(axis=2)
    return out


def _finish(Lsum, S, s, z, bits):
    mid = (2.0 ** bits - 1.0) / 2.0
    R = np.zeros(Lsum.shape[:2], dtype=np.float64)
    for gq in range(Lsum.shape[2]):
        R += s[None, :, gq] * (0.5 * Lsum[:, :, gq] + (mid - z[None, :, gq]) * S[:, gq][:, None])
    return R


def lut_mpgemm_fp16_tree(act, q, bits, scales=None, zeros=None, group=0, weight_scale=1.0,
                         zero_point=0.0, g=4):
    """The oracle's LUT route with the tables of ``precompute_lut_fp16_tree``; sums of looked-up
    entries stay in fp64."""
    q = np.asarray(q)
    M, K = q.shape
    G = K if group == 0 else group
    nq = K // G
    if group == 0:
        s = np.full((M, 1), np.float64(weight_scale))
        z = np.full((M, 1), np.float64(zero_point))
    else:
        s = np.asarray(scales).astype(np.float64)
        z = np.asarray(zeros).astype(np.float64)
    lut = precompute_lut_fp16_tree(act, g)
    S = orc.group_sums(act, G).astype(np.float64)
    Lsum = np.zeros((lut.shape[0], M, nq), dtype=np.float64)
    for i, plane in enumerate(orc.bit_planes(q, bits)):
        Lsum += (2.0 ** i) * orc.lookup_sum(lut, orc.group_indices(plane, g), G // g).astype(np.float64)
    return _finish(Lsum, S, s, z, bits)


def lut_mpgemm_narrow(act, q, bits, scales, zeros, group, g=4, tables_per_sum=8):
    """The LUT route with fp16 tables built by fp16 additions and the narrow running sum of
    ``lookup_sum_narrow`` (group scales only)."""
    q = np.asarray(q)
    M, K = q.shape
    nq = K // group
    s = np.asarray(scales).astype(np.float64)
    z = np.asarray(zeros).astype(np.float64)
    lut = precompute_lut_fp16_tree(act, g)
    S = orc.group_sums(act, group).astype(np.float64)
    Lsum = np.zeros((lut.shape[0], M, nq), dtype=np.float64)
    for i, plane in enumerate(orc.bit_planes(q, bits)):
        Lsum += (2.0 ** i) * lookup_sum_narrow(lut, orc.group_indices(plane, g), group // g, tables_per_sum)
    return _finish(Lsum, S, s, z, bits)
