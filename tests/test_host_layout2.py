"""CPU-side tests of packed layout 2 (8-row tiles, 16-k units, mirror-folded indices),
checked with an unpacker written here from the layout documented in include/tmac.h."""
import struct

import numpy as np
import pytest

import paper_2407_00088_amd as T
from paper_2407_00088_amd import binding as B


def unfold(code):
    """Stored code {negate, 3-bit entry} -> original 4-bit index (T[p] = -T[15-p])."""
    return np.where(code < 8, code, 15 - (code & 7))


def byte_meaning(bits, d, y):
    """(low row, high row, plane) that byte y of dword d stands for."""
    if bits == 4:
        return 2 * d, 2 * d + 1, y
    if bits == 2 or (bits == 3 and d < 2):
        return 4 * d + y // 2, 4 * d + 2 + y // 2, y % 2
    if bits == 1:
        return y, 4 + y, 0
    return y, 4 + y, 2            # bits == 3, dword 2


def unpack_layout2(blob: np.ndarray):
    raw = blob.tobytes()
    (magic, layout, M, K, bits, g, group, Mp, Kp, n_tiles, n_units, n_qgroups, zero_point, _r0,
     idx_off, idx_bytes, sz_off, sz_bytes, total) = struct.unpack_from("<II10ifI5Q", raw, 0)
    assert magic == 0x43414D54 and layout == 2 and g == 4
    assert Mp == (M + 7) // 8 * 8 and Kp == (K + 127) // 128 * 128 and n_units == Kp // 16
    assert total == len(raw) and idx_bytes == n_tiles * n_units * 16 * bits
    flat = np.frombuffer(raw, dtype="<u4", count=idx_bytes // 4, offset=idx_off).reshape(n_tiles, n_units * 4 * bits)
    # undo the block order: the n_units / 8 chunks (8 units = 128 k each) are split into
    # ceil(chunks / 8) blocks; inside a block of ng chunks starting at chunk c0, unit
    # 8 * (c0 + j) + pos sits in slot pos * ng + j, and 16-byte piece i of the record in slot s
    # is stored at (i * 8 * ng + s)
    rec = np.zeros((n_tiles, n_units, 4 * bits), dtype=np.uint32)
    n_chunks = n_units // 8
    nB = (n_chunks + 7) // 8
    qq, rr = divmod(n_chunks, nB)
    for blk in range(nB):
        c0 = blk * qq + min(blk, rr)
        ng = qq + 1 if blk < rr else qq
        nu = 8 * ng
        span = flat[:, 8 * c0 * 4 * bits: (8 * c0 + nu) * 4 * bits].reshape(n_tiles, bits, nu, 4)
        by_slot = span.transpose(0, 2, 1, 3).reshape(n_tiles, nu, 4 * bits)
        for j in range(ng):
            for pos in range(8):
                rec[:, 8 * (c0 + j) + pos, :] = by_slot[:, pos * ng + j, :]
    idx = rec.reshape(n_tiles, n_units, 4, bits)
    q = np.zeros((Mp, Kp), dtype=np.uint8)
    for tb in range(4):
        for d in range(bits):
            for y in range(4):
                r_lo, r_hi, plane = byte_meaning(bits, d, y)
                byte = (idx[:, :, tb, d] >> (8 * y)) & 0xFF            # [tiles, units]
                for code, r in ((byte & 15, r_lo), (byte >> 4, r_hi)):
                    p = unfold(code.astype(np.int64))
                    for e in range(4):
                        bit = ((p >> e) & 1).astype(np.uint8)
                        rows = np.arange(n_tiles) * 8 + r
                        cols = np.arange(n_units) * 16 + 4 * tb + e
                        q[np.ix_(rows, cols)] |= bit << plane
    s = z = None
    if group > 0:
        sz = np.frombuffer(raw, dtype="<u2", count=sz_bytes // 2, offset=sz_off).reshape(n_tiles, n_qgroups, 8, 2)
        s = sz[..., 0].transpose(0, 2, 1).reshape(Mp, n_qgroups).view(np.float16)
        z = sz[..., 1].transpose(0, 2, 1).reshape(Mp, n_qgroups).view(np.float16)
    hdr = dict(M=M, K=K, bits=bits, group=group, Mp=Mp, Kp=Kp, zero_point=zero_point, n_qgroups=n_qgroups)
    return hdr, q, s, z


def desc2(M, K, bits, group, zero_point=0.0):
    return T.wdesc(M, K, bits, group, zero_point=zero_point, layout=B.TMAC_LAYOUT_R8U16)


@pytest.mark.parametrize("M,K,bits,group", [
    (256, 256, 2, 32), (37, 192, 4, 64), (8, 128, 1, 128), (45, 384, 3, 128),
    (33, 320, 2, 0), (20, 64, 4, 16), (64, 512, 4, 256), (9, 4, 3, 4), (17, 1040, 1, 208),
])
def test_layout2_roundtrip_random(M, K, bits, group):
    rng = np.random.default_rng(M * 1000 + K + bits)
    q = rng.integers(0, 1 << bits, size=(M, K), dtype=np.uint8)
    s = z = None
    if group > 0:
        s = rng.uniform(0.01, 0.1, size=(M, K // group)).astype(np.float16)
        z = rng.uniform(0, (1 << bits) - 1, size=(M, K // group)).astype(np.float16)
    blob = T.tmac_pack_weights(desc2(M, K, bits, group, 1.0 if group == 0 else 0.0), q, s, z)
    hdr, q2, s2, z2 = unpack_layout2(blob)
    assert (hdr["M"], hdr["K"], hdr["bits"], hdr["group"]) == (M, K, bits, group)
    assert np.array_equal(q2[:M, :K], q)
    assert not q2[M:].any() and not q2[:, K:].any()
    if group > 0:
        assert np.array_equal(s2[:M].view(np.uint16), s.view(np.uint16))
        assert np.array_equal(z2[:M].view(np.uint16), z.view(np.uint16))
        assert not s2[M:].view(np.uint16).any()
    else:
        assert hdr["zero_point"] == 1.0 and hdr["n_qgroups"] == 0


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_layout2_special_matrices(bits):
    M, K = 24, 256
    d = desc2(M, K, bits, 0)
    top = (1 << bits) - 1
    for q in (np.zeros((M, K), np.uint8), np.full((M, K), top, np.uint8)):
        _, q2, _, _ = unpack_layout2(T.tmac_pack_weights(d, q))
        assert np.array_equal(q2, q)
    # all-max codes: every index is 15, stored as {negate, entry 0} = 8 -> exactly one bit per
    # stored nibble inside the matrix, none in the padding
    blob = T.tmac_pack_weights(d, np.full((M, K), top, np.uint8))
    idx_off, idx_bytes = struct.unpack_from("<2Q", blob.tobytes(), 56)
    ones = int(np.unpackbits(blob[idx_off: idx_off + idx_bytes]).sum())
    assert ones == M * (K // 4) * bits
    for (m, k) in ((0, 0), (17, 133), (23, 255)):
        q = np.zeros((M, K), np.uint8)
        q[m, k] = top
        _, q2, _, _ = unpack_layout2(T.tmac_pack_weights(d, q))
        assert np.array_equal(q2, q)


def test_mirror_fold_matches_table_symmetry():
    """The stored code must select an entry whose (possibly negated) value equals T[p]:
    checked against the oracle's full table for all 16 indices."""
    from oracle import tmac_oracle as orc
    a = np.array([[3.0, -5.0, 7.0, 11.0]])
    lut = orc.precompute_lut(a, 4)[0, 0]
    half = orc.mirror_half(lut)
    # one row per index value p: weights chosen so that plane 0 of row p has index p
    q = np.array([[(p >> e) & 1 for e in range(4)] for p in range(16)], dtype=np.uint8)
    blob = T.tmac_pack_weights(desc2(16, 4, 1, 0), q)
    raw = blob.tobytes()
    idx_off = struct.unpack_from("<Q", raw, 56)[0]
    n_units = 128 // 16
    idx = np.frombuffer(raw, dtype="<u4", count=2 * n_units * 4, offset=idx_off).reshape(2, n_units, 4, 1)
    for p in range(16):
        tile, r = divmod(p, 8)
        word = int(idx[tile, 0, 0, 0])
        y = r % 4
        code = (word >> (8 * y + (4 if r >= 4 else 0))) & 15
        val = -half[code & 7] if code & 8 else half[code & 7]
        assert val == lut[p]


def test_layout2_sizes_and_group_rules():
    d = desc2(4096, 4096, 4, 128)
    assert T.tmac_packed_bytes(d) == 256 + 4096 * 4096 // 2 + 4096 * 32 * 4
    assert T.tmac_workspace_bytes(d, 1) == 256
    # LUT buffer: tables, group sums, per-16 sums, per-128 sums, half tables, zero slot
    assert T.tmac_lut_bytes(1, 4096, 128, B.TMAC_LUT_F16) == 4096 * 8 + 256 + 1024 + 256 + 4096 * 4 + 256
    import ctypes as C
    fake = C.c_void_p(0x1000)
    g24 = desc2(16, 192, 2, 24)      # valid (24 % 4 == 0) but not a multiple of 16
    st = B.lib.tmac_mpgemm(C.byref(g24), fake, fake, 0, 1, None, C.c_float(1.0), fake, 0, 16, fake, 1 << 20, None)
    assert st == B.TMAC_EUNSUPPORTED
    ok = desc2(16, 192, 2, 48)
    tun = B.tmac_tuning(4, 0, 0)
    st = B.lib.tmac_mpgemm_ex(C.byref(ok), fake, fake, 0, 1, None, C.c_float(1.0), fake, 0, 16, fake, 1 << 20,
                              None, C.byref(tun))
    assert st == B.TMAC_EUNSUPPORTED   # launch-shape knobs belong to the LDS kernels
    st = B.lib.tmac_mpgemm(C.byref(ok), fake, fake, 0, 1, None, C.c_float(1.0), fake, B.TMAC_OUT_I32, 16, fake,
                           1 << 20, None)
    assert st == B.TMAC_EINVAL         # integer output needs integer tables
