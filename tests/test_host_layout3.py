"""CPU-side tests of packed layout 3 (64-row tiles, one lane per row, chunks of 32 k), checked
with the unpacker of blob_unpack.py, written from the layout documented in include/tmac.h."""
import numpy as np
import pytest

from blob_unpack import unpack_layout3

import paper_2407_00088_amd as T
from paper_2407_00088_amd import binding as B


def desc3(M, K, bits, group, zero_point=0.0):
    return T.wdesc(M, K, bits, group, zero_point=zero_point, layout=B.TMAC_LAYOUT_R64K32)


@pytest.mark.parametrize("M,K,bits,group", [(256, 256, 2, 32), (37, 192, 4, 64), (64, 128, 1, 128), (130, 384, 3, 96),
                                            (5, 36, 4, 36), (70, 200, 2, 0)])
def test_layout3_roundtrip_random(M, K, bits, group):
    rng = np.random.default_rng(M * 7 + K + bits)
    q = rng.integers(0, 1 << bits, size=(M, K), dtype=np.uint8)
    ng = K // group if group else 0
    s = rng.uniform(0.01, 0.1, size=(M, ng)).astype(np.float16) if group else None
    z = rng.uniform(0, (1 << bits) - 1, size=(M, ng)).astype(np.float16) if group else None
    blob = T.tmac_pack_weights(desc3(M, K, bits, group), q, s, z)
    hdr, q2, s2, z2 = unpack_layout3(blob)
    assert (hdr["M"], hdr["K"], hdr["bits"], hdr["group"]) == (M, K, bits, group)
    assert np.array_equal(q2[:M, :K], q)
    assert not q2[M:].any() and not q2[:, K:].any()          # padding is index 0
    if group:
        assert np.array_equal(s2[:M].view(np.uint16), s.view(np.uint16))
        assert np.array_equal(z2[:M].view(np.uint16), z.view(np.uint16))


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_layout3_special_matrices(bits):
    M, K = 66, 160
    top = (1 << bits) - 1
    for q in (np.zeros((M, K), np.uint8), np.full((M, K), top, np.uint8)):
        _, q2, _, _ = unpack_layout3(T.tmac_pack_weights(desc3(M, K, bits, 0), q))
        assert np.array_equal(q2[:M, :K], q)
    q = np.zeros((M, K), np.uint8)
    q[65, 159] = top
    q[0, 0] = 1
    _, q2, _, _ = unpack_layout3(T.tmac_pack_weights(desc3(M, K, bits, 0), q))
    assert np.array_equal(q2[:M, :K], q)


def test_layout3_sizes_and_group_rules():
    d = desc3(5120, 5120, 4, 128)
    assert T.tmac_packed_bytes(d) == 256 + 5120 * 5120 // 2 + 5120 * 40 * 4
    assert T.tmac_workspace_bytes(d, 4096) == 256            # enough (row block, n tile) pairs: K is not split
    # 256 rows: a workgroup takes two n tiles of 8 rows: 16 x 20 (n tile pair, row block) pairs; K is
    # split in 10 slices of 16 chunks (two LDS slices) each: partial sums [10][256][5120] fp32, one
    # counter per pair, 256 spare bytes
    assert T.tmac_workspace_bytes(d, 256) == 10 * 256 * 5120 * 4 + 256   # ten K slices of partial sums, nothing else
    assert T.tmac_workspace_bytes(d, 4) > 4 * 5120 * 4        # few rows: partial sums of the K slices
    assert T.tmac_packed_bytes(desc3(100, 48, 2, 16)) > 0     # packs; the kernel rejects the group size


@pytest.mark.parametrize("g", [2, 8])
def test_index_region_does_not_depend_on_g(g):
    """Bit t of an index dword is bit plane i of q[m][32c+t]: the same bytes serve g = 2, 4, 8;
    only the header's g field differs."""
    rng = np.random.default_rng(40 + g)
    M, K, bits = 70, 160, 3
    q = rng.integers(0, 1 << bits, size=(M, K), dtype=np.uint8)
    s = rng.uniform(0.01, 0.1, size=(M, K // 32)).astype(np.float16)
    z = rng.uniform(0, 7, size=(M, K // 32)).astype(np.float16)
    b4 = T.tmac_pack_weights(desc3(M, K, bits, 32), q, s, z)
    bg = T.tmac_pack_weights(T.wdesc(M, K, bits, 32, g=g, layout=B.TMAC_LAYOUT_R64K32), q, s, z)
    assert b4.size == bg.size
    diff = np.flatnonzero(b4 != bg)
    assert diff.size > 0 and diff.max() < 256          # header only
    hdr, q2, _, _ = unpack_layout3(bg)
    assert hdr["g"] == g and np.array_equal(q2[:M, :K], q)


def test_lut_bytes_for_other_group_sizes():
    # tables [n tile][Kp/g][2^g][NT] of 2 bytes (one tile of four rows here), group sums [N][nq] fp32,
    # 256 spare bytes
    assert T.tmac_lut_bytes(3, 4096, 128, B.TMAC_LUT_F16, g=2) == 4 * 2048 * 4 * 2 + 512 + 256
    assert T.tmac_lut_bytes(3, 4096, 128, B.TMAC_LUT_I16, g=8) == 4 * 512 * 256 * 2 + 512 + 256
    assert T.tmac_lut_bytes(1, 4096, 128, B.TMAC_LUT_I8Q, g=8) == 0      # int8 tables: g = 4 only
    assert T.tmac_lut_bytes(1, 4100, 0, B.TMAC_LUT_F16, g=8) == 0        # K % g
    assert T.tmac_lut_bytes(1, 4096, 4, B.TMAC_LUT_F16, g=8) == 0        # group % g


def test_lut_bytes_beyond_the_register_table_kernel():
    """More than 64 activation rows go to the batched kernels only: the buffer then holds the tables
    (n tiles of 8 rows) and the group sums, and int8 tables, which only the register-table kernel
    reads, are refused."""
    assert T.tmac_lut_bytes(64, 4096, 128, B.TMAC_LUT_F16) > 64 * 4096 * 8 + 64 * 32 * 4 + 256
    assert T.tmac_lut_bytes(65, 4096, 128, B.TMAC_LUT_F16) == 72 * 4096 * 8 + (65 * 32 * 4 + 255) // 256 * 256 + 256
    assert T.tmac_lut_bytes(256, 5120, 128, B.TMAC_LUT_I16) == 256 * 5120 * 8 + 256 * 40 * 4 + 256
    assert T.tmac_lut_bytes(64, 4096, 128, B.TMAC_LUT_I8Q) > 0
    assert T.tmac_lut_bytes(65, 4096, 128, B.TMAC_LUT_I8Q) == 0


def test_fused_workspace_regions():
    """tmac_fused_workspace_bytes = tmac_mpgemm's workspace (rounded to 256) plus a LUT buffer only
    where the tables are not built inside the lookup kernel."""
    F16, I8 = B.TMAC_ACT_F16, B.TMAC_ACT_I8
    d = desc3(4096, 4096, 4, 128)
    ws16 = T.tmac_workspace_bytes(d, 16)
    assert B.tmac_fused_workspace_bytes(d, 16, F16) == ws16                      # short slices: in the kernel
    assert B.tmac_fused_workspace_bytes(d, 16, I8) == ws16
    big = desc3(13824, 5120, 4, 128)
    assert B.tmac_fused_workspace_bytes(big, 256, F16) == \
        T.tmac_workspace_bytes(big, 256) + T.tmac_lut_bytes(256, 5120, 128, B.TMAC_LUT_F16)
    row = desc3(4096, 4096, 4, 4096)                                              # one scale per row: in the kernel too
    assert B.tmac_fused_workspace_bytes(row, 16, F16) == T.tmac_workspace_bytes(row, 16)
    assert B.tmac_fused_workspace_bytes(row, 64, F16) == \
        T.tmac_workspace_bytes(row, 64) + T.tmac_lut_bytes(64, 4096, 4096, B.TMAC_LUT_F16)   # more than 32 rows
    g96 = desc3(4096, 4608, 4, 96)                                                # 3 chunks per group
    assert B.tmac_fused_workspace_bytes(g96, 16, F16) > T.tmac_workspace_bytes(g96, 16) + 4608 * 16 * 8
    d2 = T.wdesc(4096, 4096, 4, 128, layout=B.TMAC_LAYOUT_R8U16)
    assert B.tmac_fused_workspace_bytes(d2, 1, F16) == 256                        # register-table kernel builds them
    d2b = T.wdesc(64, 4072, 2, 4072, layout=B.TMAC_LAYOUT_R8U16)
    assert B.tmac_fused_workspace_bytes(d2b, 1, F16) == 256 + T.tmac_lut_bytes(1, 4072, 4072, B.TMAC_LUT_F16)
    assert B.tmac_fused_workspace_bytes(d2b, 64, F16) > 0
    assert B.tmac_fused_workspace_bytes(d2b, 65, F16) == 0     # LUT-buffer route of the register-table kernel: 64 rows at most
    assert B.tmac_fused_workspace_bytes(d2, 65, F16) == 256     # tables built in the kernel: any number of rows
    assert B.tmac_fused_workspace_bytes(d, 0, F16) == 0 and B.tmac_fused_workspace_bytes(d, 1, 7) == 0
