"""CPU-side tests of the library's host logic: exported symbols, the offline packer
(checked with the unpackers of blob_unpack.py, written from the layouts documented in include/tmac.h),
buffer-size queries and every argument check that returns before a launch."""
import ctypes as C
import os
import re
import struct

import numpy as np
import pytest

import paper_2407_00088_amd as T
from blob_unpack import unpack_layout3
from paper_2407_00088_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    src = open(os.path.join(ROOT, "include", "tmac.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = set(re.findall(r"\b(tmac_[a-z0-9_]+)\s*\(", src))
    assert {"tmac_pack_weights", "tmac_precompute_lut", "tmac_mpgemm"} <= names
    for n in names:
        assert hasattr(B.lib, n), n
    assert names == set(B.EXPORTS)
    assert T.tmac_version() >= 1


def test_bench_library_exports_every_declared_symbol():
    """The measurement helpers live in a library of their own, declared in include/tmac_bench.h."""
    from paper_2407_00088_amd import bench_helpers as H
    src = open(os.path.join(ROOT, "include", "tmac_bench.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = set(re.findall(r"\b(tmac_bench_[a-z0-9_]+)\s*\(", src))
    assert names == set(H.EXPORTS) and len(names) == 4
    for n in names:
        assert hasattr(H.lib, n), n
        assert not hasattr(B.lib, n), n       # not part of the product library


# the default packed layout (3) is the one these generic tests pack into
def unpack_blob(blob):
    return unpack_layout3(blob)


@pytest.mark.parametrize("M,K,bits,group", [
    (256, 256, 2, 32), (37, 192, 4, 64), (16, 128, 1, 128), (48, 384, 3, 128),
    (33, 320, 2, 0), (20, 64, 4, 64), (64, 512, 4, 256),
])
def test_pack_roundtrip_random(M, K, bits, group):
    rng = np.random.default_rng(M * 1000 + K + bits)
    q = rng.integers(0, 1 << bits, size=(M, K), dtype=np.uint8)
    s = z = None
    if group > 0:
        s = rng.uniform(0.01, 0.1, size=(M, K // group)).astype(np.float16)
        z = rng.uniform(0, (1 << bits) - 1, size=(M, K // group)).astype(np.float16)
    d = T.wdesc(M, K, bits, group, zero_point=1.0 if group == 0 else 0.0)
    blob = T.tmac_pack_weights(d, q, s, z)
    hdr, q2, s2, z2 = unpack_blob(blob)
    assert (hdr["M"], hdr["K"], hdr["bits"], hdr["group"]) == (M, K, bits, group)
    assert np.array_equal(q2[:M, :K], q)
    assert not q2[M:].any() and not q2[:, K:].any()          # padding is index 0
    if group > 0:
        assert np.array_equal(s2[:M].view(np.uint16), s.view(np.uint16))
        assert np.array_equal(z2[:M].view(np.uint16), z.view(np.uint16))
        assert not s2[M:].view(np.uint16).any()
    else:
        assert hdr["zero_point"] == 1.0 and hdr["n_qgroups"] == 0


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_pack_special_matrices(bits):
    M, K = 32, 256
    d = T.wdesc(M, K, bits, 0)
    top = (1 << bits) - 1
    for q in (np.zeros((M, K), np.uint8), np.full((M, K), top, np.uint8)):
        _, q2, _, _ = unpack_blob(T.tmac_pack_weights(d, q))
        assert np.array_equal(q2[:M, :K], q) and not q2[M:].any()
    # every index nibble inside the matrix is covered exactly once: all-max codes set
    # exactly M*K*bits bits in the index region
    blob = T.tmac_pack_weights(d, np.full((M, K), top, np.uint8))
    idx_off, idx_bytes = struct.unpack_from("<2Q", blob.tobytes(), 56)
    ones = int(np.unpackbits(blob[idx_off: idx_off + idx_bytes]).sum())
    assert ones == M * K * bits
    # single-hot
    for (m, k) in ((0, 0), (17, 133), (31, 255)):
        q = np.zeros((M, K), np.uint8)
        q[m, k] = top
        _, q2, _, _ = unpack_blob(T.tmac_pack_weights(d, q))
        assert np.array_equal(q2[:M, :K], q) and not q2[M:].any()


def test_null_zeros_means_mid_level():
    M, K, bits, G = 16, 128, 4, 128
    q = np.zeros((M, K), np.uint8)
    s = np.full((M, 1), 0.5, np.float16)
    _, _, s2, z2 = unpack_blob(T.tmac_pack_weights(T.wdesc(M, K, bits, G), q, s, None))
    assert np.all(z2[:M] == np.float16(7.5)) and np.all(s2[:M] == np.float16(0.5))


def test_sizes():
    d = T.wdesc(4096, 4096, 4, 128)
    idx = 4096 * 4096 // 2
    sz = 4096 * 32 * 4
    assert T.tmac_packed_bytes(d) == 256 + idx + sz
    # tables (8 bytes per k, for whole n tiles of 4 or 8 activation rows) + group sums (one 256-byte
    # block) + per-16 sums (4 bytes per 16 k, 256-aligned) + per-128 sums (4 bytes per 128 k,
    # 256-aligned) + fp16 half tables (4 bytes per k) (+ one 256-byte tail holding an all-zero table)
    assert T.tmac_lut_bytes(1, 4096, 128, B.TMAC_LUT_F16) == 4 * 4096 * 8 + 256 + 1024 + 256 + 4096 * 4 + 256
    assert T.tmac_lut_bytes(1, 3200, 0, B.TMAC_LUT_I16) == 4 * 3200 * 8 + 256 + 1024 + 256 + 3200 * 4 + 256
    # K padded to 128 inside the LUT
    assert T.tmac_lut_bytes(2, 8640, 0, B.TMAC_LUT_I16) == 4 * 8704 * 8 + 256 + 4352 + 768 + 2 * 8704 * 4 + 256
    # n tiles: four rows up to N = 4, eight from five on where that wastes at most a fifth
    assert T.tmac_lut_bytes(6, 4096, 128, B.TMAC_LUT_F16) - T.tmac_lut_bytes(5, 4096, 128, B.TMAC_LUT_F16) == \
        1024 + 4096 * 4                                        # same 8 table rows; one more row of per-16 sums and half tables
    assert T.tmac_lut_bytes(9, 4096, 128, B.TMAC_LUT_F16) > 12 * 4096 * 8
    assert T.tmac_workspace_bytes(d, 1) > 0


# ------------------------------------------------------------- error paths ----

def _desc(**kw):
    base = dict(M=16, K=128, bits=2, group=0)
    base.update(kw)
    d = T.wdesc(base["M"], base["K"], base["bits"], base["group"])
    for k in ("g", "layout", "reserved"):
        if k in kw:
            setattr(d, k, kw[k])
    return d


@pytest.mark.parametrize("kw", [dict(bits=0), dict(bits=5), dict(g=3), dict(g=16), dict(g=8, layout=2), dict(K=126),
                                dict(K=132, g=8), dict(M=0), dict(group=48), dict(group=6), dict(group=4, g=8),
                                dict(layout=7), dict(layout=1), dict(reserved=1)])
def test_bad_desc_is_rejected(kw):
    d = _desc(**kw)
    assert T.tmac_packed_bytes(d) == 0
    q = np.zeros((max(d.M, 1), max(d.K, 1)), np.uint8)
    buf = np.zeros(1 << 16, np.uint8)
    st = B.lib.tmac_pack_weights(C.byref(d), q.ctypes.data, None, None, buf.ctypes.data, buf.size)
    assert st == B.TMAC_EINVAL
    assert B.lib.tmac_workspace_bytes(C.byref(d), 1) == 0


def test_pack_argument_errors():
    d = _desc()
    q = np.zeros((16, 128), np.uint8)
    n = T.tmac_packed_bytes(d)
    buf = np.zeros(n, np.uint8)
    assert B.lib.tmac_pack_weights(C.byref(d), None, None, None, buf.ctypes.data, n) == B.TMAC_EINVAL
    assert B.lib.tmac_pack_weights(C.byref(d), q.ctypes.data, None, None, None, n) == B.TMAC_EINVAL
    assert B.lib.tmac_pack_weights(C.byref(d), q.ctypes.data, None, None, buf.ctypes.data, n - 1) == B.TMAC_ESIZE
    q[3, 5] = 4  # code out of range for 2 bits
    assert B.lib.tmac_pack_weights(C.byref(d), q.ctypes.data, None, None, buf.ctypes.data, n) == B.TMAC_EINVAL
    dg = _desc(group=64)
    q[3, 5] = 0
    buf2 = np.zeros(T.tmac_packed_bytes(dg), np.uint8)
    # group scales requested but no scales given
    assert B.lib.tmac_pack_weights(C.byref(dg), q.ctypes.data, None, None, buf2.ctypes.data, buf2.size) == B.TMAC_EINVAL
    with pytest.raises(T.TmacError):
        T.tmac_pack_weights(d, np.full((16, 128), 9, np.uint8))


def test_device_entry_points_reject_bad_arguments_before_launch():
    """None of these calls reaches a launch, so they are safe without a GPU."""
    lib = B.lib
    fake = C.c_void_p(0x1000)          # never dereferenced: every call fails its checks first
    odd = C.c_void_p(0x1004)
    assert lib.tmac_lut_bytes(1, 126, 4, 0, 0) == 0
    assert lib.tmac_lut_bytes(1, 128, 3, 0, 0) == 0
    assert lib.tmac_lut_bytes(0, 128, 4, 0, 0) == 0
    assert lib.tmac_lut_bytes(1, 128, 4, 0, 7) == 0
    P = lib.tmac_precompute_lut
    assert P(None, 0, 1, 128, 128, 4, 0, 0, fake, 1 << 20, None) == B.TMAC_EINVAL
    assert P(fake, 0, 1, 128, 128, 4, 0, 0, None, 1 << 20, None) == B.TMAC_EINVAL
    assert P(fake, 0, 1, 128, 128, 4, 0, 1, fake, 1 << 20, None) == B.TMAC_EINVAL   # f16 act, i16 lut
    assert P(fake, 1, 1, 128, 128, 4, 0, 0, fake, 1 << 20, None) == B.TMAC_EINVAL   # i8 act, f16 lut
    assert P(fake, 0, 1, 126, 128, 4, 0, 0, fake, 1 << 20, None) == B.TMAC_EINVAL   # K % 4
    assert P(fake, 0, 1, 128, 64, 4, 0, 0, fake, 1 << 20, None) == B.TMAC_EINVAL    # lda < K
    assert P(fake, 0, 1, 128, 128, 4, 0, 0, odd, 1 << 20, None) == B.TMAC_EINVAL    # misaligned
    assert P(fake, 0, 1, 128, 128, 4, 0, 0, fake, 16, None) == B.TMAC_ESIZE
    d = _desc(M=16, K=128, bits=2, group=0)
    G = lib.tmac_mpgemm
    ok_args = [C.byref(d), fake, fake, 0, 1, None, C.c_float(1.0), fake, 0, 16, fake, 1 << 20, None]

    def call(**over):
        a = list(ok_args)
        for k, v in over.items():
            a[int(k[1:])] = v
        return G(*a)
    assert call(a1=None) == B.TMAC_EINVAL
    assert call(a2=None) == B.TMAC_EINVAL
    assert call(a7=None) == B.TMAC_EINVAL
    assert call(a1=odd) == B.TMAC_EINVAL
    assert call(a3=5) == B.TMAC_EINVAL
    assert call(a8=9) == B.TMAC_EINVAL
    assert call(a4=0) == B.TMAC_EINVAL
    assert call(a9=8) == B.TMAC_EINVAL                 # ldo < M
    assert call(a8=B.TMAC_OUT_I32) == B.TMAC_EINVAL    # int output from fp16 tables
    bad = _desc(bits=7)
    assert call(a0=C.byref(bad)) == B.TMAC_EINVAL
    g48 = _desc(M=16, K=192, bits=2, group=48)          # layout 3 needs whole 32-k chunks per group
    assert call(a0=C.byref(g48), a9=16) == B.TMAC_EUNSUPPORTED
    assert T.status_str(B.TMAC_ESIZE) == "buffer too small"


def test_blob_check_accepts_its_own_header_and_rejects_every_mismatch():
    """tmac_blob_check: the host-side check of a blob header against a desc."""
    rng = np.random.default_rng(5)
    for layout in (B.TMAC_LAYOUT_R8U16, B.TMAC_LAYOUT_R64K32):
        d = T.wdesc(40, 256, 3, 64, layout=layout)
        q = rng.integers(0, 8, size=(40, 256), dtype=np.uint8)
        s = rng.uniform(0.01, 0.1, size=(40, 4)).astype(np.float16)
        blob = T.tmac_pack_weights(d, q, s, None)
        assert B.tmac_blob_check(d, blob[:256]) == B.TMAC_OK
        assert B.tmac_blob_check(d, blob) == B.TMAC_OK
        for other in (T.wdesc(48, 256, 3, 64, layout=layout), T.wdesc(40, 512, 3, 64, layout=layout),
                      T.wdesc(40, 256, 2, 64, layout=layout), T.wdesc(40, 256, 3, 128, layout=layout),
                      T.wdesc(40, 256, 3, 0, layout=layout),
                      T.wdesc(40, 256, 3, 64, layout=5 - layout)):
            assert B.tmac_blob_check(other, blob[:256]) == B.TMAC_EINVAL
        bad = blob[:256].copy()
        bad[0] ^= 1                                   # magic
        assert B.tmac_blob_check(d, bad) == B.TMAC_EINVAL
        bad = blob[:256].copy()
        bad[struct.calcsize("<II10i") + 8 + 8] ^= 0x40   # one of the size fields
        assert B.tmac_blob_check(d, bad) == B.TMAC_EINVAL
    # per-tensor zero point is part of the header
    d0 = T.wdesc(16, 128, 2, 0, zero_point=1.0)
    blob0 = T.tmac_pack_weights(d0, np.zeros((16, 128), np.uint8))
    assert B.tmac_blob_check(d0, blob0[:256]) == B.TMAC_OK
    assert B.tmac_blob_check(T.wdesc(16, 128, 2, 0, zero_point=2.0), blob0[:256]) == B.TMAC_EINVAL
    assert B.lib.tmac_blob_check(None, blob0.ctypes.data) == B.TMAC_EINVAL
    assert B.lib.tmac_blob_check(C.byref(d0), None) == B.TMAC_EINVAL
    assert B.lib.tmac_blob_check(C.byref(_desc(bits=9)), blob0.ctypes.data) == B.TMAC_EINVAL


@pytest.mark.parametrize("K,g,group,lut", [(4096, 4, 128, 0), (3200, 4, 0, 1), (4096, 4, 128, 2), (1024, 2, 64, 0),
                                           (1024, 8, 64, 1), (136, 4, 136, 0)])
def test_largest_buffer_sizes_equal_the_brute_force_maximum(K, g, group, lut):
    """tmac_lut_bytes_max / tmac_workspace_bytes_max / tmac_fused_workspace_bytes_max against the
    maximum taken by calling the per-N queries one by one."""
    for n_max in (1, 3, 4, 5, 8, 9, 12, 13, 33, 39, 40, 41, 64, 65, 100, 300):
        sizes = [B.tmac_lut_bytes(n, K, group, lut, g=g) for n in range(1, n_max + 1)]
        want = 0 if all(v == 0 for v in sizes) else max(sizes)
        assert B.tmac_lut_bytes_max(n_max, K, group, lut, g=g) == want, n_max
    assert B.tmac_lut_bytes_max(0, K, group, lut, g=g) == 0
    if lut == 2:
        return
    for layout in (B.TMAC_LAYOUT_R8U16, B.TMAC_LAYOUT_R64K32):
        if g != 4 and layout == B.TMAC_LAYOUT_R8U16:
            continue
        d = T.wdesc(300, K, 4, group, g=g, layout=layout)
        for n_max in (1, 7, 33, 70, 200):
            assert B.tmac_workspace_bytes_max(d, n_max) == max(B.tmac_workspace_bytes(d, n) for n in range(1, n_max + 1))
            per_n = [B.tmac_fused_workspace_bytes(d, n, lut) for n in range(1, n_max + 1)]
            assert B.tmac_fused_workspace_bytes_max(d, n_max, lut) == (0 if 0 in per_n else max(per_n))
    assert B.tmac_workspace_bytes_max(_desc(bits=9), 4) == 0


def test_multi_call_rejects_bad_arguments_before_launch():
    """tmac_mpgemv_fused_multi: every check happens on the host before the launch."""
    lib = B.lib
    fake, odd = 0x1000, 0x1004
    d = T.wdesc(64, 256, 4, 128, layout=B.TMAC_LAYOUT_R8U16)
    d2 = T.wdesc(64, 512, 2, 128, layout=B.TMAC_LAYOUT_R8U16)      # other bit-width
    d3 = T.wdesc(64, 256, 4, 32, layout=B.TMAC_LAYOUT_R8U16)       # other grouping mode (per lane, not per chunk)
    d4 = T.wdesc(64, 256, 4, 128, layout=B.TMAC_LAYOUT_R64K32)     # batched layout

    def item(desc, packed=fake, A=fake, lda=None, out=fake, ldo=None):
        return B.tmac_gemv_item(C.pointer(desc), packed, A, desc.K if lda is None else lda, None, 1.0, out,
                                desc.M if ldo is None else ldo)

    def call(items, count=None, act=0, N=1, out=0, tuning=None):
        arr = (B.tmac_gemv_item * max(len(items), 1))(*items)
        return lib.tmac_mpgemv_fused_multi(arr, len(items) if count is None else count, act, N, out, None, tuning)

    assert lib.tmac_mpgemv_fused_multi(None, 1, 0, 1, 0, None, None) == B.TMAC_EINVAL
    assert call([item(d)], count=0) == B.TMAC_EUNSUPPORTED
    assert call([item(d)] * 9) == B.TMAC_EUNSUPPORTED
    assert call([item(d)], N=0) == B.TMAC_EINVAL
    assert call([item(d)], act=3) == B.TMAC_EINVAL
    assert call([item(d)], out=7) == B.TMAC_EINVAL
    assert call([item(d, packed=None)]) == B.TMAC_EINVAL
    assert call([item(d), item(d, A=odd)]) == B.TMAC_EINVAL
    assert call([item(d), item(d, out=None)]) == B.TMAC_EINVAL
    assert call([item(d, lda=128)]) == B.TMAC_EINVAL
    assert call([item(d, lda=260)]) == B.TMAC_EINVAL               # not a multiple of 8 elements
    assert call([item(d, ldo=8)]) == B.TMAC_EINVAL
    assert call([item(d4)]) == B.TMAC_EUNSUPPORTED
    assert call([item(d), item(d2)]) == B.TMAC_EUNSUPPORTED
    assert call([item(d), item(d3)]) == B.TMAC_EUNSUPPORTED
    assert call([item(d)], out=B.TMAC_OUT_I32) == B.TMAC_EINVAL    # raw integers from fp16 tables
    assert call([item(d)], tuning=C.byref(B.tmac_tuning(12))) == B.TMAC_EINVAL
    # tables quantised in the kernel: fp results only
    assert call([item(d)], act=B.TMAC_ACT_F16_TQ, out=B.TMAC_OUT_I32) == B.TMAC_EINVAL


def test_fused_call_refuses_sizes_beyond_its_index_arithmetic_before_launch():
    """The register-table kernel counts units in 16 bits, slots in 32 bits and activation rows in the
    grid's y dimension: larger calls are refused on the host (fake pointers: nothing is launched)."""
    lib = B.lib
    fake = C.c_void_p(0x1000)
    F = lib.tmac_mpgemv_fused

    def call(desc, N=1, act=0, lda=None):
        return F(C.byref(desc), fake, fake, act, N, desc.K if lda is None else lda, None, C.c_float(1.0), fake, 0,
                 desc.M, None)
    ok = T.wdesc(64, 256, 4, 128, layout=B.TMAC_LAYOUT_R8U16)
    assert call(ok, N=65536) == B.TMAC_EUNSUPPORTED                       # grid y
    assert call(ok, N=0) == B.TMAC_EINVAL
    long_k = T.wdesc(8, 1 << 20, 4, 128, layout=B.TMAC_LAYOUT_R8U16)      # 65536 units of 16 k
    assert call(long_k) == B.TMAC_EUNSUPPORTED
    many = T.wdesc(1 << 22, 1 << 19, 4, 128, layout=B.TMAC_LAYOUT_R8U16)  # row tiles x units x bits >= 2^32
    assert call(many) == B.TMAC_EUNSUPPORTED
    assert call(ok, act=B.TMAC_ACT_F16_TQ, N=65536) == B.TMAC_EUNSUPPORTED
    # int8 activations with one scale per row: the row sum travels in fp32 and must stay below 2^24
    long_int = T.wdesc(8, 1 << 18, 2, 0, layout=B.TMAC_LAYOUT_R8U16)
    assert call(long_int, act=B.TMAC_ACT_I8) == B.TMAC_EUNSUPPORTED


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's throughput; --gpus N with N > 1 ends with a message and a
    non-zero status before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
