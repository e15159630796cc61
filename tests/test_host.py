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
