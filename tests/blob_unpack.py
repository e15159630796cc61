"""Unpackers of the packed weight blobs, written from the layouts documented in include/tmac.h and
independent of the packer's code; shared by the host-side tests."""
import struct

import numpy as np


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
                word = idx[:, :, tb, d]
                byte = (word >> (8 * y)) & 0xFF                        # [tiles, units]
                nxt = (word >> (8 * ((y + 1) % 4))) & 0xFF
                # byte y = {negate_low, entry_high (3 bits), negate_high of byte y - 1, entry_low (3 bits)}
                code_lo = (byte & 7) | ((byte >> 7) << 3)
                code_hi = ((byte >> 4) & 7) | (((nxt >> 3) & 1) << 3)
                for code, r in ((code_lo, r_lo), (code_hi, r_hi)):
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


def unpack_layout3(blob: np.ndarray):
    raw = blob.tobytes()
    (magic, layout, M, K, bits, g, group, Mp, Kp, n_tiles, n_chunks, n_qgroups, zero_point, _r0,
     idx_off, idx_bytes, sz_off, sz_bytes, total) = struct.unpack_from("<II10ifI5Q", raw, 0)
    assert magic == 0x43414D54 and layout == 3 and g in (2, 4, 8)
    assert Mp == (M + 63) // 64 * 64 and Kp == (K + 127) // 128 * 128 and n_chunks == Kp // 32
    assert total == len(raw) and idx_bytes == n_tiles * n_chunks * 64 * bits * 4
    idx = np.frombuffer(raw, dtype="<u4", count=idx_bytes // 4, offset=idx_off).reshape(n_tiles, n_chunks, 64, bits)
    q = np.zeros((Mp, Kp), dtype=np.uint8)
    rows = np.arange(Mp)
    for i in range(bits):
        for j in range(8):
            nib = ((idx[:, :, :, i] >> (4 * j)) & 15).transpose(0, 2, 1).reshape(Mp, n_chunks)   # [row, chunk]
            for e in range(4):
                cols = np.arange(n_chunks) * 32 + 4 * j + e
                q[np.ix_(rows, cols)] |= (((nib >> e) & 1) << i).astype(np.uint8)
    s = z = None
    if group > 0:
        sz = np.frombuffer(raw, dtype="<u2", count=sz_bytes // 2, offset=sz_off).reshape(n_tiles, n_qgroups, 64, 2)
        s = sz[..., 0].transpose(0, 2, 1).reshape(Mp, n_qgroups).view(np.float16)
        z = sz[..., 1].transpose(0, 2, 1).reshape(Mp, n_qgroups).view(np.float16)
    return dict(M=M, K=K, bits=bits, g=g, group=group, Mp=Mp, Kp=Kp, zero_point=zero_point,
                n_qgroups=n_qgroups), q, s, z
