"""Thin ctypes binding of libtmac_hip.so: argument marshalling only.

Every step of the path (table precompute, lookup, accumulate, scale, reduce) runs in
the library's HIP kernels; the offline packer runs in the library's host code.  torch
is used for device memory and streams only.  There is no fallback: if the shared
library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libtmac_hip.so")

TMAC_OK, TMAC_EINVAL, TMAC_EUNSUPPORTED, TMAC_ESIZE, TMAC_EHIP = range(5)
TMAC_ACT_F16, TMAC_ACT_I8, TMAC_ACT_F16_TQ = 0, 1, 2
TMAC_LUT_F16, TMAC_LUT_I16, TMAC_LUT_I8Q = 0, 1, 2
TMAC_OUT_F32, TMAC_OUT_F16, TMAC_OUT_I32 = 0, 1, 2
TMAC_LAYOUT_R8U16 = 2     # register-table decode kernel (small N)
TMAC_LAYOUT_R64K32 = 3    # batched lookup kernel, lane = weight row (many activation rows)

TMAC_MULTI_MAX = 8

EXPORTS = [
    "tmac_packed_bytes", "tmac_pack_weights", "tmac_lut_bytes", "tmac_precompute_lut",
    "tmac_workspace_bytes", "tmac_mpgemm", "tmac_mpgemm_ex", "tmac_status_str", "tmac_version",
    "tmac_last_error_detail", "tmac_mpgemv_fused", "tmac_mpgemv_fused_ex",
    "tmac_fused_workspace_bytes", "tmac_mpgemm_fused", "tmac_mpgemv_fused_multi", "tmac_blob_check",
    "tmac_lut_bytes_max", "tmac_workspace_bytes_max", "tmac_fused_workspace_bytes_max", "tmac_mpgemm_noalloc",
]


class tmac_wdesc(C.Structure):
    _fields_ = [("M", C.c_int32), ("K", C.c_int32), ("bits", C.c_int32), ("g", C.c_int32),
                ("group", C.c_int32), ("layout", C.c_int32), ("zero_point", C.c_float),
                ("reserved", C.c_int32)]


class tmac_tuning(C.Structure):
    _fields_ = [("rows_per_group", C.c_int32), ("group_waves", C.c_int32), ("workgroup_waves", C.c_int32),
                ("workgroups_per_cu", C.c_int32), ("reserved", C.c_int32 * 4)]


class tmac_gemv_item(C.Structure):
    _fields_ = [("desc", C.POINTER(tmac_wdesc)), ("packed_dev", C.c_void_p), ("A_dev", C.c_void_p),
                ("lda", C.c_int64), ("act_scale_dev", C.c_void_p), ("weight_scale", C.c_float),
                ("out_dev", C.c_void_p), ("ldo", C.c_int64)]


class TmacError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = lib.tmac_last_error_detail().decode() if status in (TMAC_EHIP, TMAC_ESIZE) else ""
        super().__init__(f"{where}: {status_str(status)} (status {status}) {detail}".rstrip())


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no CPU or PyTorch fallback for the HIP path)")
    # torch bundles its own HIP runtime (same soname as ROCm's).  Import torch first so that the
    # library binds to that one runtime instead of pulling a second copy from /opt/rocm: two
    # runtimes in one process do not share streams or devices.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    P, I32, I64, SZ, F = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float
    D = C.POINTER(tmac_wdesc)
    lib.tmac_packed_bytes.restype, lib.tmac_packed_bytes.argtypes = SZ, [D]
    lib.tmac_pack_weights.restype = C.c_int
    lib.tmac_pack_weights.argtypes = [D, P, P, P, P, SZ]
    lib.tmac_lut_bytes.restype, lib.tmac_lut_bytes.argtypes = SZ, [I32, I32, I32, I32, C.c_int]
    lib.tmac_precompute_lut.restype = C.c_int
    lib.tmac_precompute_lut.argtypes = [P, C.c_int, I32, I32, I64, I32, I32, C.c_int, P, SZ, P]
    lib.tmac_workspace_bytes.restype, lib.tmac_workspace_bytes.argtypes = SZ, [D, I32]
    lib.tmac_mpgemm.restype = C.c_int
    lib.tmac_mpgemm.argtypes = [D, P, P, C.c_int, I32, P, F, P, C.c_int, I64, P, SZ, P]
    lib.tmac_mpgemm_ex.restype = C.c_int
    lib.tmac_mpgemm_ex.argtypes = [D, P, P, C.c_int, I32, P, F, P, C.c_int, I64, P, SZ, P,
                                   C.POINTER(tmac_tuning)]
    lib.tmac_mpgemm_noalloc.restype = C.c_int
    lib.tmac_mpgemm_noalloc.argtypes = [D, P, P, C.c_int, I32, P, F, P, C.c_int, I64, P]
    lib.tmac_mpgemv_fused.restype = C.c_int
    lib.tmac_mpgemv_fused.argtypes = [D, P, P, C.c_int, I32, I64, P, F, P, C.c_int, I64, P]
    lib.tmac_mpgemv_fused_ex.restype = C.c_int
    lib.tmac_mpgemv_fused_ex.argtypes = [D, P, P, C.c_int, I32, I64, P, F, P, C.c_int, I64, P, C.POINTER(tmac_tuning)]
    lib.tmac_fused_workspace_bytes.restype, lib.tmac_fused_workspace_bytes.argtypes = SZ, [D, I32, C.c_int]
    lib.tmac_mpgemm_fused.restype = C.c_int
    lib.tmac_mpgemm_fused.argtypes = [D, P, P, C.c_int, I32, I64, P, F, P, C.c_int, I64, P, SZ, P]
    lib.tmac_status_str.restype, lib.tmac_status_str.argtypes = C.c_char_p, [C.c_int]
    lib.tmac_version.restype, lib.tmac_version.argtypes = I32, []
    lib.tmac_last_error_detail.restype, lib.tmac_last_error_detail.argtypes = C.c_char_p, []
    lib.tmac_mpgemv_fused_multi.restype = C.c_int
    lib.tmac_mpgemv_fused_multi.argtypes = [C.POINTER(tmac_gemv_item), I32, C.c_int, I32, C.c_int, P,
                                            C.POINTER(tmac_tuning)]
    lib.tmac_blob_check.restype, lib.tmac_blob_check.argtypes = C.c_int, [D, P]
    lib.tmac_lut_bytes_max.restype, lib.tmac_lut_bytes_max.argtypes = SZ, [I32, I32, I32, I32, C.c_int]
    lib.tmac_workspace_bytes_max.restype, lib.tmac_workspace_bytes_max.argtypes = SZ, [D, I32]
    lib.tmac_fused_workspace_bytes_max.restype = SZ
    lib.tmac_fused_workspace_bytes_max.argtypes = [D, I32, C.c_int]
    return lib


lib = _load()


def status_str(status: int) -> str:
    return lib.tmac_status_str(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != TMAC_OK:
        raise TmacError(status, where)


def wdesc(M: int, K: int, bits: int, group: int, zero_point: float = 0.0, g: int = 4,
          layout: int = TMAC_LAYOUT_R64K32) -> tmac_wdesc:
    return tmac_wdesc(M, K, bits, g, group, layout, float(zero_point), 0)


def tmac_version() -> int:
    return int(lib.tmac_version())


def tmac_packed_bytes(desc: tmac_wdesc) -> int:
    return int(lib.tmac_packed_bytes(C.byref(desc)))


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def tmac_pack_weights(desc: tmac_wdesc, q: np.ndarray, scales: Optional[np.ndarray] = None,
                      zeros: Optional[np.ndarray] = None) -> np.ndarray:
    """Host-side offline packing; returns the blob as a uint8 numpy array."""
    q = np.ascontiguousarray(q, dtype=np.uint8)
    if q.shape != (desc.M, desc.K):
        raise ValueError("q must be [M, K]")
    s16 = None if scales is None else np.ascontiguousarray(scales, dtype=np.float16).view(np.uint16)
    z16 = None if zeros is None else np.ascontiguousarray(zeros, dtype=np.float16).view(np.uint16)
    if desc.group > 0:
        ng = desc.K // desc.group if desc.K % desc.group == 0 else -1
        for a in (s16, z16):
            if a is not None and a.shape != (desc.M, ng):
                raise ValueError("scales/zeros must be [M, K/group]")
    nbytes = tmac_packed_bytes(desc)
    if nbytes == 0:
        raise TmacError(TMAC_EINVAL, "tmac_packed_bytes")
    blob = np.empty(nbytes, dtype=np.uint8)
    _check(lib.tmac_pack_weights(C.byref(desc), _np_ptr(q), _np_ptr(s16), _np_ptr(z16),
                                 _np_ptr(blob), nbytes), "tmac_pack_weights")
    return blob


def tmac_lut_bytes(N: int, K: int, group: int, lut: int, g: int = 4) -> int:
    return int(lib.tmac_lut_bytes(N, K, g, group, lut))


def tmac_lut_bytes_max(N_max: int, K: int, group: int, lut: int, g: int = 4) -> int:
    return int(lib.tmac_lut_bytes_max(N_max, K, g, group, lut))


def tmac_workspace_bytes(desc: tmac_wdesc, N: int) -> int:
    return int(lib.tmac_workspace_bytes(C.byref(desc), N))


def tmac_workspace_bytes_max(desc: tmac_wdesc, N_max: int) -> int:
    return int(lib.tmac_workspace_bytes_max(C.byref(desc), N_max))


def tmac_fused_workspace_bytes_max(desc: tmac_wdesc, N_max: int, act: int) -> int:
    return int(lib.tmac_fused_workspace_bytes_max(C.byref(desc), N_max, act))


def tmac_blob_check(desc: tmac_wdesc, header: np.ndarray) -> int:
    """Status of the host-side header check (TMAC_OK or TMAC_EINVAL); `header`: at least the first
    256 bytes of a packed blob, as a uint8 numpy array."""
    h = np.ascontiguousarray(header, dtype=np.uint8)
    if h.size < 256:
        raise ValueError("the blob header is 256 bytes")
    return int(lib.tmac_blob_check(C.byref(desc), _np_ptr(h)))


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def tmac_precompute_lut(A, N: int, K: int, group: int, lut: int, lut_buf, act: Optional[int] = None,
                        lda: Optional[int] = None, g: int = 4, stream=None) -> None:
    """A: device tensor (fp16 or int8) [N, K]; lut_buf: device uint8 tensor of tmac_lut_bytes."""
    import torch
    if act is None:
        act = TMAC_ACT_I8 if A.dtype == torch.int8 else TMAC_ACT_F16
    _check_act_dtype(A, act)
    if lda is None:
        lda = A.stride(0) if A.dim() == 2 else K
    _check(lib.tmac_precompute_lut(C.c_void_p(A.data_ptr()), act, N, K, lda, g, group, lut,
                                   C.c_void_p(lut_buf.data_ptr()), lut_buf.numel() * lut_buf.element_size(),
                                   _stream_ptr(stream)), "tmac_precompute_lut")


def tmac_mpgemm(desc: tmac_wdesc, packed, lut_buf, lut: int, N: int, out, out_t: int,
                workspace=None, act_scale=None, weight_scale: float = 1.0, ldo: Optional[int] = None,
                stream=None, tuning: Optional[tmac_tuning] = None) -> None:
    """packed / lut_buf / out / workspace / act_scale: device tensors."""
    if ldo is None:
        ldo = out.stride(0) if out.dim() == 2 else desc.M
    ws_ptr = C.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    as_ptr = C.c_void_p(act_scale.data_ptr()) if act_scale is not None else None
    args = [C.byref(desc), C.c_void_p(packed.data_ptr()), C.c_void_p(lut_buf.data_ptr()), lut, N, as_ptr,
            C.c_float(weight_scale), C.c_void_p(out.data_ptr()), out_t, ldo, ws_ptr, ws_bytes,
            _stream_ptr(stream)]
    if tuning is None:
        _check(lib.tmac_mpgemm(*args), "tmac_mpgemm")
    else:
        _check(lib.tmac_mpgemm_ex(*args, C.byref(tuning)), "tmac_mpgemm_ex")


def tmac_mpgemm_noalloc(desc: tmac_wdesc, packed, lut_buf, lut: int, N: int, out, out_t: int,
                        act_scale=None, weight_scale: float = 1.0, ldo: Optional[int] = None, stream=None) -> None:
    """tmac_mpgemm without a workspace (the library's own fixed array takes the partial sums)."""
    if ldo is None:
        ldo = out.stride(0) if out.dim() == 2 else desc.M
    as_ptr = C.c_void_p(act_scale.data_ptr()) if act_scale is not None else None
    _check(lib.tmac_mpgemm_noalloc(C.byref(desc), C.c_void_p(packed.data_ptr()), C.c_void_p(lut_buf.data_ptr()), lut,
                                   N, as_ptr, C.c_float(weight_scale), C.c_void_p(out.data_ptr()), out_t, ldo,
                                   _stream_ptr(stream)), "tmac_mpgemm_noalloc")


def _check_act_dtype(A, act: int) -> None:
    """The C ABI takes the activation type on trust; a tensor of another element size would be read
    out of range."""
    import torch
    want = torch.int8 if act == TMAC_ACT_I8 else torch.float16
    if A.dtype != want:
        raise ValueError(f"activation type {act} needs a {want} tensor, got {A.dtype}")


def tmac_mpgemv_fused(desc: tmac_wdesc, packed, A, N: int, out, out_t: int, act: Optional[int] = None,
                      lda: Optional[int] = None, act_scale=None, weight_scale: float = 1.0,
                      ldo: Optional[int] = None, stream=None, tuning: Optional[tmac_tuning] = None) -> None:
    """packed / A / out / act_scale: device tensors; A fp16 or int8 [N, K]."""
    import torch
    if act is None:
        act = TMAC_ACT_I8 if A.dtype == torch.int8 else TMAC_ACT_F16
    _check_act_dtype(A, act)
    if lda is None:
        lda = A.stride(0) if A.dim() == 2 else desc.K
    if ldo is None:
        ldo = out.stride(0) if out.dim() == 2 else desc.M
    as_ptr = C.c_void_p(act_scale.data_ptr()) if act_scale is not None else None
    args = [C.byref(desc), C.c_void_p(packed.data_ptr()), C.c_void_p(A.data_ptr()), act, N, lda, as_ptr,
            C.c_float(weight_scale), C.c_void_p(out.data_ptr()), out_t, ldo, _stream_ptr(stream)]
    if tuning is None:
        _check(lib.tmac_mpgemv_fused(*args), "tmac_mpgemv_fused")
    else:
        _check(lib.tmac_mpgemv_fused_ex(*args, C.byref(tuning)), "tmac_mpgemv_fused_ex")


def tmac_mpgemv_fused_multi(items, N: int, out_t: int, act: Optional[int] = None, stream=None,
                            tuning: Optional[tmac_tuning] = None) -> None:
    """items: sequence of (desc, packed, A, out[, act_scale[, weight_scale]]) with device tensors;
    one launch serves them all."""
    import torch
    n = len(items)
    arr = (tmac_gemv_item * max(n, 1))()
    for i, it in enumerate(items):
        desc, packed, A, out = it[:4]
        act_scale = it[4] if len(it) > 4 else None
        wscale = it[5] if len(it) > 5 else 1.0
        a_act = TMAC_ACT_I8 if A.dtype == torch.int8 else TMAC_ACT_F16
        if act is None:
            act = a_act
        _check_act_dtype(A, act)
        arr[i] = tmac_gemv_item(C.pointer(desc), packed.data_ptr(), A.data_ptr(),
                                A.stride(0) if A.dim() == 2 else desc.K,
                                act_scale.data_ptr() if act_scale is not None else None, float(wscale),
                                out.data_ptr(), out.stride(0) if out.dim() == 2 else desc.M)
    _check(lib.tmac_mpgemv_fused_multi(arr, n, TMAC_ACT_F16 if act is None else act, N, out_t, _stream_ptr(stream),
                                       C.byref(tuning) if tuning is not None else None), "tmac_mpgemv_fused_multi")


def tmac_fused_workspace_bytes(desc: tmac_wdesc, N: int, act: int) -> int:
    return int(lib.tmac_fused_workspace_bytes(C.byref(desc), N, act))


def tmac_mpgemm_fused(desc: tmac_wdesc, packed, A, N: int, out, out_t: int, workspace, act: Optional[int] = None,
                      lda: Optional[int] = None, act_scale=None, weight_scale: float = 1.0,
                      ldo: Optional[int] = None, stream=None) -> None:
    """packed / A / out / act_scale / workspace: device tensors; A fp16 or int8 [N, K]."""
    import torch
    if act is None:
        act = TMAC_ACT_I8 if A.dtype == torch.int8 else TMAC_ACT_F16
    _check_act_dtype(A, act)
    if lda is None:
        lda = A.stride(0) if A.dim() == 2 else desc.K
    if ldo is None:
        ldo = out.stride(0) if out.dim() == 2 else desc.M
    as_ptr = C.c_void_p(act_scale.data_ptr()) if act_scale is not None else None
    _check(lib.tmac_mpgemm_fused(C.byref(desc), C.c_void_p(packed.data_ptr()), C.c_void_p(A.data_ptr()), act, N, lda,
                                 as_ptr, C.c_float(weight_scale), C.c_void_p(out.data_ptr()), out_t, ldo,
                                 C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                 _stream_ptr(stream)), "tmac_mpgemm_fused")


# ---------------------------------------------------------------------------------------
# Convenience holder for device-resident state (allocation only; no arithmetic)
# ---------------------------------------------------------------------------------------
@dataclass
class DeviceWeights:
    desc: tmac_wdesc
    packed: "object"   # torch uint8 tensor on the device
    nbytes: int


def upload_weights(desc: tmac_wdesc, q, scales=None, zeros=None, device="cuda") -> DeviceWeights:
    import torch
    blob = tmac_pack_weights(desc, q, scales, zeros)
    t = torch.from_numpy(blob).to(device)
    return DeviceWeights(desc, t, blob.size)
