"""ctypes binding of libtmac_bench.so: measurement helpers (plain streaming read, LDS lookup-rate
probe, empty kernel).  Not part of the mpGEMM library or its ABI; used by bench.py."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
BENCH_LIB_PATH = os.path.join(_PKG_DIR, "libtmac_bench.so")
EXPORTS = ["tmac_bench_stream_read", "tmac_bench_lds_lookup_probe", "tmac_bench_empty_kernel",
           "tmac_bench_valu_rate_probe"]


def _load() -> C.CDLL:
    if not os.path.exists(BENCH_LIB_PATH):
        raise ImportError(f"{BENCH_LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    import torch  # noqa: F401  (one HIP runtime per process: torch's)
    lib = C.CDLL(BENCH_LIB_PATH)
    P, I32, SZ = C.c_void_p, C.c_int32, C.c_size_t
    lib.tmac_bench_stream_read.restype, lib.tmac_bench_stream_read.argtypes = C.c_int, [P, SZ, P, I32, I32, P]
    lib.tmac_bench_lds_lookup_probe.restype, lib.tmac_bench_lds_lookup_probe.argtypes = C.c_int, [I32, I32, P, P]
    lib.tmac_bench_empty_kernel.restype, lib.tmac_bench_empty_kernel.argtypes = C.c_int, [P]
    lib.tmac_bench_valu_rate_probe.restype = C.c_int
    lib.tmac_bench_valu_rate_probe.argtypes = [I32, I32, I32, P, P]
    return lib


lib = _load()


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(code: int, where: str) -> None:
    if code != 0:
        raise RuntimeError(f"{where}: status {code}")


def stream_read(src, sink, per_thread: int = 4, nontemporal: bool = False, nbytes: Optional[int] = None,
                stream=None) -> None:
    """Plain streaming read of a device tensor."""
    n = src.numel() * src.element_size() if nbytes is None else nbytes
    _check(lib.tmac_bench_stream_read(C.c_void_p(src.data_ptr()), n, C.c_void_p(sink.data_ptr()), per_thread,
                                      1 if nontemporal else 0, _stream_ptr(stream)), "tmac_bench_stream_read")


def lds_lookup_probe(workgroups: int, rounds: int, sink, stream=None) -> None:
    """workgroups x 256 lanes x rounds x 16 LDS reads of 16 bytes."""
    _check(lib.tmac_bench_lds_lookup_probe(workgroups, rounds, C.c_void_p(sink.data_ptr()), _stream_ptr(stream)),
           "tmac_bench_lds_lookup_probe")


def empty_kernel(stream=None) -> None:
    _check(lib.tmac_bench_empty_kernel(_stream_ptr(stream)), "tmac_bench_empty_kernel")


def valu_rate_probe(kind: int, workgroups: int, iters: int, sink, stream=None) -> None:
    """kind 0 v_and_b32, 1 v_perm_b32, 2 v_dot2c_f32_f16 (iters x 64 instructions per lane), 3 the lookup
    sequence of one index dword (iters x 8 x 17 instructions per lane)."""
    _check(lib.tmac_bench_valu_rate_probe(kind, workgroups, iters, C.c_void_p(sink.data_ptr()), _stream_ptr(stream)),
           "tmac_bench_valu_rate_probe")
