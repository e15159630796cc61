"""Device-resident state for one weight matrix: buffers and call order only (no arithmetic)."""
from __future__ import annotations

from typing import Optional

import numpy as np

from . import binding as B

DECODE_MAX_N = 8  # up to this many activation rows the register-table layout is the default


def default_layout(max_N: int) -> int:
    return B.TMAC_LAYOUT_R8U16 if max_N <= DECODE_MAX_N else B.TMAC_LAYOUT_R64K32


class LinearLUT:
    """Holds the packed weights of one [M, K] matrix on the device together with the LUT,
    workspace and output buffers for up to ``max_N`` activation rows, and issues
    tmac_precompute_lut + tmac_mpgemm on the current torch stream."""

    def __init__(self, M: int, K: int, bits: int, group: int, q: np.ndarray,
                 scales: Optional[np.ndarray] = None, zeros: Optional[np.ndarray] = None,
                 zero_point: float = 0.0, weight_scale: float = 1.0, int_path: bool = False,
                 max_N: int = 1, device: str = "cuda", packed_host: Optional[np.ndarray] = None,
                 layout: Optional[int] = None, lut_t: Optional[int] = None, g: int = 4):
        import torch
        self.torch = torch
        self.device = device
        # LUT group sizes other than 4 exist in the batched layout only
        self.layout = (default_layout(max_N) if g == 4 else B.TMAC_LAYOUT_R64K32) if layout is None else layout
        self.g = g
        self.desc = B.wdesc(M, K, bits, group, zero_point, g=g, layout=self.layout)
        self.M, self.K, self.bits, self.group = M, K, bits, group
        self.weight_scale = float(weight_scale)
        self.lut_t = (B.TMAC_LUT_I16 if int_path else B.TMAC_LUT_F16) if lut_t is None else lut_t
        self.max_N = max_N
        blob = packed_host if packed_host is not None else B.tmac_pack_weights(self.desc, q, scales, zeros)
        self.packed_bytes = int(blob.size)
        self.packed = torch.from_numpy(blob).to(device)
        # the regions of the LUT buffer, the split of a call and with it the workspace depend on N:
        # both are sized for every N up to max_N
        lut_bytes = B.tmac_lut_bytes_max(max_N, K, group, self.lut_t, g=g)
        self.lut = torch.empty(max(lut_bytes, 256), dtype=torch.uint8, device=device)
        ws = B.tmac_workspace_bytes_max(self.desc, max_N)
        # (left with a non-zero pattern on purpose: the library must not rely on its contents)
        self.workspace = torch.full((max(ws, 256),), 0xA5, dtype=torch.uint8, device=device)

    def precompute(self, A, N: Optional[int] = None, stream=None):
        N = A.shape[0] if N is None else N
        B.tmac_precompute_lut(A, N, self.K, self.group, self.lut_t, self.lut, g=self.g, stream=stream)

    def mpgemm(self, N: int, out, out_t: int = B.TMAC_OUT_F32, act_scale=None, stream=None, tuning=None,
               packed=None):
        B.tmac_mpgemm(self.desc, self.packed if packed is None else packed, self.lut, self.lut_t, N, out,
                      out_t, workspace=self.workspace, act_scale=act_scale, weight_scale=self.weight_scale,
                      stream=stream, tuning=tuning)

    def mpgemv_fused(self, A, N: int, out, out_t: int = B.TMAC_OUT_F32, act_scale=None, stream=None, packed=None,
                     tuning=None, act=None):
        """One launch: tables built inside the lookup kernel (layout 2 only); act = B.TMAC_ACT_F16_TQ
        quantises them to int8 there."""
        B.tmac_mpgemv_fused(self.desc, self.packed if packed is None else packed, A, N, out, out_t, act=act,
                            act_scale=act_scale, weight_scale=self.weight_scale, stream=stream, tuning=tuning)

    def mpgemm_fused(self, A, N: int, out, out_t: int = B.TMAC_OUT_F32, act_scale=None, stream=None, packed=None):
        """One call for either layout (tmac_mpgemm_fused); its workspace is allocated on first use."""
        act = B.TMAC_ACT_I8 if A.dtype == self.torch.int8 else B.TMAC_ACT_F16
        need = B.tmac_fused_workspace_bytes_max(self.desc, self.max_N, act)
        if need == 0:
            raise B.TmacError(B.TMAC_EUNSUPPORTED, "tmac_fused_workspace_bytes_max")
        if getattr(self, "fused_ws", None) is None or self.fused_ws.numel() < need:
            self.fused_ws = self.torch.full((max(need, 256),), 0xA5, dtype=self.torch.uint8, device=self.device)
        B.tmac_mpgemm_fused(self.desc, self.packed if packed is None else packed, A, N, out, out_t, self.fused_ws,
                            act_scale=act_scale, weight_scale=self.weight_scale, stream=stream)

    def forward_one_call(self, A, out_t: int = B.TMAC_OUT_F32, act_scale=None):
        torch = self.torch
        N = A.shape[0]
        assert N <= self.max_N
        dt = {B.TMAC_OUT_F32: torch.float32, B.TMAC_OUT_F16: torch.float16, B.TMAC_OUT_I32: torch.int32}[out_t]
        out = torch.empty((N, self.M), dtype=dt, device=self.device)
        self.mpgemm_fused(A, N, out, out_t, act_scale=act_scale)
        return out

    def forward_fused(self, A, out_t: int = B.TMAC_OUT_F32, act_scale=None, tuning=None, act=None):
        torch = self.torch
        N = A.shape[0]
        dt = {B.TMAC_OUT_F32: torch.float32, B.TMAC_OUT_F16: torch.float16, B.TMAC_OUT_I32: torch.int32}[out_t]
        out = torch.empty((N, self.M), dtype=dt, device=self.device)
        self.mpgemv_fused(A, N, out, out_t, act_scale=act_scale, tuning=tuning, act=act)
        return out

    def forward(self, A, out_t: int = B.TMAC_OUT_F32, act_scale=None, tuning=None):
        torch = self.torch
        N = A.shape[0]
        assert N <= self.max_N
        dt = {B.TMAC_OUT_F32: torch.float32, B.TMAC_OUT_F16: torch.float16, B.TMAC_OUT_I32: torch.int32}[out_t]
        out = torch.empty((N, self.M), dtype=dt, device=self.device)
        self.precompute(A, N)
        self.mpgemm(N, out, out_t, act_scale=act_scale, tuning=tuning)
        return out


def layout_supports_group(layout: int, K: int, group: int) -> bool:
    """Mirror of the library's rule for which group sizes a layout's kernels can apply."""
    if group == 0 or group == K:
        return True
    if layout == B.TMAC_LAYOUT_R8U16:
        return group % 16 == 0
    return group % 32 == 0


def from_problem(p, max_N: Optional[int] = None, device: str = "cuda", layout: Optional[int] = None,
                 lut_t: Optional[int] = None, g: int = 4) -> LinearLUT:
    """Build a LinearLUT from a workload description object with fields M, K, bits, group, q,
    scales, zeros, zero_point, weight_scale and int_path."""
    return LinearLUT(p.M, p.K, p.bits, p.group, p.q, p.scales, p.zeros, zero_point=p.zero_point,
                     weight_scale=p.weight_scale, int_path=p.int_path, max_N=max_N or p.N, device=device,
                     layout=layout, lut_t=lut_t, g=g)
