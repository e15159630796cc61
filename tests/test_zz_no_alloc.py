"""tmac_mpgemm_noalloc (the entry point for callers that cannot allocate: split-K partial sums in
the library's own fixed device array) against tmac_mpgemm with a caller's workspace, through the C
ABI: bit-identical results on two calls in a row, the second with a smaller input, and the exact
integer path; also that the oversize refusal comes before anything touches the GPU."""
import numpy as np
import pytest

import tmac_workloads as wl
from oracle import tmac_oracle as orc

L3 = 3


def _pair(T, torch, p, int_path=False, out_t=None):
    """(tmac_mpgemm result, tmac_mpgemm_noalloc result) for problem p in the batched layout."""
    from paper_2407_00088_amd import binding as B
    from paper_2407_00088_amd.runner import from_problem
    out_t = B.TMAC_OUT_F32 if out_t is None else out_t
    lin = from_problem(p, layout=L3)
    assert B.tmac_workspace_bytes(lin.desc, p.N) > 256, "the case must split K (else no scratch is used)"
    A = torch.from_numpy(p.act_q if int_path else p.act).cuda()
    sc = torch.from_numpy(p.act_scale).cuda() if int_path else None
    dt = torch.int32 if out_t == B.TMAC_OUT_I32 else torch.float32
    lin.precompute(A, p.N)
    ref = torch.full((p.N, p.M), -3, dtype=dt, device="cuda")
    lin.mpgemm(p.N, ref, out_t, act_scale=sc)
    got = torch.full((p.N, p.M), -5, dtype=dt, device="cuda")
    B.tmac_mpgemm_noalloc(lin.desc, lin.packed, lin.lut, lin.lut_t, p.N, got, out_t, act_scale=sc,
                          weight_scale=lin.weight_scale)
    torch.cuda.synchronize()
    return ref.cpu().numpy(), got.cpu().numpy()


@pytest.mark.gpu
def test_noalloc_equals_workspace_call_twice_second_smaller():
    import torch
    import paper_2407_00088_amd as T
    # first call: 16 activation rows, K split into eight-chunk slices; second, smaller: 3 rows, ragged M,
    # longer slices (group 96) -- the array still holds the first call's sums
    big = wl.make_grouped(0, 1201, 16, 1024, 2048, 4, 128, name="noalloc_big")
    small = wl.make_grouped(0, 1202, 3, 200, 1152, 2, 96, name="noalloc_small")
    for p in (big, small, big):
        ref, got = _pair(T, torch, p)
        assert np.array_equal(ref.view(np.uint32), got.view(np.uint32)), p.name
        exact = orc.mpgemm_definition(p.act, p.q, p.scales, p.zeros, p.group, p.weight_scale, p.zero_point)
        assert orc.rel_frobenius(got, exact) <= 2e-3, p.name


@pytest.mark.gpu
def test_noalloc_integer_path_is_exact():
    import torch
    import paper_2407_00088_amd as T
    p = wl.make_ternary(0, 1203, 8, 320, 3200, name="noalloc_int")
    ref, got = _pair(T, torch, p, int_path=True, out_t=T.TMAC_OUT_I32)
    assert np.array_equal(ref, got)
    assert np.array_equal(got.astype(np.int64), orc.ternary_int_matmul(p.act_q, p.q, int(p.zero_point)))


def test_noalloc_refuses_oversize_before_touching_the_gpu():
    """N = 256 on 5120 x 5120 needs 52 MB of partial sums, more than the fixed array: TMAC_ESIZE, decided
    on the host from the sizes alone (the pointers are never used)."""
    import ctypes as C
    from paper_2407_00088_amd import binding as B
    d = B.wdesc(5120, 5120, 4, 128, layout=B.TMAC_LAYOUT_R64K32)
    assert B.tmac_workspace_bytes(d, 256) - 256 > (8 << 20)
    fake = C.c_void_p(4096)
    st = B.lib.tmac_mpgemm_noalloc(C.byref(d), fake, fake, B.TMAC_LUT_F16, 256, None, C.c_float(1.0), fake,
                                   B.TMAC_OUT_F32, 5120, None)
    assert st == B.TMAC_ESIZE
    assert b"TMAC_NOALLOC_MAX_WORKSPACE" in B.lib.tmac_last_error_detail()
    bad = B.wdesc(5120, 5120, 9, 128, layout=B.TMAC_LAYOUT_R64K32)
    assert B.lib.tmac_mpgemm_noalloc(C.byref(bad), fake, fake, B.TMAC_LUT_F16, 1, None, C.c_float(1.0), fake,
                                     B.TMAC_OUT_F32, 5120, None) == B.TMAC_EINVAL
