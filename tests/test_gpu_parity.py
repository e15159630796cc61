"""Parity of the HIP path (called through the C ABI) against the CPU oracle, element by
element on the same seeded inputs.

Bars: integer path bit-exact; fp16-table path within 2e-3 relative Frobenius error of the
fp64 product (the rounding of table entries to fp16 alone costs a few 1e-4)."""
import numpy as np
import pytest

import tmac_workloads as wl
from oracle import tmac_oracle as orc

pytestmark = pytest.mark.gpu

FP_TOL = 2e-3


@pytest.fixture(scope="module")
def T():
    import paper_2407_00088_amd as T
    return T


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available()
    return torch


def run_fp(T, torch, p, out_t=None, tuning=None):
    from paper_2407_00088_amd.runner import from_problem
    lin = from_problem(p)
    A = torch.from_numpy(p.act).cuda()
    out = lin.forward(A, out_t=T.TMAC_OUT_F32 if out_t is None else out_t, tuning=tuning)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def oracle_fp(p):
    return orc.mpgemm_definition(p.act, p.q, p.scales, p.zeros, p.group, p.weight_scale, p.zero_point)


def check_fp(T, torch, p, tuning=None, tol=FP_TOL):
    got = run_fp(T, torch, p, tuning=tuning)
    ref = oracle_fp(p)
    assert got.shape == ref.shape and got.dtype == np.float32
    assert np.all(np.isfinite(got))
    err = orc.rel_frobenius(got, ref)
    print(f"{p.name}: rel_frobenius={err:.3e}", flush=True)
    assert err <= tol, (p.name, err)
    return err


def run_int(T, torch, p, out_t, tuning=None):
    from paper_2407_00088_amd.runner import from_problem
    lin = from_problem(p)
    A = torch.from_numpy(p.act_q).cuda()
    s_a = torch.from_numpy(p.act_scale).cuda()
    out = lin.forward(A, out_t=out_t, act_scale=s_a, tuning=tuning)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check_int(T, torch, p, tuning=None):
    ref_i = orc.ternary_int_matmul(p.act_q, p.q, int(p.zero_point))
    got_i = run_int(T, torch, p, T.TMAC_OUT_I32, tuning)
    assert got_i.dtype == np.int32
    assert np.array_equal(got_i.astype(np.int64), ref_i), p.name
    ref_f = orc.int_path_output_f32(ref_i, p.act_scale, p.weight_scale)
    got_f = run_int(T, torch, p, T.TMAC_OUT_F32, tuning)
    assert np.array_equal(got_f.view(np.uint32), ref_f.view(np.uint32)), p.name


# ------------------------------------------------------------- small cases ----

def test_config1_tiny(T, torch):
    err = check_fp(T, torch, wl.config1())
    assert err < 1e-3


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
@pytest.mark.parametrize("group", [32, 64, 128, 384, 0])
def test_small_ragged_all_bits_all_groupings(T, torch, bits, group):
    """Several 16-row tiles with a ragged last tile, three 128-chunks; every supported
    grouping (sub-chunk, chunk, multi-chunk, per row == K, per tensor)."""
    M, K = 100, 384
    if group == 0:
        rng = np.random.default_rng(7 + bits)
        p = wl.Problem("small_pt", 0, 1, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                       weight_scale=0.037, zero_point=1.25, act=wl.gaussian_act(rng, 1, K))
    else:
        p = wl.make_grouped(0, 10 * bits + group % 7, 1, M, K, bits, group, name=f"small_w{bits}_g{group}")
    check_fp(T, torch, p)


@pytest.mark.parametrize("K", [4, 64, 192, 8640 // 5])
def test_ragged_k_padding(T, torch, K):
    """K not a multiple of the 128-wide chunk: padded tables are all-zero."""
    p = wl.make_grouped(0, 50 + K % 13, 2, 40, K, 4, K, name=f"ragk_{K}")
    check_fp(T, torch, p)
    if K % 64 == 0:
        check_fp(T, torch, wl.make_grouped(0, 51, 1, 40, K, 2, 32, name=f"ragk32_{K}"))


@pytest.mark.parametrize("ks", [2, 4, 8])
@pytest.mark.parametrize("nt", [1, 4])
def test_launch_shapes_agree(T, torch, ks, nt):
    from paper_2407_00088_amd.binding import tmac_tuning
    p = wl.make_grouped(0, 60, 6, 200, 1280, 4, 128, name=f"tune_ks{ks}_nt{nt}")
    tun = tmac_tuning(ks, nt)
    check_fp(T, torch, p, tuning=tun)


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 9])
def test_small_batches(T, torch, N):
    p = wl.make_grouped(0, 70 + N, N, 64, 512, 3, 128, name=f"batch_{N}")
    check_fp(T, torch, p)


def test_single_row_and_single_tile(T, torch):
    check_fp(T, torch, wl.make_grouped(0, 80, 1, 1, 128, 4, 128, name="m1"))
    check_fp(T, torch, wl.make_grouped(0, 81, 1, 16, 4096, 2, 128, name="one_tile_longk"))


def test_fp16_output_is_rounded_fp32(T, torch):
    p = wl.make_grouped(0, 82, 2, 48, 256, 4, 128, name="f16out")
    f32 = run_fp(T, torch, p)
    f16 = run_fp(T, torch, p, out_t=T.TMAC_OUT_F16)
    assert f16.dtype == np.float16
    assert np.array_equal(f16, f32.astype(np.float16))


def test_results_are_reproducible(T, torch):
    p = wl.make_grouped(0, 83, 1, 512, 4096, 4, 128, name="repro")
    a = run_fp(T, torch, p)
    for _ in range(3):
        assert np.array_equal(run_fp(T, torch, p).view(np.uint32), a.view(np.uint32))


def test_closed_forms_on_device(T, torch):
    """All-zero codes: R = -sum_G s z S; zero point at mid level and 1-bit: flipping all bits negates R."""
    rng = np.random.default_rng(84)
    M, K, G, b = 32, 256, 128, 4
    s = wl.group_scales(rng, M, K // G)
    z = wl.group_zeros(rng, M, K // G, b)
    a = wl.gaussian_act(rng, 1, K)
    p = wl.Problem("zeros", 0, 1, M, K, b, G, np.zeros((M, K), np.uint8), s, z, act=a)
    S = a.astype(np.float64).reshape(1, K // G, G).sum(-1)
    expect = -np.einsum("ng,mg->nm", S, s.astype(np.float64) * z.astype(np.float64))
    # the look-up term and the bias term cancel to first order here, which amplifies the fp16
    # rounding of the table entries: a few 1e-4 is expected
    assert orc.rel_frobenius(run_fp(T, torch, p), expect) < 1e-3
    q = wl.uniform_codes(rng, M, K, 1)
    half = np.full((M, K // G), 0.5, np.float16)
    p1 = wl.Problem("sign", 0, 1, M, K, 1, G, q, s, half, act=a)
    p2 = wl.Problem("sign_flipped", 0, 1, M, K, 1, G, 1 - q, s, half, act=a)
    assert np.array_equal(run_fp(T, torch, p1), -run_fp(T, torch, p2))


# ------------------------------------------------------------ integer path ----

@pytest.mark.parametrize("M,K,N", [(48, 256, 1), (100, 192, 3), (16, 8640, 1), (130, 3200, 5)])
def test_ternary_int_path_bit_exact_small(T, torch, M, K, N):
    check_int(T, torch, wl.make_ternary(0, M + K + N, N, M, K))


def test_int_path_extreme_values(T, torch):
    """Largest table entries (+-508) and code 3 (= +2): still exact."""
    M, K = 32, 512
    q = np.full((M, K), 3, np.uint8)
    q[::2] = 0
    a_q = np.full((2, K), 127, np.int8)
    a_q[1] = -127
    p = wl.Problem("extreme", 0, 2, M, K, 2, 0, q, None, None, weight_scale=0.5, zero_point=1.0,
                   act_q=a_q, act_scale=np.array([0.25, 2.0], np.float32))
    check_int(T, torch, p)


@pytest.mark.parametrize("ks", [2, 8])
def test_int_path_launch_shapes(T, torch, ks):
    from paper_2407_00088_amd.binding import tmac_tuning
    check_int(T, torch, wl.make_ternary(0, 90 + ks, 2, 144, 1664), tuning=tmac_tuning(ks, 1))


def test_int_tables_with_group_scales(T, torch):
    """int8 activations against group-quantised 4-bit weights (W4A8): exact int32 group sums,
    fp32 scale application; compared with the fp64 product of the de-quantised operands."""
    rng = np.random.default_rng(95)
    N, M, K, G, b = 2, 64, 512, 128, 4
    a_q, s_a = wl.absmax_int8(wl.gaussian_act(rng, N, K))
    q = wl.uniform_codes(rng, M, K, b)
    s, z = wl.group_scales(rng, M, K // G), wl.group_zeros(rng, M, K // G, b)
    p = wl.Problem("w4a8", 0, N, M, K, b, G, q, s, z, act_q=a_q, act_scale=s_a)
    got = run_int(T, torch, p, T.TMAC_OUT_F32)
    ref = orc.mpgemm_definition(a_q.astype(np.float64) * s_a[:, None].astype(np.float64), q, s, z, G)
    assert orc.rel_frobenius(got, ref) < 1e-5


# ------------------------------------------- full-size configurations ----

@pytest.mark.parametrize("i", [0, 1, 2])
def test_config2_llama7b_w4(T, torch, i):
    err = check_fp(T, torch, wl.config2(i))
    assert err < 1e-3


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_config3_bit_sweep(T, torch, bits):
    check_fp(T, torch, wl.config3(bits))


@pytest.mark.parametrize("i", [0, 1, 2])
def test_config4_bitnet_ternary(T, torch, i):
    check_int(T, torch, wl.config4(i))


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("i", [0, 1, 2])
def test_config5_llama13b_prefill(T, torch, i, bits):
    check_fp(T, torch, wl.config5(i, bits))


# ------------------------------------------------ both lookup kernels ----

@pytest.mark.parametrize("kernel", [1, 2])
@pytest.mark.parametrize("bits,group,K", [(4, 128, 1408), (2, 256, 1024), (3, 0, 640), (1, 896, 896)])
def test_both_kernels_fp(T, torch, kernel, bits, group, K):
    """kernel 1 = K-sliced with split-K reduction, kernel 2 = full-K decode kernel
    (K = 1408 gives 11 chunks: a ragged last batch for the 8 waves)."""
    from paper_2407_00088_amd.binding import tmac_tuning
    M, N = 72, 2
    if group == 0:
        rng = np.random.default_rng(300 + bits)
        p = wl.Problem("both_pt", 0, N, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                       weight_scale=0.05, zero_point=2.0, act=wl.gaussian_act(rng, N, K))
    else:
        p = wl.make_grouped(0, 310 + bits, N, M, K, bits, group, name=f"both_k{kernel}_w{bits}")
    check_fp(T, torch, p, tuning=tmac_tuning(0, 0, kernel))


@pytest.mark.parametrize("kernel", [1, 2])
def test_both_kernels_int(T, torch, kernel):
    from paper_2407_00088_amd.binding import tmac_tuning
    check_int(T, torch, wl.make_ternary(0, 320 + kernel, 3, 200, 2240), tuning=tmac_tuning(0, 0, kernel))


def test_full_k_kernel_rejects_what_it_cannot_do(T, torch):
    from paper_2407_00088_amd.binding import tmac_tuning
    p = wl.make_grouped(0, 330, 1, 32, 256, 2, 32, name="g32_fullk")
    with pytest.raises(T.TmacError) as ei:
        run_fp(T, torch, p, tuning=tmac_tuning(0, 0, 2))
    assert ei.value.status == T.TMAC_EUNSUPPORTED
