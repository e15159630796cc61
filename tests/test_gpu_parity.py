"""Parity of the HIP path (called through the C ABI) against the CPU oracle, element by
element on the same seeded inputs.

Bars: integer path bit-exact; fp16-table path within 2e-3 relative Frobenius error of the
fp64 product (the rounding of table entries to fp16 alone costs a few 1e-4).

Every case runs in both packed layouts where both apply: layout 3 feeds the batched lookup kernel
with one lane per weight row ("rows"), layout 2 the register-table decode kernel, called either as
tmac_precompute_lut + tmac_mpgemm ("regs") or as the single fused launch tmac_mpgemv_fused
("fused")."""
import numpy as np
import pytest

import rounding_models as rm
import tmac_workloads as wl
from oracle import tmac_oracle as orc

pytestmark = pytest.mark.gpu

FP_TOL = 2e-3
L2, L3 = 2, 3
LF = 13  # layout 2 through the fused entry point


@pytest.fixture(scope="module")
def T():
    import paper_2407_00088_amd as T
    return T


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available()
    return torch


@pytest.fixture(params=[L2, LF, L3], ids=["regs", "fused", "rows"])
def layout(request):
    return request.param


def make_lin(p, layout):
    from paper_2407_00088_amd.runner import from_problem, layout_supports_group
    if layout == LF:
        if p.K % 16 != 0:
            pytest.skip("the fused entry point needs K % 16 == 0")
        layout = L2
    if not layout_supports_group(layout, p.K, p.group):
        pytest.skip(f"group {p.group} not supported by layout {layout}")
    return from_problem(p, layout=layout)


def run_fp(T, torch, p, out_t=None, tuning=None, layout=L3):
    lin = make_lin(p, layout)
    A = torch.from_numpy(p.act).cuda()
    if layout == LF:
        out = lin.forward_fused(A, out_t=T.TMAC_OUT_F32 if out_t is None else out_t, tuning=tuning)
    else:
        out = lin.forward(A, out_t=T.TMAC_OUT_F32 if out_t is None else out_t, tuning=tuning)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def oracle_fp(p):
    return orc.mpgemm_definition(p.act, p.q, p.scales, p.zeros, p.group, p.weight_scale, p.zero_point)


ELEM_TOL_UNITS = 6.0   # allowed |got - ref| of one output, in units of u * E (see assert_elementwise)


def assert_elementwise(got, ref, p, what=""):
    """Bound on the error of EVERY output, next to the Frobenius bar over all of them.

    The error of an output is a sum of about K b / 4 independent fp16 roundings (u = 2^-11) of table
    entries and chunk sums, each proportional to the activations it covers times the weight range of
    the row: it behaves like a Gaussian of standard deviation c u E with
    E[n,m] = sqrt(sum_k (a[n,k] s[m,k] (2^b - 1))^2), whatever the distribution of the activations
    (outlier channels included: they enter E as they enter the error).  The CPU models of the kernels'
    roundings (tests/rounding_models.py) give c = 0.2-0.5 and a largest |error| of 1.5 u E over
    thousands of outputs at K = 256 ... 13824, 1-4 bit, Gaussian and heavy-tailed activations; 6 u E is
    allowed.  A typical output is 600-800 u E in size, so one that is off by 1 % of its own value
    already misses this bound, which the Frobenius bar alone would not see (one output in 4096 with a
    10 % error moves the norm by 1.5e-3)."""
    u = 2.0 ** -11
    a2 = np.asarray(p.act, dtype=np.float64) ** 2
    if p.group == 0:
        s_full = np.full((p.M, p.K), float(p.weight_scale))
    else:
        s_full = np.repeat(np.asarray(p.scales, dtype=np.float64), p.group, axis=1)
    E = np.sqrt(a2 @ ((s_full * (2 ** p.bits - 1)) ** 2).T)
    ratio = np.abs(np.asarray(got, dtype=np.float64) - ref) / np.maximum(u * E, 1e-300)
    worst = float(ratio.max())
    assert worst <= ELEM_TOL_UNITS, (p.name, what, worst, np.unravel_index(ratio.argmax(), ratio.shape))
    return worst


def check_fp(T, torch, p, tuning=None, tol=FP_TOL, layout=L3):
    got = run_fp(T, torch, p, tuning=tuning, layout=layout)
    ref = oracle_fp(p)
    assert got.shape == ref.shape and got.dtype == np.float32
    assert np.all(np.isfinite(got))
    err = orc.rel_frobenius(got, ref)
    worst = assert_elementwise(got, ref, p, f"layout{layout}")
    print(f"{p.name} layout{layout}: rel_frobenius={err:.3e} worst element {worst:.2f} u E "
          f"(bound {ELEM_TOL_UNITS})", flush=True)
    assert err <= tol, (p.name, layout, err)
    return err


def run_int(T, torch, p, out_t, tuning=None, layout=L3):
    lin = make_lin(p, layout)
    A = torch.from_numpy(p.act_q).cuda()
    s_a = torch.from_numpy(p.act_scale).cuda()
    if layout == LF:
        out = lin.forward_fused(A, out_t=out_t, act_scale=s_a, tuning=tuning)
    else:
        out = lin.forward(A, out_t=out_t, act_scale=s_a, tuning=tuning)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check_int(T, torch, p, tuning=None, layout=L3):
    ref_i = orc.ternary_int_matmul(p.act_q, p.q, int(p.zero_point))
    got_i = run_int(T, torch, p, T.TMAC_OUT_I32, tuning, layout)
    assert got_i.dtype == np.int32
    assert np.array_equal(got_i.astype(np.int64), ref_i), (p.name, layout)
    ref_f = orc.int_path_output_f32(ref_i, p.act_scale, p.weight_scale)
    got_f = run_int(T, torch, p, T.TMAC_OUT_F32, tuning, layout)
    assert np.array_equal(got_f.view(np.uint32), ref_f.view(np.uint32)), (p.name, layout)


# ------------------------------------------------------------- small cases ----

def test_config1_tiny(T, torch, layout):
    err = check_fp(T, torch, wl.config1(), layout=layout)
    assert err < 1e-3


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
@pytest.mark.parametrize("group", [16, 32, 48, 64, 128, 192, 384, 0])
def test_small_ragged_all_bits_all_groupings(T, torch, bits, group, layout):
    """Several row tiles with a ragged last tile, three 128-chunks; every supported grouping
    (sub-chunk, chunk, multi-chunk, per row == K, per tensor)."""
    M, K = 100, 384
    if group == 0:
        rng = np.random.default_rng(7 + bits)
        p = wl.Problem("small_pt", 0, 1, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                       weight_scale=0.037, zero_point=1.25, act=wl.gaussian_act(rng, 1, K))
    else:
        p = wl.make_grouped(0, 10 * bits + group % 7, 1, M, K, bits, group, name=f"small_w{bits}_g{group}")
    check_fp(T, torch, p, layout=layout)


@pytest.mark.parametrize("K", [4, 24, 64, 192, 8640 // 5])
def test_ragged_k_padding(T, torch, K, layout):
    """K not a multiple of the 128-wide chunk (nor of the 16-wide unit): padded tables are all-zero."""
    p = wl.make_grouped(0, 50 + K % 13, 2, 40, K, 4, K, name=f"ragk_{K}")
    check_fp(T, torch, p, layout=layout)
    if K % 64 == 0:
        check_fp(T, torch, wl.make_grouped(0, 51, 1, 40, K, 2, 32, name=f"ragk32_{K}"), layout=layout)


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 9])
def test_small_batches(T, torch, N, layout):
    p = wl.make_grouped(0, 70 + N, N, 64, 512, 3, 128, name=f"batch_{N}")
    check_fp(T, torch, p, layout=layout)


def test_single_row_and_single_tile(T, torch, layout):
    check_fp(T, torch, wl.make_grouped(0, 80, 1, 1, 128, 4, 128, name="m1"), layout=layout)
    check_fp(T, torch, wl.make_grouped(0, 81, 1, 16, 4096, 2, 128, name="one_tile_longk"), layout=layout)


def test_long_k_multi_pass(T, torch):
    """K beyond 16 waves x 64 units x 16: the register-table kernel walks several blocks per wave;
    the batched kernel walks 24 LDS slices (or K slices over workgroups)."""
    p = wl.make_grouped(0, 85, 1, 24, 20480, 4, 128, name="k20480")
    check_fp(T, torch, p, layout=L2)
    check_fp(T, torch, wl.make_grouped(0, 86, 2, 24, 24576, 2, 0 + 256, name="k24576"), layout=L2)
    check_fp(T, torch, wl.make_grouped(0, 86, 1, 24, 24576, 2, 256, name="k24576_rows"), layout=L3)


def test_fp16_output_is_rounded_fp32(T, torch, layout):
    p = wl.make_grouped(0, 82, 2, 48, 256, 4, 128, name="f16out")
    f32 = run_fp(T, torch, p, layout=layout)
    f16 = run_fp(T, torch, p, out_t=T.TMAC_OUT_F16, layout=layout)
    assert f16.dtype == np.float16
    assert np.array_equal(f16, f32.astype(np.float16))


def test_results_are_reproducible(T, torch, layout):
    p = wl.make_grouped(0, 83, 1, 512, 4096, 4, 128, name="repro")
    a = run_fp(T, torch, p, layout=layout)
    for _ in range(3):
        assert np.array_equal(run_fp(T, torch, p, layout=layout).view(np.uint32), a.view(np.uint32))


def test_closed_forms_on_device(T, torch, layout):
    """All-zero codes: R = -sum_G s z S; zero point at mid level and 1-bit: flipping all bits negates R."""
    rng = np.random.default_rng(84)
    M, K, G, b = 32, 256, 128, 4
    s = wl.group_scales(rng, M, K // G)
    z = wl.group_zeros(rng, M, K // G, b)
    a = wl.gaussian_act(rng, 1, K)
    p = wl.Problem("zeros", 0, 1, M, K, b, G, np.zeros((M, K), np.uint8), s, z, act=a)
    S = a.astype(np.float64).reshape(1, K // G, G).sum(-1)
    expect = -np.einsum("ng,mg->nm", S, s.astype(np.float64) * z.astype(np.float64))
    # the look-up term and the bias term cancel to first order here, and every plane looks up the
    # same entry, so the fp16 roundings (table entries; chunk sums in the batched kernel) add up
    # coherently over the planes: up to 1.2e-3 instead of the usual few 1e-4, still inside the bar
    assert orc.rel_frobenius(run_fp(T, torch, p, layout=layout), expect) < FP_TOL
    q = wl.uniform_codes(rng, M, K, 1)
    half = np.full((M, K // G), 0.5, np.float16)
    p1 = wl.Problem("sign", 0, 1, M, K, 1, G, q, s, half, act=a)
    p2 = wl.Problem("sign_flipped", 0, 1, M, K, 1, G, 1 - q, s, half, act=a)
    assert np.array_equal(run_fp(T, torch, p1, layout=layout), -run_fp(T, torch, p2, layout=layout))


def test_small_magnitude_activations(T, torch, layout):
    """Activations of magnitude 1e-2: table entries stay normal fp16 numbers; the error bar holds."""
    p = wl.make_grouped(0, 87, 1, 64, 1024, 4, 128, name="small_act")
    p.act = (p.act.astype(np.float32) * np.float32(1e-2)).astype(np.float16)
    check_fp(T, torch, p, layout=layout)


@pytest.mark.parametrize("N", [1, 16])
def test_heavy_tailed_activations(T, torch, layout, N):
    """Outlier channels (0.2 % of the activations 300 times the rest, magnitudes up to about 1000): the
    fp16 tables and chunk sums stay finite and the error stays where it is on Gaussian data."""
    if N > 8 and layout != L3:
        pytest.skip("the register-table kernel serves at most 8 rows here")
    p = wl.make_grouped(0, 88 + N, N, 96, 4096, 4, 128, name="heavy_tail")
    rng = np.random.default_rng(88)
    boost = np.where(rng.random(p.act.shape) < 0.002, 300.0, 1.0)
    p.act = (p.act.astype(np.float64) * boost).astype(np.float16)
    assert np.abs(p.act.astype(np.float64)).max() > 100
    err = check_fp(T, torch, p, layout=layout)
    assert err <= 8e-4


# ------------------------------------------------------------ integer path ----

@pytest.mark.parametrize("M,K,N", [(48, 256, 1), (100, 192, 3), (16, 8640, 1), (130, 3200, 5)])
def test_ternary_int_path_bit_exact_small(T, torch, M, K, N, layout):
    check_int(T, torch, wl.make_ternary(0, M + K + N, N, M, K), layout=layout)


def test_int_path_extreme_values(T, torch, layout):
    """Largest table entries (+-508) and code 3 (= +2): still exact."""
    M, K = 32, 512
    q = np.full((M, K), 3, np.uint8)
    q[::2] = 0
    a_q = np.full((2, K), 127, np.int8)
    a_q[1] = -127
    p = wl.Problem("extreme", 0, 2, M, K, 2, 0, q, None, None, weight_scale=0.5, zero_point=1.0,
                   act_q=a_q, act_scale=np.array([0.25, 2.0], np.float32))
    check_int(T, torch, p, layout=layout)


def test_int_path_extreme_values_four_bit_long_k(T, torch):
    """4-bit codes against +-127 activations over K = 16384: the register-table kernel carries
    integer sums in fp32 inside a wave (below 2^24) and in int32 across waves."""
    M, K = 16, 16384
    rng = np.random.default_rng(88)
    q = rng.integers(0, 16, size=(M, K), dtype=np.uint8)
    q[0] = 15
    q[1] = 0
    a_q = np.full((1, K), 127, np.int8)
    p = wl.Problem("extreme4", 0, 1, M, K, 4, 0, q, None, None, weight_scale=1.0, zero_point=0.0,
                   act_q=a_q, act_scale=np.array([1.0], np.float32))
    ref = orc.ternary_int_matmul(a_q, q, 0)
    for layout in (L3, L2):
        got = run_int(T, torch, p, T.TMAC_OUT_I32, layout=layout)
        assert np.array_equal(got.astype(np.int64), ref), layout


def test_int_tables_with_group_scales(T, torch, layout):
    """int8 activations against group-quantised 4-bit weights (W4A8): exact integer group sums,
    fp32 scale application; compared with the fp64 product of the de-quantised operands."""
    rng = np.random.default_rng(95)
    N, M, K, G, b = 2, 64, 512, 128, 4
    a_q, s_a = wl.absmax_int8(wl.gaussian_act(rng, N, K))
    q = wl.uniform_codes(rng, M, K, b)
    s, z = wl.group_scales(rng, M, K // G), wl.group_zeros(rng, M, K // G, b)
    p = wl.Problem("w4a8", 0, N, M, K, b, G, q, s, z, act_q=a_q, act_scale=s_a)
    got = run_int(T, torch, p, T.TMAC_OUT_F32, layout=layout)
    ref = orc.mpgemm_definition(a_q.astype(np.float64) * s_a[:, None].astype(np.float64), q, s, z, G)
    assert orc.rel_frobenius(got, ref) < 1e-5


# ------------------------------------------- full-size configurations ----

@pytest.mark.parametrize("i", [0, 1, 2])
def test_config2_llama7b_w4(T, torch, i, layout):
    err = check_fp(T, torch, wl.config2(i), layout=layout)
    assert err < 1e-3


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_config3_bit_sweep(T, torch, bits, layout):
    check_fp(T, torch, wl.config3(bits), layout=layout)


@pytest.mark.parametrize("i", [0, 1, 2])
def test_config4_bitnet_ternary(T, torch, i, layout):
    check_int(T, torch, wl.config4(i), layout=layout)


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("i", [0, 1, 2])
def test_config5_llama13b_prefill(T, torch, i, bits):
    check_fp(T, torch, wl.config5(i, bits), layout=L3)


# ------------------------------------- register-table kernel launch shapes ----

@pytest.mark.parametrize("fused", [False, True], ids=["regs", "fused"])
@pytest.mark.parametrize("rows", [8, 16])
@pytest.mark.parametrize("bits,group,M,K", [(4, 128, 200, 1408), (2, 64, 72, 1024), (3, 0, 41, 640),
                                            (1, 1040, 24, 1040), (4, 128, 8, 17408)])
def test_register_kernel_rows_per_group(T, torch, rows, bits, group, M, K, fused):
    """8 or 16 weight rows per workgroup (an odd number of 8-row tiles leaves the second tile of
    the last workgroup empty); K = 17408 walks two blocks of units per wave."""
    from paper_2407_00088_amd.binding import tmac_tuning

    def run(p, tun):
        return run_fp(T, torch, p, tuning=tun, layout=LF if fused else L2)

    N = 2
    if group == 0:
        rng = np.random.default_rng(400 + bits)
        p = wl.Problem("rpg_pt", 0, N, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                       weight_scale=0.05, zero_point=2.0, act=wl.gaussian_act(rng, N, K))
    else:
        p = wl.make_grouped(0, 410 + bits, N, M, K, bits, group, name=f"rpg{rows}_w{bits}")
    got = run(p, tmac_tuning(rows))
    err = orc.rel_frobenius(got, oracle_fp(p))
    assert err <= FP_TOL, err
    # both launch shapes add the same terms in the same order
    other = run(p, tmac_tuning(24 - rows))
    assert np.array_equal(got.view(np.uint32), other.view(np.uint32))


@pytest.mark.parametrize("fused", [False, True], ids=["regs", "fused"])
@pytest.mark.parametrize("rows", [8, 16])
def test_register_kernel_rows_per_group_int(T, torch, rows, fused):
    from paper_2407_00088_amd.binding import tmac_tuning
    check_int(T, torch, wl.make_ternary(0, 420 + rows, 3, 200, 2240), tuning=tmac_tuning(rows),
              layout=LF if fused else L2)


# ----------------------------------------------------------- fused entry point ----

@pytest.mark.parametrize("bits,group,M,K,N", [(4, 128, 200, 1408, 2), (2, 64, 72, 1024, 1), (3, 256, 41, 768, 3),
                                              (1, 16, 24, 1040, 1), (4, 128, 64, 11008, 1)])
def test_fused_equals_two_call_path_bitwise(T, torch, bits, group, M, K, N):
    """With group scales the fused kernel builds the same table entries and chunk sums as the
    precompute kernel and adds in the same order: results are identical bit for bit."""
    p = wl.make_grouped(0, 500 + bits, N, M, K, bits, group, name=f"fused_w{bits}_g{group}")
    two = run_fp(T, torch, p, layout=L2)
    one = run_fp(T, torch, p, layout=LF)
    assert orc.rel_frobenius(one, oracle_fp(p)) <= FP_TOL
    assert np.array_equal(one.view(np.uint32), two.view(np.uint32))


def test_fused_rejects_what_it_cannot_do(T, torch):
    from paper_2407_00088_amd import binding as B
    p = wl.make_grouped(0, 510, 1, 16, 136, 2, 8)
    A = torch.from_numpy(p.act).cuda()
    out = torch.empty((1, 16), dtype=torch.float32, device="cuda")
    for layout, K in ((L3, 128), (L2, 136)):
        q = p.q[:, :K]
        d = B.wdesc(16, K, 2, 0, 1.0, layout=layout)
        packed = torch.from_numpy(B.tmac_pack_weights(d, q)).cuda()
        with pytest.raises(T.TmacError) as e:
            B.tmac_mpgemv_fused(d, packed, A, 1, out, B.TMAC_OUT_F32, lda=K)
        assert e.value.status in (B.TMAC_EUNSUPPORTED, B.TMAC_EINVAL)


# ------------------------------------------- several matrices in one launch ----

def _multi_vs_single(T, torch, problems, N, out_t, tuning=None, int_path=False):
    """Runs tmac_mpgemv_fused_multi over `problems` and tmac_mpgemv_fused on each; returns both lists."""
    from paper_2407_00088_amd import binding as B
    from paper_2407_00088_amd.runner import from_problem
    dt = {B.TMAC_OUT_F32: torch.float32, B.TMAC_OUT_F16: torch.float16, B.TMAC_OUT_I32: torch.int32}[out_t]
    lins = [from_problem(p, layout=L2) for p in problems]
    As = [torch.from_numpy(p.act_q if int_path else p.act).cuda() for p in problems]
    scs = [torch.from_numpy(p.act_scale).cuda() if int_path else None for p in problems]
    single = []
    for lin, A, sc in zip(lins, As, scs):
        o = torch.full((N, lin.M), -7, dtype=dt, device="cuda")
        lin.mpgemv_fused(A, N, o, out_t, act_scale=sc)
        single.append(o)
    multi = [torch.full((N, lin.M), -9, dtype=dt, device="cuda") for lin in lins]
    items = [(lin.desc, lin.packed, A, o, sc, lin.weight_scale) for lin, A, o, sc in zip(lins, As, multi, scs)]
    B.tmac_mpgemv_fused_multi(items, N, out_t, tuning=tuning)
    torch.cuda.synchronize()
    return [o.cpu().numpy() for o in multi], [o.cpu().numpy() for o in single]


def test_multi_launch_config2_equals_three_separate_calls_bitwise(T, torch):
    """The three Llama-2-7B shapes of config 2 (K = 4096, 4096, 11008: four and eleven waves per group
    of row tiles) in ONE launch: every output equals the single fused call's bit for bit, and meets
    the bar against the oracle."""
    ps = [wl.config2(i) for i in range(3)]
    multi, single = _multi_vs_single(T, torch, ps, 1, T.TMAC_OUT_F32)
    for p, m, s1 in zip(ps, multi, single):
        assert np.array_equal(m.view(np.uint32), s1.view(np.uint32)), p.name
        ref = oracle_fp(p)
        assert orc.rel_frobenius(m, ref) <= FP_TOL
        assert_elementwise(m, ref, p, "multi")


@pytest.mark.parametrize("bits,group,N,rows", [(4, 128, 1, 0), (2, 128, 3, 8), (3, 64, 1, 16), (1, 0, 2, 0), (4, -1, 1, 16),
                                               (2, 256, 2, 0)])
def test_multi_launch_mixed_shapes_equal_separate_calls_bitwise(T, torch, bits, group, N, rows):
    """Matrices of unlike shape in one launch: K from one block (128) to seventeen blocks (more than the
    sixteen waves of a workgroup: two passes), ragged M (a last row tile of one row), a matrix smaller
    than one workgroup; every grouping mode, both rows-per-group settings, N > 1; up to the maximum of
    eight matrices.  Bit-identical to the single calls."""
    from paper_2407_00088_amd import binding as B
    kmin = 2 * group if group > 0 else 128   # (K == group would be one scale per row: another grouping mode)
    shapes = [(200, 4096), (8, kmin), (41, 1536 if group == 256 else 1408), (64, 11008),
              (1, max(256, kmin)), (130, 17408), (24, 5120), (77, 1024)]
    ps = []
    for i, (M, K) in enumerate(shapes):
        if group == 0:
            rng = np.random.default_rng(700 + i + bits)
            ps.append(wl.Problem(f"multi_pt{i}", 0, N, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                                 weight_scale=0.02 + 0.01 * i, zero_point=0.5 * i, act=wl.gaussian_act(rng, N, K)))
        else:
            ps.append(wl.make_grouped(0, 700 + i + bits, N, M, K, bits, K if group < 0 else group, name=f"multi{i}"))
    tuning = B.tmac_tuning(rows) if rows else None
    for count in (8, 3, 1):
        multi, single = _multi_vs_single(T, torch, ps[:count], N, T.TMAC_OUT_F32, tuning=tuning)
        for p, m, s1 in zip(ps, multi, single):
            assert np.array_equal(m.view(np.uint32), s1.view(np.uint32)), (p.name, count)
            assert orc.rel_frobenius(m, oracle_fp(p)) <= FP_TOL, (p.name, count)


def test_multi_launch_int_path_is_exact(T, torch):
    """The three BitNet-shaped ternary matrices of config 4 in one launch: int32 results equal the
    integer oracle, fp32 results its two-rounding output, bit for bit."""
    ps = [wl.config4(i) for i in range(3)]
    multi_i, _ = _multi_vs_single(T, torch, ps, 1, T.TMAC_OUT_I32, int_path=True)
    multi_f, single_f = _multi_vs_single(T, torch, ps, 1, T.TMAC_OUT_F32, int_path=True)
    for p, mi, mf, sf in zip(ps, multi_i, multi_f, single_f):
        ref_i = orc.ternary_int_matmul(p.act_q, p.q, int(p.zero_point))
        assert np.array_equal(mi.astype(np.int64), ref_i), p.name
        ref_f = orc.int_path_output_f32(ref_i, p.act_scale, p.weight_scale)
        assert np.array_equal(mf.view(np.uint32), ref_f.view(np.uint32)), p.name
        assert np.array_equal(mf.view(np.uint32), sf.view(np.uint32)), p.name


def test_multi_launch_in_graph_replay(T, torch):
    """Captured in a HIP graph and replayed with eager work in between: every replay equals the eager
    result (no state is kept between launches)."""
    from paper_2407_00088_amd import binding as B
    from paper_2407_00088_amd.runner import from_problem
    ps = [wl.make_grouped(0, 760 + i, 1, M, K, 4, 128, name=f"multig{i}") for i, (M, K) in
          enumerate([(300, 4096), (96, 11008), (520, 2048)])]
    lins = [from_problem(p, layout=L2) for p in ps]
    As = [torch.from_numpy(p.act).cuda() for p in ps]
    outs = [torch.zeros((1, p.M), dtype=torch.float32, device="cuda") for p in ps]
    items = [(lin.desc, lin.packed, A, o) for lin, A, o in zip(lins, As, outs)]
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        B.tmac_mpgemv_fused_multi(items, 1, B.TMAC_OUT_F32)
    stream.synchronize()
    eager = [o.clone() for o in outs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        B.tmac_mpgemv_fused_multi(items, 1, B.TMAC_OUT_F32)
    for rep in range(3):
        for o in outs:
            o.fill_(float(rep))          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, e, p in zip(outs, eager, ps):
            assert torch.equal(o, e), (rep, p.name)
    for e, p in zip(eager, ps):
        assert orc.rel_frobenius(e.cpu().numpy(), oracle_fp(p)) <= FP_TOL


# ------------------------------------------------- int8 table quantisation ----

# Same int8 tables on both sides (then the results agree to 1e-7: fp32 against fp64 sums) except for
# entries whose exact quotient 127 T / amax lies within an fp32 ulp of a half-integer, which the
# kernel's fp32 product rounds either way: about one entry in 50 000.  One such entry moves the
# result of the small test shape (K = 1152) by up to 1.9e-4; the bar leaves room for two of them and
# stays an order of magnitude below the loss of the quantisation itself.
TQ_VS_ORACLE_TQ = 5e-4
TQ_VS_EXACT = 1.2e-2     # Section 3.3 is lossy: a few 1e-3 on Gaussian data


def run_tq(T, torch, p, fused=False):
    """Table quantisation with a LUT buffer (tmac_precompute_lut + tmac_mpgemm, TMAC_LUT_I8Q) or inside
    the fused call (TMAC_ACT_F16_TQ)."""
    from paper_2407_00088_amd.runner import from_problem
    if fused:
        lin = from_problem(p, layout=L2)
        out = lin.forward_fused(torch.from_numpy(p.act).cuda(), act=T.TMAC_ACT_F16_TQ)
    else:
        lin = from_problem(p, layout=L2, lut_t=T.TMAC_LUT_I8Q)
        out = lin.forward(torch.from_numpy(p.act).cuda())
    torch.cuda.synchronize()
    return out.cpu().numpy()


TQ_ROUTES = pytest.mark.parametrize("fused", [False, True], ids=["lut", "in_kernel"])


def oracle_tq(p):
    return orc.lut_mpgemm_tq(p.act, p.q, p.bits, p.scales, p.zeros, p.group, p.weight_scale, p.zero_point)


@TQ_ROUTES
@pytest.mark.parametrize("bits", [1, 2, 3, 4])
@pytest.mark.parametrize("group", [16, 64, 128, 384, 0, -1])
def test_table_quantisation_small(T, torch, bits, group, fused):
    """int8 tables with one scale per 16 activations: against the oracle's quantised route
    (tight) and against the exact product (the method's own loss); ragged M, two chunks blocks."""
    M, K, N = 75, 1152, 2
    if group == 0:
        rng = np.random.default_rng(600 + bits)
        p = wl.Problem("tq_pt", 0, N, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                       weight_scale=0.05, zero_point=1.0, act=wl.gaussian_act(rng, N, K))
    else:
        p = wl.make_grouped(0, 610 + bits, N, M, K, bits, K if group < 0 else group, name=f"tq_w{bits}_g{group}")
    got = run_tq(T, torch, p, fused)
    e_tq = orc.rel_frobenius(got, oracle_tq(p))
    e_ex = orc.rel_frobenius(got, oracle_fp(p))
    print(f"{p.name}: vs quantised oracle {e_tq:.2e}, vs exact {e_ex:.2e}", flush=True)
    assert e_tq <= TQ_VS_ORACLE_TQ, e_tq
    assert e_ex <= TQ_VS_EXACT, e_ex


@pytest.mark.parametrize("K", [16, 24, 200, 1000])
def test_table_quantisation_ragged_k(T, torch, K):
    p = wl.make_grouped(0, 620, 1, 40, K, 4, K, name=f"tq_ragk_{K}")   # one group per row
    got = run_tq(T, torch, p)
    assert orc.rel_frobenius(got, oracle_tq(p)) <= TQ_VS_ORACLE_TQ


@pytest.mark.parametrize("K", [16, 48, 208, 1008, 2064])
def test_table_quantisation_in_kernel_ragged_k(T, torch, K):
    """K a multiple of 16 but not of 128 (the last chunk is partly padding), one and three blocks."""
    p = wl.make_grouped(0, 621, 2, 40, K, 4, K, name=f"tq_ragk_{K}")   # one group per row
    got = run_tq(T, torch, p, fused=True)
    assert orc.rel_frobenius(got, oracle_tq(p)) <= TQ_VS_ORACLE_TQ


def test_table_quantisation_in_kernel_has_no_row_limit(T, torch):
    """The LUT buffer of the quantised tables exists for at most 64 activation rows; the fused call
    builds them per launch and takes any N."""
    p = wl.make_grouped(0, 622, 70, 24, 512, 2, 128)
    got = run_tq(T, torch, p, fused=True)
    assert orc.rel_frobenius(got, oracle_tq(p)) <= TQ_VS_ORACLE_TQ
    assert orc.rel_frobenius(got, oracle_fp(p)) <= TQ_VS_EXACT


@TQ_ROUTES
@pytest.mark.parametrize("i", [0, 1, 2])
def test_table_quantisation_config2(T, torch, i, fused):
    p = wl.config2(i)
    got = run_tq(T, torch, p, fused)
    e_tq = orc.rel_frobenius(got, oracle_tq(p))
    e_ex = orc.rel_frobenius(got, oracle_fp(p))
    print(f"{p.name}: vs quantised oracle {e_tq:.2e}, vs exact {e_ex:.2e} (NMSE {e_ex ** 2:.2e})", flush=True)
    assert e_tq <= TQ_VS_ORACLE_TQ and e_ex <= TQ_VS_EXACT


def test_table_quantisation_zero_and_tiny_activations(T, torch):
    p = wl.make_grouped(0, 630, 2, 24, 256, 2, 32)
    p.act[0, :] = 0
    p.act[1, 16:48] = 0
    p.act[1, 64:] = (p.act[1, 64:].astype(np.float32) * 1e-3).astype(np.float16)
    for fused in (False, True):
        got = run_tq(T, torch, p, fused)
        assert np.all(got[0] == 0)
        assert orc.rel_frobenius(got, oracle_tq(p)) <= 5e-4


@pytest.mark.parametrize("bits,group,M,K,N", [(4, 128, 200, 1408, 2), (2, 64, 72, 1024, 1), (3, 0, 41, 640, 3),
                                              (1, -1, 130, 2064, 1)])
def test_table_quantisation_in_kernel_rows_per_group(T, torch, bits, group, M, K, N):
    """One and two row tiles per group of waves share or do not share a lane's int8 tables: the same
    tables, the same sums, the same result bit for bit (ragged M: a last tile of one row tile)."""
    from paper_2407_00088_amd import binding as B
    from paper_2407_00088_amd.runner import from_problem
    if group == 0:
        rng = np.random.default_rng(650 + bits)
        p = wl.Problem("tq_rows_pt", 0, N, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                       weight_scale=0.05, zero_point=1.0, act=wl.gaussian_act(rng, N, K))
    else:
        p = wl.make_grouped(0, 650 + bits, N, M, K, bits, K if group < 0 else group, name="tq_rows")
    lin = from_problem(p, layout=L2)
    A = torch.from_numpy(p.act).cuda()
    o8 = lin.forward_fused(A, act=B.TMAC_ACT_F16_TQ, tuning=B.tmac_tuning(8)).cpu().numpy()
    o16 = lin.forward_fused(A, act=B.TMAC_ACT_F16_TQ, tuning=B.tmac_tuning(16)).cpu().numpy()
    assert np.array_equal(o8.view(np.uint32), o16.view(np.uint32))
    assert orc.rel_frobenius(o16, oracle_tq(p)) <= TQ_VS_ORACLE_TQ


def test_table_quantisation_multi_launch(T, torch):
    """The three config-2 shapes in one launch with tables quantised in the kernel: each output equals
    the single fused call's bit for bit and meets the bars of the quantised route."""
    from paper_2407_00088_amd import binding as B
    from paper_2407_00088_amd.runner import from_problem
    ps = [wl.config2(i) for i in range(3)]
    lins = [from_problem(p, layout=L2) for p in ps]
    As = [torch.from_numpy(p.act).cuda() for p in ps]
    single = [lin.forward_fused(A, act=B.TMAC_ACT_F16_TQ) for lin, A in zip(lins, As)]
    multi = [torch.full((1, lin.M), -9, dtype=torch.float32, device="cuda") for lin in lins]
    B.tmac_mpgemv_fused_multi([(lin.desc, lin.packed, A, o) for lin, A, o in zip(lins, As, multi)], 1, B.TMAC_OUT_F32,
                              act=B.TMAC_ACT_F16_TQ)
    torch.cuda.synchronize()
    for p, m, s1 in zip(ps, multi, single):
        m, s1 = m.cpu().numpy(), s1.cpu().numpy()
        assert np.array_equal(m.view(np.uint32), s1.view(np.uint32)), p.name
        assert orc.rel_frobenius(m, oracle_tq(p)) <= TQ_VS_ORACLE_TQ
        assert orc.rel_frobenius(m, oracle_fp(p)) <= TQ_VS_EXACT


def test_table_quantisation_rejects_what_it_cannot_do(T, torch):
    from paper_2407_00088_amd import binding as B
    from paper_2407_00088_amd.runner import from_problem
    p = wl.make_grouped(0, 640, 1, 16, 128, 2, 128)
    with pytest.raises(T.TmacError) as e:
        from_problem(p, layout=L3, lut_t=B.TMAC_LUT_I8Q).forward(torch.from_numpy(p.act).cuda())
    assert e.value.status == B.TMAC_EUNSUPPORTED
    t = wl.make_ternary(0, 641, 1, 16, 128)
    lut = torch.empty(B.tmac_lut_bytes(1, 128, 0, B.TMAC_LUT_I8Q), dtype=torch.uint8, device="cuda")
    with pytest.raises(T.TmacError) as e:
        B.tmac_precompute_lut(torch.from_numpy(t.act_q).cuda(), 1, 128, 0, B.TMAC_LUT_I8Q, lut)
    assert e.value.status == B.TMAC_EINVAL
    # in the kernel: layout 2 only, one row tile per group of waves only, fp16 activations only
    A = torch.from_numpy(p.act).cuda()
    out = torch.empty((1, 16), dtype=torch.float32, device="cuda")
    lin3 = from_problem(p, layout=L3)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(T.TmacError) as e:
        B.tmac_mpgemm_fused(lin3.desc, lin3.packed, A, 1, out, B.TMAC_OUT_F32, ws, act=B.TMAC_ACT_F16_TQ)
    assert e.value.status == B.TMAC_EUNSUPPORTED
    lin2 = from_problem(p, layout=L2)
    with pytest.raises(ValueError):
        lin2.mpgemv_fused(torch.from_numpy(t.act_q).cuda(), 1, out, act=B.TMAC_ACT_F16_TQ)
    # through the one-call entry point on layout 2 it is the fused call
    B.tmac_mpgemm_fused(lin2.desc, lin2.packed, A, 1, out, B.TMAC_OUT_F32, ws, act=B.TMAC_ACT_F16_TQ)
    torch.cuda.synchronize()
    assert orc.rel_frobenius(out.cpu().numpy(), oracle_tq(p)) <= TQ_VS_ORACLE_TQ


# ----------------------------------------------------- launch configuration of bench.py ----

@pytest.mark.parametrize("i", [0, 2])
def test_fused_call_in_graph_replay_over_a_weight_ring(T, torch, i):
    """The benchmark replays a HIP graph of fused calls that walk a ring of packed-weight copies;
    every replay must give the eager result (and the oracle's) for every copy."""
    from paper_2407_00088_amd.runner import from_problem
    p = wl.config2(i)
    lin = from_problem(p, layout=L2)
    A = torch.from_numpy(p.act).cuda()
    ring = [lin.packed, lin.packed.clone(), lin.packed.clone()]
    outs = [torch.zeros((1, p.M), dtype=torch.float32, device="cuda") for _ in ring]
    eager = lin.forward_fused(A)
    torch.cuda.synchronize()
    assert orc.rel_frobenius(eager.cpu().numpy(), oracle_fp(p)) <= FP_TOL
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        lin.mpgemv_fused(A, 1, outs[0], packed=ring[0])
    stream.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        for pk, o in zip(ring, outs):
            lin.mpgemv_fused(A, 1, o, packed=pk)
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o in outs:
            assert torch.equal(o, eager), rep


# --------------------------------------------- batched lookup kernel (layout 3) ----

@pytest.mark.parametrize("N", [1, 3, 4, 5, 17, 64])
@pytest.mark.parametrize("bits,group,M,K", [(4, 128, 200, 1408), (2, 32, 72, 1024), (3, 96, 41, 2304), (1, 0, 300, 1040),
                                            (4, -1, 64, 3200)])
def test_batched_kernel_shapes(T, torch, N, bits, group, M, K):
    """Ragged M (tiles of 64), N not a multiple of the four rows a workgroup serves, K that spans
    several LDS slices and ends inside one, group sizes from one chunk up, per-row and per-tensor."""
    if group == 0:
        rng = np.random.default_rng(700 + bits + N)
        p = wl.Problem("rows_pt", 0, N, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                       weight_scale=0.05, zero_point=0.5, act=wl.gaussian_act(rng, N, K))
    else:
        p = wl.make_grouped(0, 710 + bits + N, N, M, K, bits, K if group < 0 else group, name=f"rows_w{bits}_n{N}")
    check_fp(T, torch, p, layout=L3)


@pytest.mark.parametrize("N", [1, 6, 33])
def test_batched_kernel_int_path(T, torch, N):
    check_int(T, torch, wl.make_ternary(0, 720 + N, N, 200, 2240), layout=L3)


def test_batched_kernel_rejects_what_it_cannot_do(T, torch):
    from paper_2407_00088_amd import binding as B
    from paper_2407_00088_amd.runner import from_problem
    p = wl.make_grouped(0, 730, 4, 16, 128, 2, 16)
    with pytest.raises(T.TmacError) as e:
        from_problem(p, layout=L3).forward(torch.from_numpy(p.act).cuda())
    assert e.value.status == B.TMAC_EUNSUPPORTED
    p = wl.make_grouped(0, 731, 4, 16, 128, 2, 128)
    with pytest.raises(T.TmacError) as e:
        from_problem(p, layout=L3, lut_t=B.TMAC_LUT_I8Q).forward(torch.from_numpy(p.act).cuda())
    assert e.value.status == B.TMAC_EUNSUPPORTED


# ------------------------------------------- LUT group sizes 2 and 8 (layout 3) ----

def run_g(T, torch, p, g, int_out=None):
    from paper_2407_00088_amd.runner import from_problem
    lin = from_problem(p, layout=L3, g=g)
    if p.int_path:
        out = lin.forward(torch.from_numpy(p.act_q).cuda(), out_t=int_out, act_scale=torch.from_numpy(p.act_scale).cuda())
    else:
        out = lin.forward(torch.from_numpy(p.act).cuda())
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("g", [2, 8])
@pytest.mark.parametrize("N", [1, 5, 13, 72])
@pytest.mark.parametrize("bits,group,M,K", [(4, 128, 200, 1408), (2, 32, 72, 1024), (3, 96, 41, 2304), (1, -1, 130, 3208)])
def test_other_lut_group_sizes_fp(T, torch, g, N, bits, group, M, K):
    """g = 2 (4-entry tables, sixteen look-ups per chunk and plane) and g = 8 (256-entry tables,
    four look-ups): ragged M and N, K that ends inside a chunk (g = 8: K % 8 == 0) and spans several
    LDS slices and K slices, group sizes from one chunk up and one group per row."""
    p = wl.make_grouped(0, 800 + 10 * g + bits + N, N, M, K, bits, K if group < 0 else group, name=f"g{g}_w{bits}_n{N}")
    got = run_g(T, torch, p, g)
    err = orc.rel_frobenius(got, oracle_fp(p))
    print(f"{p.name}: rel_frobenius={err:.3e}", flush=True)
    assert err <= FP_TOL


@pytest.mark.parametrize("g", [2, 8])
@pytest.mark.parametrize("N,M,K", [(1, 3200, 3200), (9, 100, 8640), (40, 257, 1032)])
def test_other_lut_group_sizes_int_exact(T, torch, g, N, M, K):
    """Ternary weights, int8 activations: bit-exact int32 and fp32 outputs at g = 2 and g = 8."""
    p = wl.make_ternary(0, 820 + g + N, N, M, K, name=f"g{g}_ternary_n{N}")
    ref_i = orc.ternary_int_matmul(p.act_q, p.q, 1)
    assert np.array_equal(run_g(T, torch, p, g, T.TMAC_OUT_I32).astype(np.int64), ref_i)
    ref_f = orc.int_path_output_f32(ref_i, p.act_scale, p.weight_scale)
    assert np.array_equal(run_g(T, torch, p, g, T.TMAC_OUT_F32).view(np.uint32), ref_f.view(np.uint32))


@pytest.mark.parametrize("g", [2, 8])
def test_other_lut_group_sizes_full_shape(T, torch, g):
    """Config-2 shape 4096 x 4096, 16 activation rows."""
    p = wl.make_grouped(2, 830 + g, 16, 4096, 4096, 4, 128, name=f"g{g}_4096x4096_n16")
    err = orc.rel_frobenius(run_g(T, torch, p, g), oracle_fp(p))
    print(f"{p.name}: rel_frobenius={err:.3e}", flush=True)
    assert err <= 1e-3


def test_other_lut_group_sizes_are_layout3_only(T, torch):
    from paper_2407_00088_amd.runner import from_problem
    p = wl.make_grouped(0, 840, 1, 64, 256, 2, 64, name="g8_l2")
    with pytest.raises(Exception):
        from_problem(p, layout=L2, g=8)


@pytest.mark.parametrize("N,M,K,group", [(16, 1024, 2048, 128), (16, 1024, 2304, 96), (256, 512, 1024, 128)])
def test_batched_calls_in_graph_replay(T, torch, N, M, K, group):
    """precompute + lookup of the batched layout captured in a HIP graph and replayed, as bench.py
    times them: K slices of eight chunks summed by the second kernel (group 128), longer slices of
    the general kernel summed by the same second kernel (group 96), and no split at all.  The
    workspace starts with arbitrary contents.  Every replay must give the eager result bit for bit."""
    from paper_2407_00088_amd.runner import from_problem
    p = wl.make_grouped(0, 860 + N + group, N, M, K, 4, group, name="graph_rows")
    lin = from_problem(p, layout=L3)
    A = torch.from_numpy(p.act).cuda()
    eager = lin.forward(A)
    torch.cuda.synchronize()
    assert orc.rel_frobenius(eager.cpu().numpy(), oracle_fp(p)) <= FP_TOL
    out = torch.zeros((N, M), dtype=torch.float32, device="cuda")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        lin.precompute(A)
        lin.mpgemm(N, out)
    stream.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        for _ in range(2):
            lin.precompute(A)
            lin.mpgemm(N, out)
    for rep in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
        assert torch.equal(lin.forward(A), eager)   # eager calls between replays share the workspace


# ----------------------------------------------------- seeded random shapes ----

@pytest.mark.parametrize("seed", range(80))
def test_random_shapes_all_paths(T, torch, seed):
    """Seeded random problems (ragged M, K a multiple of 32 up to 6 k, 1-4 bits, N up to 80, group
    sizes 32..K, per-row and per-tensor scales) through whichever of the paths accepts them:
    register-table kernel from the LUT buffer and fused, batched kernels at g = 4, 2 and 8."""
    from paper_2407_00088_amd.runner import from_problem, layout_supports_group
    rng = np.random.default_rng(9000 + seed)
    bits = int(rng.integers(1, 5))
    K = 32 * int(rng.integers(1, 190))
    M = int(rng.integers(1, 400))
    N = int(rng.choice([1, 1, 2, 3, 5, 8, 9, 16, 23, 40, 80]))
    divisors = [d for d in (32, 64, 96, 128, 256, 512) if K % d == 0]
    mode = rng.choice(["group", "row", "tensor"])
    if mode == "group":
        p = wl.make_grouped(0, 9000 + seed, N, M, K, bits, int(rng.choice(divisors)), name=f"rand{seed}")
    elif mode == "row":
        p = wl.make_grouped(0, 9000 + seed, N, M, K, bits, K, name=f"rand{seed}")
    else:
        p = wl.Problem(f"rand{seed}", 0, N, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                       weight_scale=0.03, zero_point=float(rng.integers(0, 1 << bits)), act=wl.gaussian_act(rng, N, K))
    ref = oracle_fp(p)
    A = torch.from_numpy(p.act).cuda()
    ran = []
    for layout, g, fused in ((L2, 4, False), (L2, 4, True), (L3, 4, False), (L3, 2, False), (L3, 8, False)):
        if layout == L2 and N > 8:
            continue
        if not layout_supports_group(layout, K, p.group) or K % g:
            continue
        lin = from_problem(p, layout=layout, g=g)
        out = lin.forward_fused(A) if fused else lin.forward(A)
        torch.cuda.synchronize()
        err = orc.rel_frobenius(out.cpu().numpy(), ref)
        assert err <= FP_TOL, (seed, layout, g, fused, M, K, N, bits, p.group, err)
        ran.append(err)
        if not fused:   # the one-call entry point on the same matrix
            err1 = orc.rel_frobenius(lin.forward_one_call(A).cpu().numpy(), ref)
            assert err1 <= FP_TOL, (seed, layout, g, "one call", M, K, N, bits, p.group, err1)
    assert ran
    print(f"rand{seed}: M={M} K={K} N={N} b={bits} G={p.group} paths={len(ran)} max_err={max(ran):.2e}", flush=True)


@pytest.mark.parametrize("seed", range(40))
def test_random_shapes_int_path_exact(T, torch, seed):
    """Seeded random ternary problems with int8 activations: every path must give the oracle's int32
    result and its two-rounding fp32 output bit for bit."""
    from paper_2407_00088_amd.runner import from_problem
    rng = np.random.default_rng(9500 + seed)
    K = 32 * int(rng.integers(1, 280))
    M = int(rng.integers(1, 500))
    N = int(rng.choice([1, 1, 2, 4, 7, 8, 12, 33, 70]))
    p = wl.make_ternary(0, 9500 + seed, N, M, K, weight_scale=float(rng.uniform(0.005, 0.05)), name=f"randint{seed}")
    ref_i = orc.ternary_int_matmul(p.act_q, p.q, 1)
    ref_f = orc.int_path_output_f32(ref_i, p.act_scale, p.weight_scale)
    A = torch.from_numpy(p.act_q).cuda()
    s_a = torch.from_numpy(p.act_scale).cuda()
    for layout, g, fused in ((L2, 4, False), (L2, 4, True), (L3, 4, False), (L3, 2, False), (L3, 8, False)):
        if layout == L2 and N > 8:
            continue
        if K % g:
            continue
        lin = from_problem(p, layout=layout, g=g)
        run = lin.forward_fused if fused else lin.forward
        got_i = run(A, out_t=T.TMAC_OUT_I32, act_scale=s_a).cpu().numpy()
        got_f = run(A, out_t=T.TMAC_OUT_F32, act_scale=s_a).cpu().numpy()
        assert np.array_equal(got_i.astype(np.int64), ref_i), (seed, layout, g, fused, M, K, N)
        assert np.array_equal(got_f.view(np.uint32), ref_f.view(np.uint32)), (seed, layout, g, fused, M, K, N)
        if not fused:   # the one-call entry point on the same matrix
            one_i = lin.forward_one_call(A, out_t=T.TMAC_OUT_I32, act_scale=s_a).cpu().numpy()
            assert np.array_equal(one_i.astype(np.int64), ref_i), (seed, layout, g, "one call", M, K, N)


@pytest.mark.parametrize("N,bits", [(16, 4), (48, 2), (3, 3)])
def test_batched_kernel_matches_the_narrow_sum_route(T, torch, N, bits):
    """The batched kernel adds the eight entries of a 32-k chunk and plane pairwise in fp16 before
    widening: against the CPU model that takes exactly these roundings (tests/rounding_models.py) (fp64 elsewhere) only the
    fp32 accumulation is left, orders of magnitude below the distance to the exact product."""
    p = wl.make_grouped(0, 880 + N, N, 256, 2048, bits, 128, name=f"narrow_n{N}")
    got = run_fp(T, torch, p, layout=L3)
    model = rm.lut_mpgemm_narrow(p.act, p.q, bits, p.scales, p.zeros, p.group)
    exact = oracle_fp(p)
    e_model, e_exact = orc.rel_frobenius(got, model), orc.rel_frobenius(got, exact)
    print(f"{p.name}: vs narrow-sum route {e_model:.2e}, vs exact {e_exact:.2e}", flush=True)
    assert e_model <= 2e-6 and e_exact <= FP_TOL


@pytest.mark.parametrize("lay", [L2, LF], ids=["regs", "fused"])
@pytest.mark.parametrize("bits,group", [(4, 128), (2, 32), (3, 0), (1, -1)])
def test_decode_kernel_matches_the_fp16_table_route(T, torch, lay, bits, group):
    """The register-table kernel builds its tables with fp16 additions and accumulates in fp32:
    against the CPU model with tables of the same construction (tests/rounding_models.py) (fp64 elsewhere) only the fp32
    accumulation is left."""
    M, K = 200, 4096
    if group == 0:
        rng = np.random.default_rng(890 + bits)
        p = wl.Problem("tabroute", 0, 1, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                       weight_scale=0.04, zero_point=2.0, act=wl.gaussian_act(rng, 1, K))
    else:
        p = wl.make_grouped(0, 890 + bits, 1, M, K, bits, K if group < 0 else group, name="tabroute")
    got = run_fp(T, torch, p, layout=lay)
    model = rm.lut_mpgemm_fp16_tree(p.act, p.q, bits, p.scales, p.zeros, p.group, p.weight_scale, p.zero_point)
    e_model, e_exact = orc.rel_frobenius(got, model), orc.rel_frobenius(got, oracle_fp(p))
    print(f"tabroute b{bits} G{p.group} layout{lay}: vs fp16-table route {e_model:.2e}, vs exact {e_exact:.2e}", flush=True)
    assert e_model <= 2e-6 and e_exact <= FP_TOL


@pytest.mark.parametrize("g", [2, 4, 8])
@pytest.mark.parametrize("K", [8, 16, 24, 40, 136])
def test_tiny_k_all_lut_group_sizes(T, torch, g, K):
    """K shorter than one 32-k chunk or ending inside one (padding chunks and tables are zero), one
    scale per row and per tensor, a single weight row and a handful of activation rows."""
    from paper_2407_00088_amd.runner import from_problem
    for M, N, per_tensor in ((1, 1, False), (5, 3, True), (70, 9, False)):
        rng = np.random.default_rng(950 + K + g + M)
        if per_tensor:
            p = wl.Problem("tinyk", 0, N, M, K, 3, 0, wl.uniform_codes(rng, M, K, 3), None, None,
                           weight_scale=0.07, zero_point=3.0, act=wl.gaussian_act(rng, N, K))
        else:
            p = wl.make_grouped(0, 950 + K + g + M, N, M, K, 3, K, name="tinyk")
        out = from_problem(p, layout=L3, g=g).forward(torch.from_numpy(p.act).cuda())
        torch.cuda.synchronize()
        got, ref = out.cpu().numpy().astype(np.float64), oracle_fp(p)
        if M * N > 1:
            assert orc.rel_frobenius(got, ref) <= FP_TOL, (g, K, M, N)
        # a single output of a few dozen terms can cancel to a fraction of its terms (the 1 x 1 case is
        # held to the Frobenius bar together with its siblings in the next test): each output is also
        # held against the sum of the magnitudes of its terms, which the rounding errors scale with
        assert_elementwise(got, ref, p, f"g{g} K{K} M{M} N{N}")


def test_tiny_k_single_outputs_meet_the_frobenius_bar_together(T, torch):
    """The fifteen 1 x 1 cases of the test above (g = 2, 4, 8 times five short K) as one vector of
    outputs: relative Frobenius error within the 2e-3 bar.  One output alone has no norm to be
    relative to but its own value, which a cancelling sum of a few dozen terms makes arbitrarily
    small; fifteen of them do not all cancel."""
    from paper_2407_00088_amd.runner import from_problem
    got, ref = [], []
    for g in (2, 4, 8):
        for K in (8, 16, 24, 40, 136):
            p = wl.make_grouped(0, 950 + K + g + 1, 1, 1, K, 3, K, name="tinyk")
            out = from_problem(p, layout=L3, g=g).forward(torch.from_numpy(p.act).cuda())
            torch.cuda.synchronize()
            got.append(float(out.cpu().numpy()[0, 0]))
            ref.append(float(oracle_fp(p)[0, 0]))
    err = orc.rel_frobenius(np.array(got), np.array(ref))
    print(f"tiny K, fifteen single outputs: rel_frobenius={err:.3e}", flush=True)
    assert err <= FP_TOL


# ------------------------------------------------- one-call entry point ----

@pytest.mark.parametrize("layout,g,N,M,K,bits,group", [
    (L3, 4, 16, 300, 2048, 4, 128),    # tables built in the eight-chunk kernel
    (L3, 4, 9, 64, 4096, 2, 32),
    (L3, 4, 32, 130, 1280, 3, 256),
    (L3, 4, 40, 130, 1280, 3, 256),    # more than 32 rows: precompute launch inside the call
    (L3, 4, 3, 70, 1024, 1, 64),       # four activation rows per workgroup
    (L3, 4, 16, 200, 2304, 4, 96),     # group size does not divide 256: precompute launch inside the call
    (L3, 4, 16, 200, 2048, 4, -1),     # one scale per row: tables and row sums built in the kernel
    (L3, 4, 5, 70, 3208, 2, -1),       # K ends inside a chunk
    (L3, 4, 5, 70, 3204, 2, -1),       # K % 8 != 0: precompute launch inside the call
    (L3, 4, 256, 512, 1024, 4, 128),   # many rows, no short slices: the same
    (L3, 8, 16, 128, 2048, 4, 128),    # other LUT group size: the same
    (L2, 4, 1, 100, 4096, 4, 128),     # register-table kernel, tables built in the kernel
    (L2, 4, 4, 100, 4072, 2, -1),      # K % 16 != 0: precompute launch inside the call
])
def test_one_call_entry_point_fp(T, torch, layout, g, N, M, K, bits, group):
    """tmac_mpgemm_fused against the oracle and against tmac_precompute_lut + tmac_mpgemm (same table
    entries; only the order of the activation sums may differ)."""
    from paper_2407_00088_amd.runner import from_problem
    p = wl.make_grouped(0, 960 + N + bits, N, M, K, bits, K if group < 0 else group, name="onecall")
    lin = from_problem(p, layout=layout, g=g)
    A = torch.from_numpy(p.act).cuda()
    two = lin.forward(A).cpu().numpy()
    for _ in range(2):   # twice: the workspace is reused
        one = lin.forward_one_call(A).cpu().numpy()
        assert orc.rel_frobenius(one, oracle_fp(p)) <= FP_TOL
        assert orc.rel_frobenius(one, two) <= 2e-6


@pytest.mark.parametrize("layout,N,M,K", [(L3, 12, 257, 3200), (L3, 70, 100, 8640), (L2, 2, 64, 3200)])
def test_one_call_entry_point_int_exact(T, torch, layout, N, M, K):
    from paper_2407_00088_amd.runner import from_problem
    p = wl.make_ternary(0, 970 + N, N, M, K, name="onecall_int")
    lin = from_problem(p, layout=layout)
    A, s_a = torch.from_numpy(p.act_q).cuda(), torch.from_numpy(p.act_scale).cuda()
    ref_i = orc.ternary_int_matmul(p.act_q, p.q, 1)
    got = lin.forward_one_call(A, out_t=T.TMAC_OUT_I32, act_scale=s_a).cpu().numpy()
    assert np.array_equal(got.astype(np.int64), ref_i)
    got_f = lin.forward_one_call(A, out_t=T.TMAC_OUT_F32, act_scale=s_a).cpu().numpy()
    assert np.array_equal(got_f.view(np.uint32), orc.int_path_output_f32(ref_i, p.act_scale, p.weight_scale).view(np.uint32))


def test_one_call_entry_point_int_group_scales_in_kernel(T, torch):
    """int8 activations with group scales, tables and group sums built in the kernel: integer tables
    and sums are exact, so the result must equal the two-call path bit for bit."""
    from paper_2407_00088_amd.runner import from_problem
    rng = np.random.default_rng(975)
    N, M, K, G = 16, 200, 2048, 128
    q = wl.uniform_codes(rng, M, K, 4)
    a_q, s_a = wl.absmax_int8(wl.gaussian_act(rng, N, K))
    p = wl.Problem("onecall_intg", 0, N, M, K, 4, G, q, wl.group_scales(rng, M, K // G), wl.group_zeros(rng, M, K // G, 4),
                   act_q=a_q, act_scale=s_a)
    lin = from_problem(p, layout=L3)
    A, sa = torch.from_numpy(a_q).cuda(), torch.from_numpy(s_a).cuda()
    two = lin.forward(A, act_scale=sa)
    one = lin.forward_one_call(A, act_scale=sa)
    assert torch.equal(one, two)
    ref = orc.mpgemm_definition(a_q.astype(np.float64) * s_a[:, None].astype(np.float64), q, p.scales, p.zeros, G)
    assert orc.rel_frobenius(one.cpu().numpy(), ref) <= 1e-5


def test_one_call_entry_point_rejects(T, torch):
    from paper_2407_00088_amd import binding as B
    from paper_2407_00088_amd.runner import from_problem
    p = wl.make_grouped(0, 980, 16, 64, 1024, 4, 128, name="onecall_bad")
    lin = from_problem(p, layout=L3)
    A = torch.from_numpy(p.act).cuda()
    out = torch.empty((16, 64), dtype=torch.float32, device="cuda")
    need = B.tmac_fused_workspace_bytes(lin.desc, 16, B.TMAC_ACT_F16)
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    B.tmac_mpgemm_fused(lin.desc, lin.packed, A, 16, out, B.TMAC_OUT_F32, ws)
    with pytest.raises(Exception):
        B.tmac_mpgemm_fused(lin.desc, lin.packed, A, 16, out, B.TMAC_OUT_F32, ws[: need - 256])
    with pytest.raises(Exception):
        B.tmac_mpgemm_fused(lin.desc, lin.packed, A, 16, out, B.TMAC_OUT_F32, ws, lda=1028)


# ------------------------------------------------- the precompute step alone ----

@pytest.mark.parametrize("g", [2, 4, 8])
@pytest.mark.parametrize("int_act", [False, True], ids=["f16", "i8"])
def test_precompute_tables_against_the_oracle(T, torch, g, int_act):
    """Step a2 on its own: the tables [n tile][Kp/g][2^g][NT] and the group sums S[N][K/G] that
    tmac_precompute_lut leaves at the start of the LUT buffer, entry by entry against the oracle's
    tables (Algorithm 1 Precompute).  Integer tables are exact; fp16 tables are built with fp16
    additions, pair sums first, and equal the oracle's tables of the same construction bit for bit
    (and the exact sums within the roundings of the partial sums)."""
    from paper_2407_00088_amd import binding as B
    rng = np.random.default_rng(990 + g)
    N, K, G = 5, 1160 if g != 8 else 1168, 0
    lut_t = B.TMAC_LUT_I16 if int_act else B.TMAC_LUT_F16
    if int_act:
        a = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    else:
        a = wl.gaussian_act(rng, N, K)
    buf = torch.zeros(B.tmac_lut_bytes(N, K, G, lut_t, g=g), dtype=torch.uint8, device="cuda")
    B.tmac_precompute_lut(torch.from_numpy(a).cuda(), N, K, G, lut_t, buf, g=g)
    torch.cuda.synchronize()
    raw = buf.cpu().numpy()
    Kp = (K + 127) // 128 * 128
    KG, ENT = Kp // g, 1 << g
    NT = 4 if g == 8 else 8                                          # rows per n tile at N = 5 (tmac.h)
    n_pad = (N + NT - 1) // NT * NT
    ref = orc.precompute_lut(a, g)                                   # [N, K/g, 2^g]
    # the buffer holds [n tile][KG][2^g][NT]: back to [n][KG][2^g]
    dt = np.int16 if int_act else np.float16
    tab = raw[: n_pad * KG * ENT * 2].view(dt).reshape(n_pad // NT, KG, ENT, NT).transpose(0, 3, 1, 2).reshape(n_pad, KG, ENT)
    assert not tab[N:].any()                                          # rows that pad the last n tile
    tab = tab[:N]
    if int_act:
        assert np.array_equal(tab[:, : K // g].astype(np.int64), ref)
    else:
        want = rm.precompute_lut_fp16_tree(a, g)
        got = tab[:, : K // g]
        assert np.array_equal(got.astype(np.float64), want.astype(np.float64))     # (-0 == +0)
        # within the roundings of the exact table's partial sums: g - 1 additions, each off by at most
        # half a spacing of a number no larger than sum |a_j|
        top = np.abs(a.astype(np.float64)).reshape(N, K // g, g).sum(-1).astype(np.float16)
        bound = 0.5 * (g - 1) * np.spacing(top).astype(np.float64)
        assert np.all(np.abs(got.astype(np.float64) - ref) <= bound[..., None])
    assert not tab[:, K // g:].any()                                  # tables of the k padding are zero
    s_off = (n_pad * KG * ENT * 2 + 255) // 256 * 256
    if int_act:
        S = raw[s_off: s_off + N * 4].view(np.int32)
        assert np.array_equal(S.astype(np.int64), a.astype(np.int64).sum(axis=1))
    else:
        S = raw[s_off: s_off + N * 4].view(np.float32)
        assert np.allclose(S, a.astype(np.float64).sum(axis=1), rtol=1e-5, atol=1e-4)


@pytest.mark.parametrize("N", [71, 129, 200])
@pytest.mark.parametrize("bits,group", [(4, 128), (2, 64), (3, -1), (4, 0)])
def test_many_rows_two_n_tiles_per_workgroup(T, torch, N, bits, group):
    """From 64 activation rows on a workgroup of the many-row kernel serves two n tiles of eight rows
    (one address for two LDS reads).  Row counts that are no multiple of 16 leave the last workgroup a
    second n tile that repeats the first or is only partly filled; group scales, one scale per row and
    one per tensor; fp16 and exact integer tables."""
    from paper_2407_00088_amd.runner import from_problem
    M, K = 150, 1536
    if group == 0:
        rng = np.random.default_rng(1400 + N + bits)
        p = wl.Problem("oct", 0, N, M, K, bits, 0, wl.uniform_codes(rng, M, K, bits), None, None,
                       weight_scale=0.05, zero_point=3.0, act=wl.gaussian_act(rng, N, K))
    else:
        p = wl.make_grouped(0, 1400 + N + bits, N, M, K, bits, K if group < 0 else group, name="oct")
    check_fp(T, torch, p, layout=L3)
    pt = wl.make_ternary(0, 1450 + N, N, M, K, name="oct_int")
    check_int(T, torch, pt, layout=L3)


def test_large_call_takes_two_row_tiles_per_workgroup_by_default(T, torch):
    """From about 8000 wavefronts on (here 8192 x 8192: 1024 row tiles x 8 waves) the register-table
    kernel serves 16 rows per workgroup unless told otherwise: the default call, the call with 8 rows
    per workgroup and the fused call agree with the oracle on sampled rows (the oracle takes them one
    at a time at this size) and, the order of additions per row being the same, with each other."""
    from paper_2407_00088_amd.binding import tmac_tuning
    p = wl.make_grouped(0, 1300, 1, 8192, 8192, 4, 128, name="rt_auto")
    lin = make_lin(p, L2)
    A = torch.from_numpy(p.act).cuda()
    auto = lin.forward(A).cpu().numpy()
    rows8 = lin.forward(A, tuning=tmac_tuning(8)).cpu().numpy()
    fused = lin.forward_fused(A).cpu().numpy()
    rows = np.random.default_rng(1300).choice(p.M, size=96, replace=False)
    ref = orc.mpgemm_definition(p.act, p.q[rows], p.scales[rows], p.zeros[rows], p.group)
    for got in (auto, rows8, fused):
        assert orc.rel_frobenius(got[:, rows], ref) <= FP_TOL
    assert np.array_equal(auto.view(np.uint32), rows8.view(np.uint32))
    assert np.array_equal(auto.view(np.uint32), fused.view(np.uint32))


# ------------------------------------------------------ measurement helpers ----

def test_measurement_helpers_run_and_check_their_arguments(T, torch):
    """The plain-read kernel, the LDS probe and the empty kernel (libtmac_bench.so) take no part in the
    path; they must launch, finish, leave the sink alone (their stores practically never happen) and
    refuse bad arguments."""
    from paper_2407_00088_amd import bench_helpers as H
    src = torch.arange(1 << 16, dtype=torch.int32, device="cuda")
    sink = torch.zeros(256, dtype=torch.uint8, device="cuda")
    for per_thread in (1, 4, 8):
        for nt in (False, True):
            H.stream_read(src, sink, per_thread, nt)
    H.lds_lookup_probe(64, 8, sink)
    H.empty_kernel()
    torch.cuda.synchronize()
    assert not sink.cpu().numpy().any()
    with pytest.raises(RuntimeError):
        H.stream_read(src, sink, 3, False)
    with pytest.raises(RuntimeError):
        H.lds_lookup_probe(0, 8, sink)
    with pytest.raises(RuntimeError):
        H.lds_lookup_probe(64, 0, sink)


def test_one_holder_serves_every_row_count_up_to_its_maximum(T, torch):
    """The LUT buffer's regions and the split of a call depend on N (64 rows need a larger LUT buffer
    than 65): a holder sized for 100 rows must serve any smaller call."""
    from paper_2407_00088_amd.runner import from_problem
    p = wl.make_grouped(0, 1200, 100, 130, 1280, 4, 128, name="holder")
    lin = from_problem(p, layout=L3)
    ref = oracle_fp(p)
    for N in (100, 64, 65, 3, 1):
        out = lin.forward(torch.from_numpy(p.act[:N]).cuda())
        one = lin.forward_one_call(torch.from_numpy(p.act[:N]).cuda())
        torch.cuda.synchronize()
        assert orc.rel_frobenius(out.cpu().numpy(), ref[:N]) <= FP_TOL, N
        assert orc.rel_frobenius(one.cpu().numpy(), ref[:N]) <= FP_TOL, N
