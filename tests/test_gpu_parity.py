"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Tolerance: max relative error 2e-3 (fp32 accumulation of fp16/bf16 products),
both against the output scale and element-wise against sum|a||b|; plans bit-exact."""
import numpy as np
import pytest
import torch

import paper_2407_21418_amd as ft
import synth_inputs as si
from oracle import contraction as oc
from oracle import planner as P

from gpu_util import GUARD, REL_TOL, alloc_out, check, check_epilogue, dev_bits, matmul_op, out_view, run, run_epilogue, stream
from oracle import epilogue as oe

pytestmark = pytest.mark.gpu


def test_hw_query_reports_gfx950():
    hw = ft.ft_hw_query(0)
    assert hw.num_cus == 256 and hw.wave_size == 64 and hw.lds_bytes_per_cu == 163840


def test_config0_odd_m_matmul():
    p = si.config0()
    op = matmul_op(p["N"], p["K"], ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=p["M"]), mode)
        got = run(plan, p["A"], p["B"], p["M"] * p["N"])
        ref, refabs = oc.matmul(p["A"], p["B"], si.F16, want_abs=True)
        check(got, ref, refabs, f"config0 mode {mode}")


def family():
    op = P.Op(P.OP_BMM, P.F16, k_range=(0, 4096), m_range=(0, 8192), n_range=(0, 8192))
    return [(u.tm, u.tn, u.wm, u.wn, u.gm, u.gn) for u in P.derive_ukernels(op)]


@pytest.mark.parametrize("aligned", [True, False], ids=["dma", "general"])
@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
@pytest.mark.parametrize("body", family(), ids=lambda b: "t%dx%d_w%dx%d" % b[:4])
def test_every_ukernel_body(body, dtype, aligned):
    """Each compiled body alone (forced single-uKernel program): 2 x 2 tiles with a ragged tail
    on both axes, a k extent that is not a multiple of the k-tile, and batch 2.  aligned: row
    lengths are multiples of 8 elements (LDS-DMA bodies, zero-page k tail); otherwise odd row
    lengths (general bodies: unaligned vector loads, chunks that straddle a row's end fetched from
    inside the row and shifted)."""
    tm, tn, wm, wn, gm, gn = body
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=dtype, m_lo=0, m_hi=8192, n_lo=0, n_hi=8192,
                                         k_lo=0, k_hi=4096))
    s = ft.ft_ukernels_derive(op)
    ids = [i for i in range(ft.ft_ukset_size(s))
           if (lambda u: (u.tm, u.tn, u.wm, u.wn) == (tm, tn, wm, wn))(ft.ft_ukset_get(s, i))]
    assert len(ids) == 1
    M, N, K, nb = (2 * tm - 5, 2 * tn - 8, 200, 2) if aligned else (2 * tm - 5, 2 * tn - 11, 203, 2)
    g = np.random.default_rng(tm * 7 + tn * 3 + wm + dtype + 1000 * aligned)
    A = si.normal_bits(g, (nb, M, K), 1.0, dtype)
    B = si.normal_bits(g, (nb, K, N), 1.0, dtype)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=nb, m=M, n=N, k=K), ft.FT_PLAN_FORCED,
                             ft.ft_forced_program(k1=ids[0], count1=2))
    st = ft.ft_plan_stats_get(plan)
    assert st.n_tiles == nb * 4
    got = run(plan, A, B, nb * M * N)
    ref, refabs = oc.bmm(A, B, dtype, want_abs=True)
    check(got, ref, refabs, f"body {body} dtype {dtype}")


RING_BODIES = [  # (tm, tn, wm, wn, teams): single-team loops of both fragment schemes, split-k wave grids
    (128, 64, 64, 32, 1), (64, 64, 32, 32, 1), (128, 128, 64, 64, 1), (256, 128, 128, 64, 1), (32, 128, 16, 64, 1),
    (64, 64, 64, 64, 1), (16, 64, 16, 64, 1),
]


@pytest.mark.parametrize("zeta", [1, 2, 4])
@pytest.mark.parametrize("body", RING_BODIES, ids=lambda b: "t%dx%d_w%dx%d_g%d" % b)
def test_ring_depths_and_short_reduce_axes(body, zeta):
    """The k loops keep one to three (single team) or ring depth - 1 (two teams, split-k grid) tiles in
    flight: every ring depth the planner can hand over (zeta workgroups per CU sharing the LDS) against
    reduce extents of one k-tile up to more than the deepest ring, whole and ragged, so that prologue,
    steady state and drain of each loop run with every count of tiles."""
    tm, tn, wm, wn, teams = body
    tuning = ft.ft_tuning_default()
    tuning.zeta = zeta
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, m_lo=0, m_hi=8192, n_lo=0, n_hi=8192,
                                         k_lo=0, k_hi=4096))
    s = ft.ft_ukernels_derive(op, ft.ft_hw_query(0), tuning)
    ids = [i for i in range(ft.ft_ukset_size(s))
           if (lambda u: (u.tm, u.tn, u.wm, u.wn) == (tm, tn, wm, wn) and (u.gk == 2) == (teams == 2)
               and u.gm * u.gn * (1 if u.gk == 2 else u.gk) == 4)(ft.ft_ukset_get(s, i))]
    if not ids:
        pytest.skip("this ring does not fit the LDS share of that zeta")
    M, N = 2 * tm - 5, 2 * tn - 8
    for K in (64, 72, 128, 192, 200, 256, 320, 448, 584):
        g = np.random.default_rng(K * 31 + tm + tn + zeta)
        A = si.normal_bits(g, (1, M, K), 1.0, ft.FT_F16)
        B = si.normal_bits(g, (1, K, N), 1.0, ft.FT_F16)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=1, m=M, n=N, k=K), ft.FT_PLAN_FORCED,
                                 ft.ft_forced_program(k1=ids[0], count1=2))
        got = run(plan, A, B, M * N)
        ref, refabs = oc.bmm(A, B, ft.FT_F16, want_abs=True)
        check(got, ref, refabs, f"body {body} zeta {zeta} K {K} stages {ft.ft_ukset_get(s, ids[0]).stages}")


@pytest.mark.parametrize("body", [(128, 64, 64, 32), (64, 64, 32, 32), (64, 16, 16, 16)], ids=lambda b: "t%dx%d_w%dx%d" % b)
def test_two_team_rings_on_short_reduce_axes(body):
    """Two-team uKernels (rings of 3, 5 and 8 stages per team) on reduce extents from the shortest they
    are derived for (four k-tiles) up: each team then runs its loop with fewer tiles than its ring holds,
    with exactly as many, and with more; odd tile counts give the teams different numbers of tiles."""
    tm, tn, wm, wn = body
    N = 768
    for K in (256, 264, 320, 448, 576, 584, 1096):
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=N, k=K, m_lo=1, m_hi=8192))
        s = ft.ft_ukernels_derive(op)
        ids = [i for i in range(ft.ft_ukset_size(s))
               if (lambda u: (u.tm, u.tn, u.wm, u.wn, u.gk) == (tm, tn, wm, wn, 2))(ft.ft_ukset_get(s, i))]
        assert len(ids) == 1
        M = 2 * tm - 5
        g = np.random.default_rng(K * 17 + tm + tn)
        A = si.normal_bits(g, (M, K), 1.0, ft.FT_F16)
        B = si.normal_bits(g, (K, N), 1.0, ft.FT_F16)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED, ft.ft_forced_program(k1=ids[0], count1=2))
        got = run(plan, A, B, M * N)
        ref, refabs = oc.matmul(A, B, ft.FT_F16, want_abs=True)
        check(got, ref, refabs, f"two-team body {body} K {K} stages {ft.ft_ukset_get(s, ids[0]).stages}")


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
def test_permutation_matrix_is_bit_exact(dtype):
    """A = permutation matrix: every output is a single product 1*b, exact in fp32; pins the
    MFMA operand and accumulator lane layouts and the LDS swizzles."""
    g = np.random.default_rng(4)
    n, N = 384, 768
    B = si.normal_bits(g, (n, N), 1.0, dtype)
    perm = g.permutation(n)
    Pm = np.zeros((n, n), dtype=np.float32)
    Pm[np.arange(n), perm] = 1.0
    A = si.to_bits(Pm, dtype)
    op = matmul_op(N, n, dtype)
    s = ft.ft_ukernels_derive(op)
    want = oc.decode(B, dtype)[perm]
    for i in range(ft.ft_ukset_size(s)):
        u = ft.ft_ukset_get(s, i)
        if n % u.tm:
            continue
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=n), ft.FT_PLAN_FORCED,
                                 ft.ft_forced_program(k1=i, count1=n // u.tm))
        got = run(plan, A, B, n * N).reshape(n, N)
        assert np.array_equal(got, want), (u.tm, u.tn, u.wm, u.wn)


@pytest.mark.parametrize("M,N,K", [(80, 768, 768), (272, 3072, 768), (528, 768, 3072), (1232, 768, 768)])
def test_bert_shapes_patchwork_and_baseline(M, N, K):
    p = si.config1_problem(M, N, K)
    op = matmul_op(N, K, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    ref, refabs = oc.matmul(p["A"], p["B"], si.F16, want_abs=True)
    oop = P.Op(P.OP_MATMUL, P.F16, n=N, k=K, m_range=(0, 8192))
    ouk = P.derive_ukernels(oop)
    for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), mode)
        assert ft.ft_plan_descriptors(plan) == b"".join(d.pack() for d in P.plan(oop, ouk, (1, M, N, K), mode).descs)
        check(run(plan, p["A"], p["B"], M * N), ref, refabs, f"bert {M}x{N}x{K} mode {mode}")


def test_two_ukernel_program_mixed_in_one_launch():
    """A program of two different uKernel shapes runs as ONE launch over the descriptor table."""
    M, N, K = 1232, 768, 768
    p = si.config1_problem(M, N, K)
    op = matmul_op(N, K, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    infos = [ft.ft_ukset_get(s, i) for i in range(ft.ft_ukset_size(s))]
    big = next(u for u in infos if (u.tm, u.tn, u.gk) == (128, 64, 1))
    small = next(u for u in infos if (u.tm, u.tn, u.gk) == (16, 64, 4))
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED,
                             ft.ft_forced_program(k1=big.id, count1=9, k2=small.id, count2=5))
    st = ft.ft_plan_stats_get(plan)
    assert st.n_ukernels == 2 and st.n_tiles == 9 * 12 + 5 * 12
    ref, refabs = oc.matmul(p["A"], p["B"], si.F16, want_abs=True)
    check(run(plan, p["A"], p["B"], M * N), ref, refabs, "mixed program")


@pytest.mark.parametrize("L", [1, 7, 8, 9, 15, 33, 77, 100, 257])
def test_attention_bmm_dynamic_length(L):
    """QK^T (two dynamic space axes) and PV (dynamic reduce axis) with odd lengths: rows that
    are not 16-byte aligned, partial chunks, k tails."""
    nb = 24
    qk_op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512))
    pv_op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, n=64, m_lo=0, m_hi=512, k_lo=0, k_hi=512))
    for which, op, shape in (("qk", qk_op, ft.ft_shape(batch=nb, m=L, n=L)), ("pv", pv_op, ft.ft_shape(batch=nb, m=L, k=L))):
        p = si.config2_problem(2, L, which)
        s = ft.ft_ukernels_derive(op)
        for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
            plan = ft.ft_plan_create(op, s, shape, mode)
            got = run(plan, p["A"], p["B"], nb * p["M"] * p["N"])
            ref, refabs = oc.bmm(p["A"], p["B"], si.F16, want_abs=True)
            check(got, ref, refabs, f"{which} L={L} mode {mode}")


@pytest.mark.parametrize("res,batch", [(5, 2), (13, 3), (28, 8), (37, 8)])
def test_conv2d_implicit_gemm(res, batch):
    p = si.config4_problem(res, batch=batch)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_CONV2D, dtype=ft.FT_F16, c_in=64, c_out=128, r=3, s=3,
                                         stride=1, pad=1, m_lo=0, m_hi=1 << 22))
    s = ft.ft_ukernels_derive(op)
    ref, refabs = oc.conv2d_nhwc(p["X"], p["Wt"], si.F16, want_abs=True)
    for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
        plan = ft.ft_plan_create(op, s, ft.ft_shape(img_n=batch, img_h=res, img_w=res), mode)
        got = run(plan, p["X"], p["Wt"], batch * res * res * 128)
        check(got, ref, refabs, f"conv res {res} mode {mode}")


def test_conv2d_dma_gather_wide_channels_and_stride():
    """LDS-DMA gather path (c_in a multiple of 64): c_in = 128 so a filter tap spans two k-tiles,
    stride 2, c_out not a multiple of any tile width."""
    g = np.random.default_rng(78)
    n, H, W, Cin, Cout = 3, 17, 13, 128, 72
    X = si.normal_bits(g, (n, H, W, Cin), 1.0, si.F16)
    Wt = si.normal_bits(g, (3, 3, Cin, Cout), 0.1, si.F16)
    for stride, pad in ((1, 1), (2, 1), (2, 0)):
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_CONV2D, dtype=ft.FT_F16, c_in=Cin, c_out=Cout, r=3, s=3,
                                             stride=stride, pad=pad, m_lo=0, m_hi=1 << 20))
        s = ft.ft_ukernels_derive(op)
        ref, refabs = oc.conv2d_nhwc(X, Wt, si.F16, stride=stride, pad=pad, want_abs=True)
        for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
            plan = ft.ft_plan_create(op, s, ft.ft_shape(img_n=n, img_h=H, img_w=W), mode)
            check(run(plan, X, Wt, ref.size), ref, refabs, f"conv dma stride {stride} pad {pad} mode {mode}")


def test_conv2d_full_size_sampled_pixels():
    """Configured convolution at 8 x 112 x 112 (M = 100352 output pixels) in the default plan; the
    oracle checks image corners, edges, tile-boundary pixels and random ones."""
    res, batch = 112, 8
    p = si.config4_problem(res, batch=batch)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_CONV2D, dtype=ft.FT_F16, c_in=64, c_out=128, r=3, s=3,
                                         stride=1, pad=1, m_lo=0, m_hi=1 << 22))
    s = ft.ft_ukernels_derive(op)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(img_n=batch, img_h=res, img_w=res))
    M = batch * res * res
    X, Wt = dev_bits(p["X"]), dev_bits(p["Wt"])
    Y = torch.full((M, 128), float("nan"), dtype=torch.float32, device="cuda")
    ft.ft_launch(plan, X.data_ptr(), Wt.data_ptr(), Y.data_ptr(), stream())
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Y).all())
    g = np.random.default_rng(6)
    special = [0, res - 1, res, res * res - 1, res * res, M - 1, M - res, 127, 128, 129, 511, 512, 513,
               (3 * res + 5) * res, (3 * res + 5) * res + res - 1]
    pix = np.unique(np.concatenate([g.integers(0, M, 300), special])).astype(np.int64)
    ref, refabs = oc.conv2d_nhwc(p["X"], p["Wt"], si.F16, pixels=pix, want_abs=True)
    got = Y[torch.from_numpy(pix).cuda()].cpu().numpy().astype(np.float64)
    check(got, ref, refabs, "conv 8x112x112")


def test_attention_full_size_sampled_batches():
    """Largest attention problem (B = 64, L = 512: 768 batch entries) in the default plans; the
    oracle recomputes a few whole batch entries, the rest must be finite."""
    nb, L = 768, 512
    g = np.random.default_rng(12)
    for which, (M, K, N), kw in (("qk", (L, 64, L), dict(k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512)),
                                 ("pv", (L, L, 64), dict(n=64, m_lo=0, m_hi=512, k_lo=0, k_hi=512))):
        A = torch.randn((nb, M, K), device="cuda").half()
        B = torch.randn((nb, K, N), device="cuda").half()
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, **kw))
        s = ft.ft_ukernels_derive(op)
        shape = ft.ft_shape(batch=nb, m=L, n=L) if which == "qk" else ft.ft_shape(batch=nb, m=L, k=L)
        plan = ft.ft_plan_create(op, s, shape)
        Cd = torch.full((nb, M, N), float("nan"), dtype=torch.float32, device="cuda")
        ft.ft_launch(plan, A.data_ptr(), B.data_ptr(), Cd.data_ptr(), stream())
        torch.cuda.synchronize()
        assert bool(torch.isfinite(Cd).all())
        for b in (0, 1, 383, 767, int(g.integers(0, nb))):
            Ab = A[b].cpu().numpy().view(np.uint16)
            Bb = B[b].cpu().numpy().view(np.uint16)
            ref, refabs = oc.matmul(Ab, Bb, si.F16, want_abs=True)
            check(Cd[b].cpu().numpy().astype(np.float64), ref, refabs, f"{which} batch {b}")


def test_conv2d_general_geometry():
    """Stride 2, no padding, channel count not a multiple of 8 (element-wise gather path)."""
    g = np.random.default_rng(77)
    n, H, W, Cin, Cout = 2, 11, 9, 12, 32
    X = si.normal_bits(g, (n, H, W, Cin), 1.0, si.F16)
    Wt = si.normal_bits(g, (3, 3, Cin, Cout), 1.0, si.F16)
    for stride, pad in ((2, 0), (2, 1), (1, 0)):
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_CONV2D, dtype=ft.FT_F16, c_in=Cin, c_out=Cout, r=3, s=3,
                                             stride=stride, pad=pad, m_lo=0, m_hi=1 << 20))
        s = ft.ft_ukernels_derive(op)
        ref, refabs = oc.conv2d_nhwc(X, Wt, si.F16, stride=stride, pad=pad, want_abs=True)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(img_n=n, img_h=H, img_w=W))
        got = run(plan, X, Wt, ref.size)
        check(got, ref, refabs, f"conv stride {stride} pad {pad}")


def test_llm_bf16_sampled_rows_full_size():
    """Largest configured GEMM (8192 x 11008 x 4096, bf16) in the launch configuration the
    benchmark uses; the oracle checks 64 sampled rows plus the rows around tile boundaries."""
    M, N = 8192, 11008
    p = si.config3_problem(M, N)
    op = matmul_op(N, si.LLM_K, ft.FT_BF16)
    s = ft.ft_ukernels_derive(op)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
    A, B = dev_bits(p["A"]), dev_bits(p["B"])
    Cd = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ft.ft_launch(plan, A.data_ptr(), B.data_ptr(), Cd.data_ptr(), stream())
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Cd).all())
    g = np.random.default_rng(5)
    rows = np.unique(np.concatenate([g.integers(0, M, 64), [0, 1, 127, 128, 255, 256, 257, M - 2, M - 1]])).astype(np.int64)
    ref, refabs = oc.matmul(p["A"], p["B"], si.BF16, rows=rows, want_abs=True)
    got = Cd[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    check(got, ref, refabs, "llm 8192x11008")


@pytest.mark.parametrize("M", [1, 3, 16, 45, 300])
def test_llm_bf16_small_token_counts(M):
    N = 4096
    p = si.config3_problem(M, N)
    op = matmul_op(N, si.LLM_K, ft.FT_BF16)
    s = ft.ft_ukernels_derive(op)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
    ref, refabs = oc.matmul(p["A"], p["B"], si.BF16, want_abs=True)
    check(run(plan, p["A"], p["B"], M * N), ref, refabs, f"llm M={M}")


def test_empty_and_degenerate_inputs():
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, n=64, m_lo=0, m_hi=512, k_lo=0, k_hi=512))
    s = ft.ft_ukernels_derive(op)
    # empty output: nothing is launched, nothing is touched
    plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=3, m=0, k=7))
    assert ft.ft_plan_stats_get(plan).n_tiles == 0
    buf = alloc_out(16)
    ft.ft_launch(plan, 0, 0, buf.data_ptr(), stream())
    torch.cuda.synchronize()
    assert bool(torch.isnan(buf[256:272]).all())
    # empty reduce axis: the sum over no terms is zero
    plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=2, m=5, k=0))
    A = torch.zeros(16, dtype=torch.int16, device="cuda")
    got = out_view_after(plan, A, A, 2 * 5 * 64)
    assert np.array_equal(got, np.zeros(2 * 5 * 64))


def out_view_after(plan, A, B, n):
    buf = alloc_out(n)
    ft.ft_launch(plan, A.data_ptr(), B.data_ptr(), buf.data_ptr() + 4 * 256, stream())
    torch.cuda.synchronize()
    return out_view(buf, n)


def test_launch_on_a_side_stream_and_relaunch():
    p = si.config1_problem(272, 768, 768)
    op = matmul_op(768, 768, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=272))
    ref, refabs = oc.matmul(p["A"], p["B"], si.F16, want_abs=True)
    side = torch.cuda.Stream()
    A, B = dev_bits(p["A"]), dev_bits(p["B"])
    torch.cuda.synchronize()
    for _ in range(3):
        buf = alloc_out(272 * 768)
        torch.cuda.synchronize()
        ft.ft_launch(plan, A.data_ptr(), B.data_ptr(), buf.data_ptr() + 4 * 256, side.cuda_stream)
        side.synchronize()
        check(out_view(buf, 272 * 768), ref, refabs, "side stream")


# ---- fused epilogue and 16-bit output (Dense + bias-add, Sec. 6.2) ----------------------------------
@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
@pytest.mark.parametrize("out16,with_bias", [(False, True), (True, False), (True, True)])
@pytest.mark.parametrize("M", [1, 77, 300, 1232])
def test_matmul_bias_and_narrow_output(M, out16, with_bias, dtype):
    """C = A B (+ bias), stored as fp32 or rounded once to the inputs' 16-bit type.  M = 1 and 77 run
    split-k bodies, 300 a two-uKernel program, 1232 large tiles with an edge; N is not a multiple of
    any tile width, so column-edge wave tiles take the predicated store."""
    N, K = 760, 768
    g = np.random.default_rng(1000 * M + 10 * dtype + 2 * out16 + with_bias)
    A = si.normal_bits(g, (M, K), 1.0, dtype)
    B = si.normal_bits(g, (K, N), 0.05, dtype)
    bias = g.normal(0, 1.0, N).astype(np.float32) if with_bias else None
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dtype, n=N, k=K, m_lo=0, m_hi=8192,
                                         out_dtype=ft.FT_OUT_SAME if out16 else ft.FT_OUT_F32,
                                         epilogue=ft.FT_EPI_BIAS if with_bias else ft.FT_EPI_NONE))
    s = ft.ft_ukernels_derive(op)
    ref, refabs = oc.matmul(A, B, dtype, want_abs=True)
    if with_bias:
        ref = oe.add_bias(ref, bias)
    for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), mode)
        got = run_epilogue(plan, A, B, M * N, bias=bias, out16=dtype if out16 else None)
        check_epilogue(got, ref, refabs, bias, dtype if out16 else None, f"epilogue M={M} out16={out16} bias={with_bias} mode {mode}")


def test_epilogue_argument_checks():
    op_b = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=64, k=64, m_lo=0, m_hi=64, epilogue=ft.FT_EPI_BIAS))
    op_n = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=64, k=64, m_lo=0, m_hi=64))
    buf = torch.zeros(64 * 64, dtype=torch.float32, device="cuda")
    ab = torch.zeros(64 * 64, dtype=torch.int16, device="cuda")
    for op, bias_ptr in ((op_b, 0), (op_n, buf.data_ptr())):
        plan = ft.ft_plan_create(op, ft.ft_ukernels_derive(op), ft.ft_shape(m=64))
        with pytest.raises(ft.FtError) as e:
            ft.ft_launch_epilogue(plan, ab.data_ptr(), ab.data_ptr(), buf.data_ptr(), bias_ptr, stream())
        assert e.value.status == ft.FT_ERR_INVALID_ARG
    with pytest.raises(ft.FtError):
        ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=64, k=64, m_lo=0, m_hi=64, out_dtype=7))


def test_conv_and_bmm_with_epilogue():
    """Convolution (LDS-DMA gather path) with bias and fp16 output; BMM with odd L (general bodies)
    and bf16 output."""
    g = np.random.default_rng(91)
    n, H, W, Cin, Cout = 2, 19, 23, 64, 128
    X = si.normal_bits(g, (n, H, W, Cin), 1.0, si.F16)
    Wt = si.normal_bits(g, (3, 3, Cin, Cout), 0.05, si.F16)
    bias = g.normal(0, 0.5, Cout).astype(np.float32)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_CONV2D, dtype=ft.FT_F16, c_in=Cin, c_out=Cout, r=3, s=3, stride=1, pad=1,
                                         m_lo=0, m_hi=1 << 20, out_dtype=ft.FT_OUT_SAME, epilogue=ft.FT_EPI_BIAS))
    s = ft.ft_ukernels_derive(op)
    ref, refabs = oc.conv2d_nhwc(X, Wt, si.F16, want_abs=True)
    ref = oe.add_bias(ref, bias)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(img_n=n, img_h=H, img_w=W))
    got = run_epilogue(plan, X, Wt, ref.size, bias=bias, out16=ft.FT_F16)
    check_epilogue(got, ref, refabs, bias, ft.FT_F16, "conv + bias -> fp16")
    nb, L = 5, 77
    A = si.normal_bits(g, (nb, L, 64), 1.0, si.BF16)
    B = si.normal_bits(g, (nb, 64, L), 1.0, si.BF16)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_BF16, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512,
                                         out_dtype=ft.FT_OUT_SAME))
    s = ft.ft_ukernels_derive(op)
    ref, refabs = oc.bmm(A, B, si.BF16, want_abs=True)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=nb, m=L, n=L))
    got = run_epilogue(plan, A, B, ref.size, out16=ft.FT_BF16)
    check_epilogue(got, ref, refabs, None, ft.FT_BF16, "bmm -> bf16")


def test_timing_entry_points_leave_correct_results():
    """ft_launch_timed and ft_launch_timed_graph (stream capture + replay of the same launches) run
    the plan on rotating buffer sets: every set must hold the oracle's result afterwards, after
    several replays with eager launches and synchronisations in between."""
    p = si.config1_problem(272, 768, 768)
    op = matmul_op(768, 768, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=272))
    ref, refabs = oc.matmul(p["A"], p["B"], si.F16, want_abs=True)
    side = torch.cuda.Stream()
    n_sets = 3
    A = [dev_bits(p["A"]) for _ in range(n_sets)]
    B = [dev_bits(p["B"]) for _ in range(n_sets)]
    for use_graph in (False, True, True):
        bufs = [alloc_out(272 * 768) for _ in range(n_sets)]
        torch.cuda.synchronize()
        ms = ft.ft_launch_timed(plan, [t.data_ptr() for t in A], [t.data_ptr() for t in B],
                                [b.data_ptr() + 4 * GUARD for b in bufs], side.cuda_stream, 7, graph=use_graph)
        torch.cuda.synchronize()
        assert 0.0 < ms < 10.0
        for b in bufs:
            check(out_view(b, 272 * 768), ref, refabs, f"timed launch graph={use_graph}")
        # eager work between the replays
        check(run(plan, p["A"], p["B"], 272 * 768), ref, refabs, "eager launch between timed runs")


def test_cached_plan_launches_like_a_fresh_one():
    p = si.config1_problem(528, 768, 768)
    op = matmul_op(768, 768, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    cached = ft.ft_plan_cached(op, s, ft.ft_shape(m=528))
    assert ft.ft_plan_cached(op, s, ft.ft_shape(m=528)).ptr == cached.ptr
    ref, refabs = oc.matmul(p["A"], p["B"], si.F16, want_abs=True)
    got = run(cached, p["A"], p["B"], 528 * 768)
    check(got, ref, refabs, "cached plan")
    assert np.array_equal(got, run(ft.ft_plan_create(op, s, ft.ft_shape(m=528)), p["A"], p["B"], 528 * 768))


def test_chained_dense_layers_on_one_stream():
    """Three Dense + bias-add launches (Sec. 6.2) issued back to back on one stream with no host
    wait, each reading the 16-bit C of the one before it, plans from the per-shape cache: every
    stage is checked against the oracle applied to the bits that stage actually read."""
    M, H, F = 300, 768, 3072
    g = np.random.default_rng(4242)
    dt = ft.FT_F16
    ctx = si.normal_bits(g, (M, H), 1.0, dt)
    stages = [("o", H, H), ("ffn1", F, H), ("ffn2", H, F)]
    Wb = {n: si.normal_bits(g, (k, nn), 0.03, dt) for n, nn, k in stages}
    bias = {n: g.normal(0, 0.5, nn).astype(np.float32) for n, nn, k in stages}
    plans = {}
    for n, nn, k in stages:
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dt, n=nn, k=k, m_lo=1, m_hi=8192,
                                             out_dtype=ft.FT_OUT_SAME, epilogue=ft.FT_EPI_BIAS))
        plans[n] = ft.ft_plan_cached(op, ft.ft_ukernels_derive(op), ft.ft_shape(m=M))
    dW = {n: dev_bits(Wb[n]) for n in Wb}
    dB = {n: torch.from_numpy(bias[n]).cuda() for n in bias}
    bufs = {"ctx": dev_bits(ctx)}
    for n, nn, k in stages:
        bufs[n] = torch.full((M * nn,), 0x7e00, dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    src = "ctx"
    for n, nn, k in stages:
        ft.ft_launch_epilogue(plans[n], bufs[src].data_ptr(), dW[n].data_ptr(), bufs[n].data_ptr(), dB[n].data_ptr(), stream())
        src = n
    torch.cuda.synchronize()
    src_bits = ctx
    for n, nn, k in stages:
        got_bits = bufs[n].cpu().numpy().view(np.uint16).reshape(M, nn)
        ref, refabs = oc.matmul(src_bits, Wb[n], dt, want_abs=True)
        ref = oe.add_bias(ref, bias[n])
        check_epilogue(got_bits.view(np.float16).astype(np.float64), ref, refabs, bias[n], dt, f"chained stage {n}")
        src_bits = got_bits


@pytest.mark.parametrize("K", [1, 8, 12])
def test_reduce_axis_of_a_few_elements(K):
    """A static K below anything Eq. 6's threshold admits: the uKernel set is still derived and the
    product is right (bf16, odd M, N = 304)."""
    M, N = 543, 304
    g = np.random.default_rng(31 + K)
    A = si.normal_bits(g, (M, K), 1.0, ft.FT_BF16)
    B = si.normal_bits(g, (K, N), 1.0, ft.FT_BF16)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_BF16, n=N, k=K, m_lo=0, m_hi=1024))
    plan = ft.ft_plan_create(op, ft.ft_ukernels_derive(op), ft.ft_shape(m=M))
    ref, refabs = oc.matmul(A, B, ft.FT_BF16, want_abs=True)
    check(run(plan, A, B, M * N), ref, refabs, f"K={K}")
