"""GPU parity of operand B handed over as [N][K] (FT_B_NK: k contiguous, the K matrix of Q K^T, a
linear layer's weight as stored): the same GEMM view (Sec. 4.1; BatchMatmul, Fig. 12 caption), so the
oracle is the same definition on the re-laid-out operand.  Every four-wave standard body alone, the
planner's own plans on ragged shapes with odd N, batched scores of odd lengths, the reduce-axis
split, the fused epilogue, grouped launches, and the error for operands the LDS-DMA bodies cannot
take.  Tolerance as everywhere: 2e-3 of fp32-accumulated 16-bit products."""
import numpy as np
import pytest
import torch

import paper_2407_21418_amd as ft
import synth_inputs as si
from oracle import contraction as oc
from oracle import planner as P

from gpu_util import GUARD, alloc_out, check, check_epilogue, dev_bits, out_view, run, run_epilogue, stream

pytestmark = pytest.mark.gpu

STANDARD_BODIES = [(wm, wn, gm, gn) for (wm, wn, _) in P.wave_tiles() for (gm, gn, gk) in P.WAVE_GRIDS
                   if gk == 1 and gm * gn == 4]


def nk_op(kind, dtype, **kw):
    return ft.ft_op_register(ft.ft_op_desc(kind=kind, dtype=dtype, b_layout=ft.FT_B_NK, **kw))


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
@pytest.mark.parametrize("body", STANDARD_BODIES, ids=lambda b: "w%dx%d_g%dx%d" % b)
def test_every_standard_body_with_b_as_nk(body, dtype):
    """Each four-wave body alone as a forced program: 2 x 4 tiles, ragged tails on both axes with an
    ODD N; reduce extents of several k-tiles with a tail chunk, one k-tile, and a single chunk."""
    wm, wn, gm, gn = body
    tm, tn = wm * gm, wn * gn
    for K in (200, 64, 8):
        N, M = 4 * tn - 3, 2 * tm - 5
        op = nk_op(ft.FT_OP_MATMUL, dtype, n=N, k=K, m_lo=0, m_hi=1 << 16)
        s = ft.ft_ukernels_derive(op)
        infos = [ft.ft_ukset_get(s, i) for i in range(ft.ft_ukset_size(s))]
        assert all(u.gk == 1 and u.gm * u.gn == 4 for u in infos), "this layout derives the four-wave standard grids only"
        ids = [u.id for u in infos if (u.tm, u.tn, u.wm, u.wn, u.gm, u.gn) == (tm, tn, wm, wn, gm, gn)]
        if not ids:
            continue            # the workload filters of this operator dropped the shape
        g = np.random.default_rng(wm * 5 + wn + gm + K + dtype)
        A = si.normal_bits(g, (M, K), 1.0, dtype)
        Bt = si.normal_bits(g, (N, K), 1.0, dtype)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED, ft.ft_forced_program(k1=ids[0], count1=2))
        ref, refabs = oc.matmul_nk(A, Bt, dtype, want_abs=True)
        check(run(plan, A, Bt, M * N), ref, refabs, f"NK body {body} K {K} dtype {dtype}")


@pytest.mark.parametrize("M,N,K,dtype", [(77, 1000, 200, ft.FT_F16), (1232, 768, 768, ft.FT_F16), (300, 4096, 4096, ft.FT_BF16),
                                         (1, 304, 72, ft.FT_BF16), (2048, 333, 512, ft.FT_F16)])
def test_planner_plans_with_b_as_nk(M, N, K, dtype):
    op = nk_op(ft.FT_OP_MATMUL, dtype, n=N, k=K, m_lo=0, m_hi=8192)
    s = ft.ft_ukernels_derive(op)
    g = np.random.default_rng(M + N + K)
    A = si.normal_bits(g, (M, K), 1.0, dtype)
    Bt = si.normal_bits(g, (N, K), K ** -0.5, dtype)
    ref, refabs = oc.matmul_nk(A, Bt, dtype, want_abs=True)
    for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), mode)
        check(run(plan, A, Bt, M * N), ref, refabs, f"NK plan {M}x{N}x{K} mode {mode}")


def test_nk_equals_kn_bit_for_bit_on_the_same_tiles():
    """The two layouts feed the MFMAs the same fragments in the same order: forced onto the same
    uKernel, the fp32 outputs are identical."""
    M, N, K = 315, 768, 776
    g = np.random.default_rng(5)
    A = si.normal_bits(g, (M, K), 1.0, ft.FT_F16)
    B = si.normal_bits(g, (K, N), 1.0, ft.FT_F16)
    outs = []
    for layout, Bm in ((ft.FT_B_KN, B), (ft.FT_B_NK, np.ascontiguousarray(B.T))):
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=N, k=K, m_lo=0, m_hi=8192, b_layout=layout))
        s = ft.ft_ukernels_derive(op)
        ids = [i for i in range(ft.ft_ukset_size(s))
               if (lambda u: (u.tm, u.tn, u.wm, u.wn, u.gk) == (64, 128, 32, 64, 1))(ft.ft_ukset_get(s, i))]
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED, ft.ft_forced_program(k1=ids[0], count1=5))
        outs.append(run(plan, A, Bm, M * N))
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
def test_attention_scores_of_odd_lengths(dtype):
    """Q K^T with K stored [L, 64]: every length, odd ones included, runs the LDS-DMA bodies."""
    op = nk_op(ft.FT_OP_BMM, dtype, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512, batch_hi=768)
    s = ft.ft_ukernels_derive(op)
    for nb, L in ((12, 1), (12, 7), (12, 77), (24, 255), (12, 313), (3, 511), (12, 512), (5, 100)):
        g = np.random.default_rng(L + nb + dtype)
        Q = si.normal_bits(g, (nb, L, 64), 1.0, dtype)
        Kt = si.normal_bits(g, (nb, L, 64), 1.0, dtype)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=nb, m=L, n=L))
        ref, refabs = oc.bmm_nk(Q, Kt, dtype, want_abs=True)
        check(run(plan, Q, Kt, nb * L * L), ref, refabs, f"NK scores batch {nb} L {L} dtype {dtype}")
    # rectangular scores (cross attention): M != N, both odd
    Q = si.normal_bits(np.random.default_rng(1), (6, 133, 64), 1.0, dtype)
    Kt = si.normal_bits(np.random.default_rng(2), (6, 281, 64), 1.0, dtype)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=6, m=133, n=281))
    ref, refabs = oc.bmm_nk(Q, Kt, dtype, want_abs=True)
    check(run(plan, Q, Kt, 6 * 133 * 281), ref, refabs, "NK scores 133 x 281")


def test_reduce_axis_split_with_b_as_nk():
    M, N, K = 571, 768, 3072
    op = nk_op(ft.FT_OP_MATMUL, ft.FT_F16, n=N, k=K, m_lo=0, m_hi=8192)
    s = ft.ft_ukernels_derive(op)
    ids = [i for i in range(ft.ft_ukset_size(s))
           if (lambda u: (u.tm, u.tn, u.wm, u.wn, u.gk) == (64, 64, 32, 32, 1))(ft.ft_ukset_get(s, i))]
    g = np.random.default_rng(9)
    A = si.normal_bits(g, (M, K), 1.0, ft.FT_F16)
    Bt = si.normal_bits(g, (N, K), 0.02, ft.FT_F16)
    ref, refabs = oc.matmul_nk(A, Bt, ft.FT_F16, want_abs=True)
    for kp in (2, 4):
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED, ft.ft_forced_program(k1=ids[0], count1=9, k_parts=kp))
        assert ft.ft_plan_stats_get(plan).k_parts == kp
        check(run(plan, A, Bt, M * N), ref, refabs, f"NK split in {kp} parts")
        check(run(plan, A, Bt, M * N), ref, refabs, f"NK split in {kp} parts, second launch")


@pytest.mark.parametrize("out16", [None, ft.FT_BF16])
def test_bias_and_16_bit_output_with_b_as_nk(out16):
    M, N, K = 272, 2304, 768
    dtype = ft.FT_BF16
    op = nk_op(ft.FT_OP_MATMUL, dtype, n=N, k=K, m_lo=0, m_hi=8192, epilogue=ft.FT_EPI_BIAS,
               out_dtype=ft.FT_OUT_SAME if out16 is not None else ft.FT_OUT_F32)
    s = ft.ft_ukernels_derive(op)
    g = np.random.default_rng(21)
    A = si.normal_bits(g, (M, K), 1.0, dtype)
    Bt = si.normal_bits(g, (N, K), K ** -0.5, dtype)
    bias = g.standard_normal(N).astype(np.float32)
    ref, refabs = oc.matmul_nk(A, Bt, dtype, want_abs=True)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
    got = run_epilogue(plan, A, Bt, M * N, bias=bias, out16=out16)
    check_epilogue(got, ref + bias.astype(np.float64), refabs, bias.astype(np.float64), out16, "NK bias epilogue")


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
def test_ragged_scores_grouped_with_b_as_nk(dtype):
    """Sequences of different, mostly odd lengths in one grouped launch, K matrices stored [L, 64]."""
    lengths = [77, 5, 128, 0, 257, 33, 100, 1, 511, 16]
    op = nk_op(ft.FT_OP_BMM, dtype, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512, batch_hi=768)
    s = ft.ft_ukernels_derive(op)
    groups = [ft.ft_shape(batch=12, m=L, n=L) for L in lengths]
    for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
        plan = ft.ft_plan_create_grouped(op, s, groups, mode)
        na, nb, nc = ft.ft_plan_group_layout(plan, len(groups))
        g = np.random.default_rng(31 + dtype)
        A = si.normal_bits(g, (na,), 1.0, dtype)
        B = si.normal_bits(g, (nb,), 1.0, dtype)
        buf = alloc_out(nc)
        dA, dB = dev_bits(A), dev_bits(B)
        ft.ft_launch(plan, dA.data_ptr(), dB.data_ptr(), buf.data_ptr() + 4 * GUARD, stream())
        torch.cuda.synchronize()
        Cout = out_view(buf, nc)
        assert np.isfinite(Cout).all(), "an element of the packed C was not written"
        for gi, L in enumerate(lengths):
            if L == 0:
                continue
            oa, ob, oc_ = ft.ft_plan_group_layout(plan, gi)
            Ag = A[oa:oa + 12 * L * 64].reshape(12, L, 64)
            Bg = B[ob:ob + 12 * L * 64].reshape(12, L, 64)
            ref, refabs = oc.bmm_nk(Ag, Bg, dtype, want_abs=True)
            check(Cout[oc_:oc_ + 12 * L * L], ref, refabs, f"NK grouped scores L {L} mode {mode}")


def test_operands_the_nk_bodies_cannot_take_are_refused():
    """Rows shorter than one 16-byte chunk (K < 8) have no body for this layout: FT_ERR_UNSUPPORTED, C untouched.
    A reduce extent that is not a multiple of 8 and operands that are only 2-byte aligned run."""
    op = nk_op(ft.FT_OP_BMM, ft.FT_F16, n=64, m_lo=0, m_hi=512, k_lo=0, k_hi=512, batch_hi=768)
    s = ft.ft_ukernels_derive(op)
    A = torch.zeros(4 * 77 * 77 + 64, dtype=torch.int16, device="cuda")
    B = torch.zeros(4 * 64 * 77 + 64, dtype=torch.int16, device="cuda")
    Cd = torch.full((4 * 77 * 64,), 7.0, dtype=torch.float32, device="cuda")
    plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=4, m=77, k=5))
    with pytest.raises(ft.FtError) as e:
        ft.ft_launch(plan, A.data_ptr(), B.data_ptr(), Cd.data_ptr(), stream())
    assert e.value.status == ft.FT_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((Cd == 7.0).all())
    for k, shift in ((77, 0), (72, 2), (77, 6)):
        Cd.fill_(7.0)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=4, m=77, k=k))
        ft.ft_launch(plan, A.data_ptr() + shift, B.data_ptr() + shift, Cd.data_ptr(), stream())
        torch.cuda.synchronize()
        assert bool((Cd == 0.0).all())
