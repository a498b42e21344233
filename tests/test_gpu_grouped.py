"""GPU parity of grouped launches: groups of different shapes in one launch, each group checked
against the oracle's batched Matmul on its own slice of the packed buffers (same tolerance as the
other parity tests)."""
import numpy as np
import pytest
import torch

import paper_2407_21418_amd as ft
import synth_inputs as si
from oracle import contraction as oc

from gpu_util import GUARD, alloc_out, check, check_epilogue, dev_bits, out_view, stream

pytestmark = pytest.mark.gpu


def run_grouped(op, groups, dims, dtype, seed, mode=ft.FT_PLAN_PATCHWORK, scale_b=1.0):
    """dims: per group (batch, M, N, K).  Returns (plan, packed A bits, packed B bits, C as fp64)."""
    s = ft.ft_ukernels_derive(op)
    plan = ft.ft_plan_create_grouped(op, s, groups, mode)
    na, nb, nc = ft.ft_plan_group_layout(plan, len(groups))
    g = np.random.default_rng(seed)
    A = si.normal_bits(g, (max(na, 1),), 1.0, dtype)
    B = si.normal_bits(g, (max(nb, 1),), scale_b, dtype)
    buf = alloc_out(nc)
    dA, dB = dev_bits(A), dev_bits(B)
    ft.ft_launch(plan, dA.data_ptr(), dB.data_ptr(), buf.data_ptr() + 4 * GUARD, stream())
    torch.cuda.synchronize()
    return plan, A, B, out_view(buf, nc)


def check_groups(plan, dims, A, B, Cout, dtype, what):
    for gi, (b, M, N, K) in enumerate(dims):
        oa, ob, oc_ = ft.ft_plan_group_layout(plan, gi)
        if b * M * N == 0:
            continue
        Ag = A[oa:oa + b * M * K].reshape(b, M, K)
        Bg = B[ob:ob + b * K * N].reshape(b, K, N)
        if K == 0:
            assert (Cout[oc_:oc_ + b * M * N] == 0).all(), f"{what} group {gi}: K = 0 must give zeros"
            continue
        ref, refabs = oc.bmm(Ag, Bg, dtype, want_abs=True)
        check(Cout[oc_:oc_ + b * M * N], ref, refabs, f"{what} group {gi} {b}x{M}x{N}x{K}")


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
def test_ragged_attention_scores_in_one_launch(dtype):
    """QK^T of sequences of different lengths, 12 heads each: odd, aligned, tiny, empty and long
    ones next to each other."""
    lengths = [77, 5, 128, 0, 257, 33, 100, 1, 512, 16]
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=dtype, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512, batch_hi=768))
    groups = [ft.ft_shape(batch=12, m=L, n=L) for L in lengths]
    dims = [(12, L, L, 64) for L in lengths]
    for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
        plan, A, B, Cout = run_grouped(op, groups, dims, dtype, 7 + dtype, mode)
        assert np.isfinite(Cout).all(), "an element of the packed C was not written"
        check_groups(plan, dims, A, B, Cout, dtype, f"ragged qk mode {mode}")


def test_ragged_pv_dynamic_reduce_axis():
    """PV: the reduce axis differs from group to group (k tails and partial chunks per group)."""
    lengths = [77, 5, 128, 257, 1, 100, 64]
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, n=64, m_lo=0, m_hi=512, k_lo=0, k_hi=512, batch_hi=768))
    groups = [ft.ft_shape(batch=3, m=L, k=L) for L in lengths]
    dims = [(3, L, 64, L) for L in lengths]
    plan, A, B, Cout = run_grouped(op, groups, dims, ft.FT_F16, 11, scale_b=0.2)
    assert np.isfinite(Cout).all()
    check_groups(plan, dims, A, B, Cout, ft.FT_F16, "ragged pv")


def test_groups_of_unrelated_shapes_and_batches():
    """Every extent dynamic: groups differ in batch, M, N and K; one group alone equals a plain launch."""
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_BF16, m_lo=0, m_hi=512, n_lo=0, n_hi=512,
                                         k_lo=0, k_hi=512, batch_hi=768))
    dims = [(1, 300, 40, 200), (5, 17, 333, 9), (2, 128, 128, 128), (7, 1, 1, 1), (1, 512, 512, 64), (3, 45, 77, 301)]
    groups = [ft.ft_shape(batch=b, m=M, n=N, k=K) for b, M, N, K in dims]
    plan, A, B, Cout = run_grouped(op, groups, dims, ft.FT_BF16, 3, scale_b=0.3)
    assert np.isfinite(Cout).all()
    check_groups(plan, dims, A, B, Cout, ft.FT_BF16, "mixed groups")
    # one group: same bits as the plain batched launch of that shape
    b, M, N, K = dims[5]
    plan1, A1, B1, C1 = run_grouped(op, groups[5:6], dims[5:6], ft.FT_BF16, 99, scale_b=0.3)
    plain = ft.ft_plan_create(op, ft.ft_ukernels_derive(op), groups[5])
    buf = alloc_out(b * M * N)
    dA, dB = dev_bits(A1), dev_bits(B1)
    ft.ft_launch(plain, dA.data_ptr(), dB.data_ptr(), buf.data_ptr() + 4 * GUARD, stream())
    torch.cuda.synchronize()
    assert (out_view(buf, b * M * N) == C1).all()


def test_grouped_launch_with_bias_and_16_bit_output_and_relaunch():
    """Epilogue through a grouped plan (bias per column needs one N: PV-like groups), launched twice."""
    lengths = [33, 200, 7]
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, n=64, m_lo=0, m_hi=512, k_lo=0, k_hi=512, batch_hi=768,
                                         out_dtype=ft.FT_OUT_SAME, epilogue=ft.FT_EPI_BIAS))
    groups = [ft.ft_shape(batch=2, m=L, k=L) for L in lengths]
    plan = ft.ft_plan_create_grouped(op, ft.ft_ukernels_derive(op), groups)
    na, nb, nc = ft.ft_plan_group_layout(plan, len(groups))
    g = np.random.default_rng(5)
    A = si.normal_bits(g, (na,), 1.0, ft.FT_F16)
    B = si.normal_bits(g, (nb,), 0.2, ft.FT_F16)
    bias = g.normal(0, 0.5, 64).astype(np.float32)
    dA, dB, dbias = dev_bits(A), dev_bits(B), torch.from_numpy(bias).cuda()
    out = torch.full((nc + 2 * GUARD,), 0x7e00, dtype=torch.int16, device="cuda")
    for _ in range(2):
        ft.ft_launch_epilogue(plan, dA.data_ptr(), dB.data_ptr(), out.data_ptr() + 2 * GUARD, dbias.data_ptr(), stream())
    torch.cuda.synchronize()
    assert bool((out[:GUARD] == 0x7e00).all()) and bool((out[-GUARD:] == 0x7e00).all()), "write outside C"
    got = out[GUARD:GUARD + nc].cpu().numpy().view(np.float16).astype(np.float64)
    for gi, L in enumerate(lengths):
        oa, ob, oc_ = ft.ft_plan_group_layout(plan, gi)
        ref, refabs = oc.bmm(A[oa:oa + 2 * L * L].reshape(2, L, L), B[ob:ob + 2 * L * 64].reshape(2, L, 64), ft.FT_F16, want_abs=True)
        ref = ref + bias[None, None, :]
        check_epilogue(got[oc_:oc_ + 2 * L * 64], ref, refabs, bias[None, None, :], ft.FT_F16, f"grouped epilogue group {gi}")


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
def test_aligned_groups_take_the_vector_path_and_agree_with_the_general_one(dtype):
    """Lengths that are multiples of 8: the grouped launch runs the LDS-DMA bodies.  The same
    batch from an A that is only 2-byte aligned runs the general bodies; both against the oracle."""
    lengths = [64, 8, 128, 256, 40, 512, 16, 0, 200]
    for which in ("qk", "pv"):
        if which == "qk":
            op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=dtype, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512, batch_hi=768))
            groups = [ft.ft_shape(batch=6, m=L, n=L) for L in lengths]
            dims = [(6, L, L, 64) for L in lengths]
        else:
            op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=dtype, n=64, m_lo=0, m_hi=512, k_lo=0, k_hi=512, batch_hi=768))
            groups = [ft.ft_shape(batch=6, m=L, k=L) for L in lengths]
            dims = [(6, L, 64, L) for L in lengths]
        plan = ft.ft_plan_create_grouped(op, ft.ft_ukernels_derive(op), groups)
        na, nb, nc = ft.ft_plan_group_layout(plan, len(groups))
        g = np.random.default_rng(17 + dtype)
        A = si.normal_bits(g, (na + 8,), 1.0, dtype)
        B = si.normal_bits(g, (nb,), 0.2, dtype)
        dA, dB = dev_bits(A), dev_bits(B)
        for shift in (0, 1):                      # elements: 0 -> 16-byte aligned A, 1 -> 2-byte aligned
            buf = alloc_out(nc)
            ft.ft_launch(plan, dA.data_ptr() + 2 * shift, dB.data_ptr(), buf.data_ptr() + 4 * GUARD, stream())
            torch.cuda.synchronize()
            Cout = out_view(buf, nc)
            assert np.isfinite(Cout).all()
            check_groups(plan, dims, A[shift:shift + na], B, Cout, dtype, f"aligned ragged {which} shift {shift}")


def test_grouped_plan_through_the_timing_entry_points_and_a_graph():
    """Back-to-back launches of one grouped plan on rotating buffers, eagerly and as a replayed HIP
    graph, with eager launches in between: every buffer set holds the bits of a single eager launch."""
    lengths = [77, 128, 5, 300]
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512, batch_hi=768))
    groups = [ft.ft_shape(batch=4, m=L, n=L) for L in lengths]
    dims = [(4, L, L, 64) for L in lengths]
    plan, A, B, single = run_grouped(op, groups, dims, ft.FT_F16, 23)
    check_groups(plan, dims, A, B, single, ft.FT_F16, "single grouped launch")
    nc = single.size
    side = torch.cuda.Stream()
    dA, dB = [dev_bits(A) for _ in range(3)], [dev_bits(B) for _ in range(3)]
    for use_graph in (False, True, True):
        bufs = [alloc_out(nc) for _ in range(3)]
        torch.cuda.synchronize()
        ms = ft.ft_launch_timed(plan, [t.data_ptr() for t in dA], [t.data_ptr() for t in dB],
                                [b.data_ptr() + 4 * GUARD for b in bufs], side.cuda_stream, 7, graph=use_graph)
        torch.cuda.synchronize()
        assert 0.0 < ms < 10.0
        for b in bufs:
            assert np.array_equal(out_view(b, nc), single), f"timed grouped launches, graph={use_graph}"
        buf = alloc_out(nc)
        ft.ft_launch(plan, dA[0].data_ptr(), dB[0].data_ptr(), buf.data_ptr() + 4 * GUARD, stream())
        torch.cuda.synchronize()
        assert np.array_equal(out_view(buf, nc), single), "eager launch between timed runs"
