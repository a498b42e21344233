"""ft_launch_noalloc (for callers that cannot allocate device memory) against ft_launch on the same
inputs: bit-identical outputs, on two calls in a row that share the library's static workspace, the
second with a smaller input; a plan that never had a device table; and the size limit."""
import numpy as np
import pytest
import torch

import paper_2407_21418_amd as ft
import synth_inputs as si

from gpu_util import GUARD, alloc_out, dev_bits, matmul_op, out_view, run, stream

pytestmark = pytest.mark.gpu


def run_noalloc(plan, A_bits, B_bits, n_out):
    A, B = dev_bits(A_bits), dev_bits(B_bits)
    buf = alloc_out(n_out)
    ft.ft_launch_noalloc(plan, A.data_ptr(), B.data_ptr(), buf.data_ptr() + 4 * GUARD, 0, stream())
    torch.cuda.synchronize()
    return out_view(buf, n_out)


def test_noalloc_matches_the_allocating_entry_point_on_two_calls_in_a_row():
    N, K = 768, 3072
    op = matmul_op(N, K, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    seen_split = 0
    for M in (528, 80):                                   # the second call is the smaller one
        p = si.config1_problem(M, N, K)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
        st = ft.ft_plan_stats_get(plan)
        seen_split += st.k_parts > 1
        want = run(plan, p["A"], p["B"], M * N)
        # the same plan, then a plan that was never given anything on the device
        got = run_noalloc(plan, p["A"], p["B"], M * N)
        assert np.array_equal(got, want), f"M={M} k_parts={st.k_parts}"
        host_only = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_PATCHWORK | ft.FT_PLAN_HOST_ONLY)
        assert ft.ft_plan_stats_get(host_only).table_order == 0
        got = run_noalloc(host_only, p["A"], p["B"], M * N)
        assert np.array_equal(got, want), f"host-only plan, M={M}"
    assert seen_split == 2, "both shapes are meant to split the reduce axis (they use the static workspace)"


def test_noalloc_back_to_back_on_one_stream_without_host_waits():
    """Launches of different plans queued on one stream share the workspace one after the other."""
    N, K = 768, 3072
    op = matmul_op(N, K, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    jobs = []
    for M in (528, 80, 272, 528):
        p = si.config1_problem(M, N, K)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_PATCHWORK | ft.FT_PLAN_HOST_ONLY)
        ref_plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
        jobs.append((M, plan, dev_bits(p["A"]), dev_bits(p["B"]), alloc_out(M * N), run(ref_plan, p["A"], p["B"], M * N)))
    torch.cuda.synchronize()
    for M, plan, A, B, buf, _ in jobs:
        ft.ft_launch_noalloc(plan, A.data_ptr(), B.data_ptr(), buf.data_ptr() + 4 * GUARD, 0, stream())
    torch.cuda.synchronize()
    for M, _, _, _, buf, want in jobs:
        assert np.array_equal(out_view(buf, M * N), want), M


def test_noalloc_with_bias_and_without_split():
    M, N, K = 300, 760, 768
    g = np.random.default_rng(5)
    A = si.normal_bits(g, (M, K), 1.0, ft.FT_BF16)
    B = si.normal_bits(g, (K, N), 0.05, ft.FT_BF16)
    bias = g.normal(0, 1.0, N).astype(np.float32)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_BF16, n=N, k=K, m_lo=0, m_hi=8192, epilogue=ft.FT_EPI_BIAS))
    s = ft.ft_ukernels_derive(op)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_PATCHWORK | ft.FT_PLAN_HOST_ONLY)
    ref_plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
    dA, dB, dbias = dev_bits(A), dev_bits(B), torch.from_numpy(bias).cuda()
    outs = []
    for which in (0, 1):
        buf = alloc_out(M * N)
        if which == 0:
            ft.ft_launch_epilogue(ref_plan, dA.data_ptr(), dB.data_ptr(), buf.data_ptr() + 4 * GUARD, dbias.data_ptr(), stream())
        else:
            ft.ft_launch_noalloc(plan, dA.data_ptr(), dB.data_ptr(), buf.data_ptr() + 4 * GUARD, dbias.data_ptr(), stream())
        torch.cuda.synchronize()
        outs.append(out_view(buf, M * N))
    assert np.array_equal(outs[0], outs[1])
    with pytest.raises(ft.FtError) as e:                  # an operator with a bias wants one
        ft.ft_launch_noalloc(plan, dA.data_ptr(), dB.data_ptr(), dbias.data_ptr(), 0, stream())
    assert e.value.status == ft.FT_ERR_INVALID_ARG


def test_noalloc_refuses_what_the_static_workspace_cannot_hold():
    N, K, M = 4096, 4096, 2048
    op = matmul_op(N, K, ft.FT_BF16)
    s = ft.ft_ukernels_derive(op)
    ids = [i for i in range(ft.ft_ukset_size(s))
           if (lambda u: (u.tm, u.tn, u.gk) == (128, 128, 1))(ft.ft_ukset_get(s, i))]
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED | ft.FT_PLAN_HOST_ONLY,
                             ft.ft_forced_program(k1=ids[0], count1=M // 128, k_parts=8))
    st = ft.ft_plan_stats_get(plan)
    assert st.k_parts == 8 and st.workspace_bytes > (32 << 20)
    x = torch.zeros(16, dtype=torch.int16, device="cuda")
    with pytest.raises(ft.FtError) as e:
        ft.ft_launch_noalloc(plan, x.data_ptr(), x.data_ptr(), x.data_ptr(), 0, stream())
    assert e.value.status == ft.FT_ERR_UNSUPPORTED
    # grouped plans read their tables: not for this entry point
    bop = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512))
    gp = ft.ft_plan_create_grouped(bop, ft.ft_ukernels_derive(bop), [ft.ft_shape(batch=2, m=40, n=40)])
    with pytest.raises(ft.FtError) as e:
        ft.ft_launch_noalloc(gp, x.data_ptr(), x.data_ptr(), x.data_ptr(), 0, stream())
    assert e.value.status == ft.FT_ERR_UNSUPPORTED
