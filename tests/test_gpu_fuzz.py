"""Seeded random shapes through the planner's own plans: Matmul with any M, N, K (aligned to 8
elements or not), both input types, optional bias / 16-bit output, optional forced reduce-axis split
and table order.  Same oracle and tolerance as the other parity tests; the cases are fixed by the
seed, so a failure names its case.  FT_FUZZ_SEED / FT_FUZZ_CASES in the environment draw another or a
longer list (a soak run; the defaults are what the suite runs)."""
import os

import numpy as np
import pytest

import paper_2407_21418_amd as ft
import synth_inputs as si
from oracle import contraction as oc

from gpu_util import check, check_epilogue, run, run_epilogue

pytestmark = pytest.mark.gpu


FUZZ_SEED = int(os.environ.get("FT_FUZZ_SEED", "20240721"))
FUZZ_CASES = int(os.environ.get("FT_FUZZ_CASES", "0"))


def _cases(n=72):
    n = FUZZ_CASES or n
    g = np.random.default_rng(FUZZ_SEED)
    out = []
    for i in range(n):
        aligned = bool(g.integers(0, 2))
        q = 8 if aligned else 1
        M = int(g.integers(1, 700))
        N = int(g.integers(1, 130)) * q if aligned else int(g.integers(1, 1040))
        K = int(g.integers(1, 260)) * q if aligned else int(g.integers(1, 2080))
        dtype = int(g.integers(0, 2))
        epi = int(g.integers(0, 4))            # 0 plain, 1 bias, 2 16-bit C, 3 both
        parts = int(g.choice([0, 0, 2, 3, 5])) if aligned else 0
        table = bool(g.integers(0, 4) == 0)
        out.append((i, M, N, K, dtype, epi, parts, table))
    return out


@pytest.mark.parametrize("case", _cases(), ids=lambda c: "c%d_%dx%dx%d_dt%d_e%d_p%d_t%d" % (c[0], c[1], c[2], c[3], c[4], c[5], c[6], int(c[7])))
def test_random_matmul(case):
    i, M, N, K, dtype, epi, parts, table = case
    g = np.random.default_rng([1000 + i, FUZZ_SEED])
    A = si.normal_bits(g, (M, K), 1.0, dtype)
    B = si.normal_bits(g, (K, N), 0.1, dtype)
    bias = g.standard_normal(N).astype(np.float32) if epi & 1 else None
    out16 = dtype if epi & 2 else None
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dtype, n=N, k=K, m_lo=0, m_hi=1024,
                                         out_dtype=ft.FT_OUT_SAME if epi & 2 else ft.FT_OUT_F32,
                                         epilogue=ft.FT_EPI_BIAS if epi & 1 else ft.FT_EPI_NONE))
    s = ft.ft_ukernels_derive(op)
    flags = ft.FT_PLAN_TABLE_ORDER if table else 0
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), flags)
    st = ft.ft_plan_stats_get(plan)
    covered_rows = sum(st.count_tau[j] * ft.ft_ukset_get(s, st.ukernel_id[j]).tm for j in range(st.n_ukernels))
    # (a program that pads the rows beyond the 16-row granule -- the fallback when no uKernel
    # extent fits -- cannot be named through ft_forced_program, which takes exact covers only)
    if parts and covered_rows == -(-M // 16) * 16:
        # the planner's program again, its tiles split over `parts` workgroups
        forced = ft.ft_forced_program(k1=st.ukernel_id[0], count1=st.count_tau[0],
                                      k2=st.ukernel_id[1] if st.n_ukernels == 2 else 0,
                                      count2=st.count_tau[1] if st.n_ukernels == 2 else 0, k_parts=parts)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED | flags, forced)
    ref, refabs = oc.matmul(A, B, dtype, want_abs=True)
    if epi:
        if bias is not None:
            ref = ref + bias[None, :]
        got = run_epilogue(plan, A, B, M * N, bias=bias, out16=out16)
        check_epilogue(got, ref, refabs, bias[None, :] if bias is not None else None, out16, str(case))
    else:
        check(run(plan, A, B, M * N), ref, refabs, str(case))


def _bmm_cases(n=48):
    n = FUZZ_CASES or n
    g = np.random.default_rng(99173 if FUZZ_SEED == 20240721 else FUZZ_SEED + 1)
    out = []
    for i in range(n):
        aligned = bool(g.integers(0, 2))
        q = 8 if aligned else 1
        nb = int(g.integers(1, 7))
        M = int(g.integers(1, 400))
        N = int(g.integers(1, 50)) * q if aligned else int(g.integers(1, 400))
        K = int(g.integers(1, 40)) * q if aligned else int(g.integers(1, 300))
        dtype = int(g.integers(0, 2))
        strips = bool(g.integers(0, 2))
        parts = int(g.choice([0, 0, 2, 3])) if aligned and not strips else 0
        static = int(g.integers(0, 3))         # 0: every extent dynamic, 1: K static (QK^T-like), 2: N static (PV-like)
        if static == 1:
            K = int(g.choice([16, 64, 128]))
        elif static == 2:
            N = int(g.choice([16, 64, 128]))
        out.append((i, nb, M, N, K, dtype, strips, parts, static))
    return out


@pytest.mark.parametrize("case", _bmm_cases(), ids=lambda c: "b%d_%dx%dx%dx%d_dt%d_s%d_p%d_st%d" % (c[0], c[1], c[2], c[3], c[4], c[5], int(c[6]), c[7], c[8]))
def test_random_batched_matmul_all_axes_dynamic(case):
    """Batched Matmul with every extent dynamic, or with a static reduce axis (QK^T-like: two dynamic
    space axes, where the second-axis strips can apply; they are switched on for half of the cases) or
    a static N (PV-like: dynamic reduce axis)."""
    i, nb, M, N, K, dtype, strips, parts, static = case
    g = np.random.default_rng([5000 + i, FUZZ_SEED])
    A = si.normal_bits(g, (nb, M, K), 1.0, dtype)
    B = si.normal_bits(g, (nb, K, N), 0.2, dtype)
    ranges = dict(m_lo=0, m_hi=512, n_lo=0, n_hi=512, k_lo=0, k_hi=512)
    if static == 1:
        ranges.update(k=K, k_lo=0, k_hi=0)
    elif static == 2:
        ranges.update(n=N, n_lo=0, n_hi=0)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=dtype, batch_hi=768, **ranges))
    t = ft.ft_tuning_default()
    t.second_axis_strips = 1 if strips else 0
    s = ft.ft_ukernels_derive(op, None, t)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=nb, m=M, n=N, k=K))
    st = ft.ft_plan_stats_get(plan)
    tau_ext = lambda u: u.tm if st.tau == 0 else u.tn
    covered = sum(st.count_tau[j] * tau_ext(ft.ft_ukset_get(s, st.ukernel_id[j])) for j in range(st.n_ukernels))
    if parts and covered == -(-(M if st.tau == 0 else N) // 16) * 16:
        forced = ft.ft_forced_program(k1=st.ukernel_id[0], count1=st.count_tau[0],
                                      k2=st.ukernel_id[1] if st.n_ukernels == 2 else 0,
                                      count2=st.count_tau[1] if st.n_ukernels == 2 else 0, k_parts=parts)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=nb, m=M, n=N, k=K), ft.FT_PLAN_FORCED, forced)
    ref, refabs = oc.bmm(A, B, dtype, want_abs=True)
    check(run(plan, A, B, nb * M * N), ref, refabs, str(case))


def _conv_cases(n=32):
    n = FUZZ_CASES or n
    g = np.random.default_rng(4711 if FUZZ_SEED == 20240721 else FUZZ_SEED + 2)
    out = []
    for i in range(n):
        R = int(g.choice([1, 3, 5]))
        S = int(g.choice([1, 3, 5]))
        stride = int(g.integers(1, 4))
        pad = int(g.integers(0, 3))
        nimg = int(g.integers(1, 4))
        H = int(g.integers(max(1, R - 2 * pad), 30))
        W = int(g.integers(max(1, S - 2 * pad), 30))
        Cin = int(g.choice([3, 8, 12, 16, 64, 72, 128]))
        Cout = int(g.integers(1, 200))
        dtype = int(g.integers(0, 2))
        epi = int(g.integers(0, 4))
        out.append((i, nimg, H, W, Cin, Cout, R, S, stride, pad, dtype, epi))
    return out


@pytest.mark.parametrize("case", _conv_cases(), ids=lambda c: "v%d_n%d_%dx%d_c%d_k%d_f%dx%d_s%d_p%d_dt%d_e%d" % c)
def test_random_conv2d(case):
    """Implicit-GEMM convolution with random geometry: filter 1/3/5, stride 1-3, padding 0-2, channel
    counts that take the LDS-DMA gather (multiples of 64), the vector gather (multiples of 8) and the
    element-wise gather; any c_out; optional bias / 16-bit output."""
    i, nimg, H, W, Cin, Cout, R, S, stride, pad, dtype, epi = case
    g = np.random.default_rng([9000 + i, FUZZ_SEED])
    X = si.normal_bits(g, (nimg, H, W, Cin), 1.0, dtype)
    Wt = si.normal_bits(g, (R, S, Cin, Cout), 0.2, dtype)
    bias = g.standard_normal(Cout).astype(np.float32) if epi & 1 else None
    out16 = dtype if epi & 2 else None
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_CONV2D, dtype=dtype, c_in=Cin, c_out=Cout, r=R, s=S, stride=stride,
                                         pad=pad, m_lo=0, m_hi=1 << 20,
                                         out_dtype=ft.FT_OUT_SAME if epi & 2 else ft.FT_OUT_F32,
                                         epilogue=ft.FT_EPI_BIAS if epi & 1 else ft.FT_EPI_NONE))
    plan = ft.ft_plan_create(op, ft.ft_ukernels_derive(op), ft.ft_shape(img_n=nimg, img_h=H, img_w=W))
    ref, refabs = oc.conv2d_nhwc(X, Wt, dtype, stride=stride, pad=pad, want_abs=True)
    ref, refabs = ref.reshape(-1, Cout), refabs.reshape(-1, Cout)
    if epi:
        if bias is not None:
            ref = ref + bias[None, :]
        got = run_epilogue(plan, X, Wt, ref.size, bias=bias, out16=out16)
        check_epilogue(got, ref, refabs, bias[None, :] if bias is not None else None, out16, str(case))
    else:
        check(run(plan, X, Wt, ref.size), ref, refabs, str(case))


def _grouped_cases(n=24):
    n = FUZZ_CASES or n
    g = np.random.default_rng(8086 if FUZZ_SEED == 20240721 else FUZZ_SEED + 3)
    out = []
    for i in range(n):
        static = int(g.integers(0, 3))         # 0: every extent dynamic, 1: K static, 2: N static
        fixed = int(g.choice([16, 64, 128]))
        all_aligned = bool(g.integers(0, 3) == 0)   # every group aligned: the launch takes the LDS-DMA bodies
        dims = []
        for _ in range(int(g.integers(1, 21))):
            b = int(g.integers(0, 5))
            M, N, K = (int(g.integers(0 if j < 2 else 1, 301)) for j in range(3))
            if all_aligned or bool(g.integers(0, 3) == 0):    # else some aligned groups among the odd ones
                M, N, K = M // 8 * 8, N // 8 * 8, max(8, K // 8 * 8)
            if static == 1:
                K = fixed
            elif static == 2:
                N = fixed
            dims.append((b, M, N, K))
        out.append((i, static, int(g.integers(0, 2)), int(g.integers(0, 2)), tuple(dims)))
    return out


@pytest.mark.parametrize("case", _grouped_cases(), ids=lambda c: "g%d_st%d_dt%d_base%d_n%d" % (c[0], c[1], c[2], c[3], len(c[4])))
def test_random_grouped_launch(case):
    """Grouped launches over 1-20 random groups (empty ones included): every group against the
    oracle on its slice of the packed buffers; nothing outside C is written."""
    import torch
    from gpu_util import GUARD, alloc_out, dev_bits, out_view, stream
    i, static, dtype, baseline, dims = case
    ranges = dict(m_lo=0, m_hi=512, n_lo=0, n_hi=512, k_lo=0, k_hi=512)
    if static == 1:
        ranges.update(k=dims[0][3], k_lo=0, k_hi=0)
    elif static == 2:
        ranges.update(n=dims[0][2], n_lo=0, n_hi=0)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=dtype, batch_hi=768, **ranges))
    groups = [ft.ft_shape(batch=b, m=M, n=N, k=K) for b, M, N, K in dims]
    plan = ft.ft_plan_create_grouped(op, ft.ft_ukernels_derive(op), groups,
                                     ft.FT_PLAN_PAD_BASELINE if baseline else ft.FT_PLAN_PATCHWORK)
    na, nb, nc = ft.ft_plan_group_layout(plan, len(groups))
    g = np.random.default_rng([7000 + i, FUZZ_SEED])
    A = si.normal_bits(g, (max(na, 1),), 1.0, dtype)
    B = si.normal_bits(g, (max(nb, 1),), 0.3, dtype)
    buf = alloc_out(nc)
    dA, dB = dev_bits(A), dev_bits(B)
    ft.ft_launch(plan, dA.data_ptr(), dB.data_ptr(), buf.data_ptr() + 4 * GUARD, stream())
    torch.cuda.synchronize()
    C = out_view(buf, nc)
    for gi, (b, M, N, K) in enumerate(dims):
        oa, ob, oc_ = ft.ft_plan_group_layout(plan, gi)
        if b * M * N == 0:
            continue
        ref, refabs = oc.bmm(A[oa:oa + b * M * K].reshape(b, M, K), B[ob:ob + b * K * N].reshape(b, K, N), dtype, want_abs=True)
        check(C[oc_:oc_ + b * M * N], ref, refabs, f"{case[:4]} group {gi} {b}x{M}x{N}x{K}")
