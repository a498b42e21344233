"""GPU parity of exactly what the benchmarks time: every GEMM of the BERT-shaped sweep with the
operator registered as bench.py registers it (M in 1..8192, hardware model queried from the device),
in the patchwork plan and in the pad-to-library plan (plan bytes == planner oracle, every output
element against the contraction oracle), and the large members of the other configurations
(convolution resolutions 56..224, LLM token counts at both widths) on sampled rows / pixels.
Tolerance as everywhere: max relative error 2e-3 of fp32-accumulated 16-bit products."""
import numpy as np
import pytest
import torch

import paper_2407_21418_amd as ft
import synth_inputs as si
from oracle import contraction as oc
from oracle import planner as P

from gpu_util import check, dev_bits, run, stream

pytestmark = pytest.mark.gpu

_sets = {}


def bench_operator(N, K):
    """(op, uKernel set, oracle op, oracle set, oracle hw) of one dense layer, as bench.py makes them."""
    if (N, K) not in _sets:
        hw = ft.ft_hw_query(0)
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=N, k=K, m_lo=1, m_hi=8192))
        uks = ft.ft_ukernels_derive(op, hw, None)
        ohw = {k: v for k, v in hw.as_dict().items() if k != "struct_size"}
        oop = P.Op(P.OP_MATMUL, P.F16, n=N, k=K, m_range=(1, 8192))
        _sets[(N, K)] = (op, uks, oop, P.derive_ukernels(oop, hw=ohw), ohw)
    return _sets[(N, K)]


@pytest.mark.parametrize("M,N,K", si.config1_shapes(), ids=lambda v: str(v))
def test_every_benched_gemm_in_both_plans(M, N, K):
    op, uks, oop, ouk, ohw = bench_operator(N, K)
    p = si.config1_problem(M, N, K)
    ref, refabs = oc.matmul(p["A"], p["B"], si.F16, want_abs=True)
    for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
        plan = ft.ft_plan_create(op, uks, ft.ft_shape(m=M), mode)
        want = b"".join(d.pack() for d in P.plan(oop, ouk, (1, M, N, K), mode, hw=ohw).descs)
        assert ft.ft_plan_descriptors(plan) == want, f"plan bytes differ from the oracle: {M}x{N}x{K} mode {mode}"
        check(run(plan, p["A"], p["B"], M * N), ref, refabs, f"benched {M}x{N}x{K} mode {mode}")


def test_benched_uKernel_sets_match_the_oracle():
    for (K, N) in si.BERT_LAYERS:
        _, uks, _, ouk, _ = bench_operator(N, K)
        got = [ft.ft_ukset_get(uks, i) for i in range(ft.ft_ukset_size(uks))]
        assert [(u.tm, u.tn, u.tk, u.wm, u.wn, u.gm, u.gn, u.gk, u.stages, u.cmr_q20, u.cmr_shared_q20) for u in got] == \
               [(u.tm, u.tn, u.tk, u.wm, u.wn, u.gm, u.gn, u.gk, u.stages, u.cmr_q, u.cmr2_q) for u in ouk]


@pytest.mark.parametrize("res", [56, 91, 150, 224])
def test_conv_resolutions_sampled_pixels(res):
    """The configured convolution (8 x res x res x 64 -> 128, 3x3, stride 1, pad 1) in the default plan
    and the pad-to-library plan: image corners and edges, pixels around tile boundaries and random
    pixels against the oracle; every output finite."""
    batch = si.CONV_BATCH
    p = si.config4_problem(res, batch=batch)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_CONV2D, dtype=ft.FT_F16, c_in=64, c_out=128, r=3, s=3,
                                         stride=1, pad=1, m_lo=0, m_hi=1 << 22))
    s = ft.ft_ukernels_derive(op, ft.ft_hw_query(0), None)
    M = batch * res * res
    X, Wt = dev_bits(p["X"]), dev_bits(p["Wt"])
    g = np.random.default_rng(600 + res)
    special = [0, res - 1, res, res * res - 1, res * res, M - 1, M - res, 15, 16, 17, 127, 128, 129, 255, 256, 257,
               511, 512, 513, (3 * res + 5) * res, (3 * res + 5) * res + res - 1]
    pix = np.unique(np.concatenate([g.integers(0, M, 200), special])).astype(np.int64)
    ref, refabs = oc.conv2d_nhwc(p["X"], p["Wt"], si.F16, pixels=pix, want_abs=True)
    for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
        plan = ft.ft_plan_create(op, s, ft.ft_shape(img_n=batch, img_h=res, img_w=res), mode)
        Y = torch.full((M, 128), float("nan"), dtype=torch.float32, device="cuda")
        ft.ft_launch(plan, X.data_ptr(), Wt.data_ptr(), Y.data_ptr(), stream())
        torch.cuda.synchronize()
        assert bool(torch.isfinite(Y).all())
        got = Y[torch.from_numpy(pix).cuda()].cpu().numpy().astype(np.float64)
        check(got, ref, refabs, f"conv 8x{res}x{res} mode {mode}")
        del Y


@pytest.mark.parametrize("M,N", [(1, 11008), (300, 11008), (2048, 11008), (8192, 4096), (1024, 4096)])
def test_llm_token_counts_sampled_rows(M, N):
    """bf16 GEMMs of the token-count configuration at both widths, default plan: rows around tile
    boundaries plus random rows against the oracle, whole matrix for the small ones."""
    p = si.config3_problem(M, N)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_BF16, n=N, k=si.LLM_K, m_lo=1, m_hi=8192))
    s = ft.ft_ukernels_derive(op, ft.ft_hw_query(0), None)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
    A, B = dev_bits(p["A"]), dev_bits(p["B"])
    Cd = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ft.ft_launch(plan, A.data_ptr(), B.data_ptr(), Cd.data_ptr(), stream())
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Cd).all())
    g = np.random.default_rng(M + N)
    if M <= 300:
        rows = np.arange(M, dtype=np.int64)
    else:
        near = [r for b in (128, 256, 512, 1024) for r in (b - 1, b, b + 1) if r < M]
        rows = np.unique(np.concatenate([g.integers(0, M, 48), [0, 1, M - 2, M - 1], near])).astype(np.int64)
    ref, refabs = oc.matmul(p["A"], p["B"], si.BF16, rows=rows, want_abs=True)
    got = Cd[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    check(got, ref, refabs, f"llm {M}x{N}")


TWO_TEAM_FAMILY = [(wm, wn, gm, gn) for (wm, wn) in ((16, 16), (16, 32), (16, 64), (32, 32), (32, 64), (64, 32), (64, 64))
                   for (gm, gn) in ((1, 4), (2, 2), (4, 1)) if (gm * wm + gn * wn) * 128 <= 40960]


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
@pytest.mark.parametrize("body", TWO_TEAM_FAMILY, ids=lambda b: "w%dx%d_g%dx%d" % b)
def test_every_two_team_body(body, dtype):
    """The eight-wave bodies (two teams of four waves on alternate k-tiles, partial sums added through
    LDS), each alone as a forced program: 2 x 4 tiles with ragged tails on both axes; reduce extents
    with an odd and an even number of k-tiles, a k tail, a single k-tile (team 1 idle) and K = 1."""
    wm, wn, gm, gn = body
    tm, tn = wm * gm, wn * gn
    tuning = ft.ft_tuning_default()
    tuning.two_team_bodies = 1
    for K in (200, 712, 512, 64, 1):
        N, M = 4 * tn, 2 * tm - 5
        # (a static reduce axis of fewer than four k-tiles gets no two-team uKernels: the short ones run
        # through an operator whose reduce axis is dynamic)
        kdesc = dict(k=K) if K >= 200 else dict(k_lo=0, k_hi=4096)
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dtype, n=N, m_lo=0, m_hi=1 << 16, **kdesc))
        s = ft.ft_ukernels_derive(op, None, tuning)
        ids = [i for i in range(ft.ft_ukset_size(s))
               if (lambda u: (u.tm, u.tn, u.wm, u.wn, u.gk) == (tm, tn, wm, wn, 2))(ft.ft_ukset_get(s, i))]
        assert len(ids) == 1, (body, K)
        g = np.random.default_rng(wm * 7 + wn + gm + K + dtype)
        A = si.normal_bits(g, (M, K), 1.0, dtype)
        B = si.normal_bits(g, (K, N), 1.0, dtype)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M, k=0 if K >= 200 else K), ft.FT_PLAN_FORCED,
                                 ft.ft_forced_program(k1=ids[0], count1=2))
        assert ft.ft_plan_stats_get(plan).n_tiles == 8
        ref, refabs = oc.matmul(A, B, dtype, want_abs=True)
        check(run(plan, A, B, M * N), ref, refabs, f"two-team body {body} K {K} dtype {dtype}")


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
@pytest.mark.parametrize("body", sorted(P.EIGHT_WAVE_FAMILY), ids=lambda b: "w%dx%d_g%dx%d" % b)
def test_every_eight_wave_grid_body(body, dtype):
    """The eight-wave grids (two waves per SIMD on the same k-tiles; tiles of 256 x 256, 128 x 256 and
    256 x 128), each alone as a forced program: 2 x 4 tiles with ragged tails, a k tail, one k-tile."""
    wm, wn, gm, gn = body
    tm, tn = wm * gm, wn * gn
    for K in (200, 712, 64):
        N, M = 4 * tn - 24, 2 * tm - 5
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dtype, n=N, k=K, m_lo=0, m_hi=1 << 16))
        s = ft.ft_ukernels_derive(op)
        ids = [i for i in range(ft.ft_ukset_size(s))
               if (lambda u: (u.tm, u.tn, u.wm, u.wn, u.gm, u.gn, u.gk) == (tm, tn, wm, wn, gm, gn, 1))(ft.ft_ukset_get(s, i))]
        if not ids:             # a static N that the tile does not divide after rounding to 16: use one it divides
            N = 4 * tn
            op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dtype, n=N, k=K, m_lo=0, m_hi=1 << 16))
            s = ft.ft_ukernels_derive(op)
            ids = [i for i in range(ft.ft_ukset_size(s))
                   if (lambda u: (u.tm, u.tn, u.wm, u.wn, u.gm, u.gn, u.gk) == (tm, tn, wm, wn, gm, gn, 1))(ft.ft_ukset_get(s, i))]
        assert len(ids) == 1, (body, K)
        g = np.random.default_rng(wm + wn + gm + K + dtype)
        A = si.normal_bits(g, (M, K), 1.0, dtype)
        B = si.normal_bits(g, (K, N), 1.0, dtype)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED, ft.ft_forced_program(k1=ids[0], count1=2))
        ref, refabs = oc.matmul(A, B, dtype, want_abs=True)
        check(run(plan, A, B, M * N), ref, refabs, f"eight-wave body {body} K {K} dtype {dtype}")
