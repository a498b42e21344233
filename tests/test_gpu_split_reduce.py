"""GPU parity of the reduce-axis split over workgroups (occupancy rescue for shapes with few
tiles): k_parts workgroups per tile leave fp32 partials in the plan's workspace and the last to
arrive sums them in part order.  Same oracle, same tolerance as the unsplit path; on top of that
two launches of one plan must agree bit for bit (fixed summation order, counters back at zero)."""
import numpy as np
import pytest

import paper_2407_21418_amd as ft
import synth_inputs as si
from oracle import contraction as oc
from oracle import planner as P

import torch

from gpu_util import GUARD, alloc_out, check, check_epilogue, dev_bits, matmul_op, out_view, run, run_epilogue, stream

pytestmark = pytest.mark.gpu


def family():
    op = P.Op(P.OP_BMM, P.F16, k_range=(0, 4096), m_range=(0, 8192), n_range=(0, 8192))
    return [(u.tm, u.tn, u.wm, u.wn, u.gm, u.gn, u.gk) for u in P.derive_ukernels(op)]


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
@pytest.mark.parametrize("body", family(), ids=lambda b: "t%dx%d_w%dx%d_gk%d" % (b[0], b[1], b[2], b[3], b[6]))
def test_every_fast_body_split_in_three(body, dtype):
    """2 x 2 ragged tiles x batch 2, K = 11 k-tiles + a tail of 8: three parts of 4, 4 and 4 k-tiles
    (the last holding the zero-filled tail)."""
    tm, tn, wm, wn = body[:4]
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=dtype, m_lo=0, m_hi=8192, n_lo=0, n_hi=8192,
                                         k_lo=0, k_hi=4096))
    s = ft.ft_ukernels_derive(op)
    ids = [i for i in range(ft.ft_ukset_size(s))
           if (lambda u: (u.tm, u.tn, u.wm, u.wn) == (tm, tn, wm, wn))(ft.ft_ukset_get(s, i))]
    assert len(ids) == 1
    M, N, K, nb = 2 * tm - 5, 2 * tn - 8, 712, 2
    g = np.random.default_rng(tm * 11 + tn * 5 + wm + dtype)
    A = si.normal_bits(g, (nb, M, K), 1.0, dtype)
    B = si.normal_bits(g, (nb, K, N), 1.0, dtype)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=nb, m=M, n=N, k=K), ft.FT_PLAN_FORCED,
                             ft.ft_forced_program(k1=ids[0], count1=2, k_parts=3))
    st = ft.ft_plan_stats_get(plan)
    if wm * wn // 64 > P.KPART_ACC_MAX:           # no registers left for the exchange: never split
        assert (st.n_tiles, st.k_parts, st.k_part_tiles, st.workspace_bytes) == (nb * 4, 1, 12, 0)
    else:
        assert (st.n_tiles, st.k_parts, st.k_part_tiles) == (nb * 4, 3, 4)
        assert st.workspace_bytes == st.n_tiles * 3 * tm * tn * 4
    ref, refabs = oc.bmm(A, B, dtype, want_abs=True)
    first = run(plan, A, B, nb * M * N)
    check(first, ref, refabs, f"body {body} dtype {dtype} split 3")
    again = run(plan, A, B, nb * M * N)
    assert np.array_equal(first, again), "second launch of the same plan differs"


@pytest.mark.parametrize("parts,K", [(2, 768), (4, 3072), (5, 1000), (8, 3072), (64, 200)])
def test_mixed_program_bias_and_16bit_output(parts, K):
    """Two uKernel shapes in one launch (a standard grid and a split-k wave grid), every tile split
    over `parts` workgroups, with the fused bias and a 16-bit C.  parts = 64 exceeds the k-tiles of
    K = 200 and is cut down to one k-tile per part."""
    M, N = 1232, 768
    g = np.random.default_rng(parts * 1000 + K)
    A = si.normal_bits(g, (M, K), 1.0, ft.FT_F16)
    B = si.normal_bits(g, (K, N), 0.05, ft.FT_F16)
    bias = g.standard_normal(N).astype(np.float32)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=N, k=K, m_lo=0, m_hi=8192,
                                         out_dtype=ft.FT_OUT_SAME, epilogue=ft.FT_EPI_BIAS))
    s = ft.ft_ukernels_derive(op)
    infos = [ft.ft_ukset_get(s, i) for i in range(ft.ft_ukset_size(s))]
    big = next(u for u in infos if u.tm == 128 and u.gk == 1)
    small = next(u for u in infos if u.tm == 16)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED,
                             ft.ft_forced_program(k1=big.id, count1=9, k2=small.id, count2=5, k_parts=parts))
    st = ft.ft_plan_stats_get(plan)
    nk = -(-K // 64)
    per = -(-nk // min(parts, nk))
    assert (st.k_parts, st.k_part_tiles) == (-(-nk // per), per)
    assert st.workspace_bytes == st.n_tiles * st.k_parts * max(big.tm * big.tn, small.tm * small.tn) * 4
    ref, refabs = oc.matmul(A, B, si.F16, want_abs=True)
    ref = ref + bias[None, :]
    got = run_epilogue(plan, A, B, M * N, bias=bias, out16=ft.FT_F16)
    check_epilogue(got, ref, refabs, bias[None, :], ft.FT_F16, f"mixed split {parts} K {K}")
    again = run_epilogue(plan, A, B, M * N, bias=bias, out16=ft.FT_F16)
    assert np.array_equal(got, again)


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
def test_permutation_matrix_stays_bit_exact_when_split(dtype):
    """A = permutation matrix: each output is one product plus zeros from the other parts."""
    g = np.random.default_rng(14)
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
                                 ft.ft_forced_program(k1=i, count1=n // u.tm, k_parts=3))
        assert ft.ft_plan_stats_get(plan).k_parts == (3 if u.acc_regs <= P.KPART_ACC_MAX and u.gk != 2 and u.gm * u.gn != 8 else 1)
        got = run(plan, A, B, n * N).reshape(n, N)
        assert np.array_equal(got, want), (u.tm, u.tn, u.wm, u.wn)


@pytest.mark.parametrize("M,N,K", [(80, 768, 3072), (272, 768, 3072), (528, 768, 3072), (1232, 768, 3072), (16, 4096, 4096),
                                   (1600, 768, 3072), (400, 1536, 4096), (200, 5120, 2048)])
def test_planner_chosen_split_matches_oracle(M, N, K):
    """Patchwork plans of shapes with few tiles: the library's choice of k_parts is the oracle's,
    and the result is within tolerance."""
    dtype = ft.FT_F16
    g = np.random.default_rng(M + N + K)
    A = si.normal_bits(g, (M, K), 1.0, dtype)
    B = si.normal_bits(g, (K, N), 0.02, dtype)
    op = matmul_op(N, K, dtype)
    s = ft.ft_ukernels_derive(op)
    oop = P.Op(P.OP_MATMUL, P.F16, n=N, k=K, m_range=(0, 8192))
    want = P.plan(oop, P.derive_ukernels(oop), (1, M, N, K))
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
    st = ft.ft_plan_stats_get(plan)
    assert (st.k_parts, st.k_part_tiles) == (want.k_parts, want.k_part_tiles)
    assert ft.ft_plan_descriptors(plan) == b"".join(d.pack() for d in want.descs)
    ref, refabs = oc.matmul(A, B, si.F16, want_abs=True)
    check(run(plan, A, B, M * N), ref, refabs, f"{M}x{N}x{K} k_parts {st.k_parts}")


def test_shapes_without_the_vector_path_are_never_split():
    """Odd row lengths take the general bodies, which walk the whole reduce axis themselves: a forced
    split is cut down to one part when the plan is made, so the statistics describe what runs."""
    M, N, K = 100, 203, 331
    g = np.random.default_rng(5)
    A = si.normal_bits(g, (M, K), 1.0, ft.FT_F16)
    B = si.normal_bits(g, (K, N), 1.0, ft.FT_F16)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=N, k=K, m_lo=0, m_hi=4096))
    s = ft.ft_ukernels_derive(op)
    Hp = -(-M // 16) * 16
    ids = [i for i in range(ft.ft_ukset_size(s)) if Hp % ft.ft_ukset_get(s, i).tm == 0]
    u = ft.ft_ukset_get(s, ids[0])
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED,
                             ft.ft_forced_program(k1=ids[0], count1=Hp // u.tm, k_parts=3))
    st = ft.ft_plan_stats_get(plan)
    assert (st.k_parts, st.workspace_bytes) == (1, 0)
    ref, refabs = oc.matmul(A, B, si.F16, want_abs=True)
    check(run(plan, A, B, M * N), ref, refabs, "general path")


def test_split_plan_with_misaligned_pointers():
    """A plan that splits the reduce axis, launched on operands that are not 16-byte aligned (the
    LDS-DMA copies take any 2-byte aligned source): the result is still right."""
    M, N, K = 528, 768, 3072
    p = si.config1_problem(M, N, K)
    op = matmul_op(N, K, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
    assert ft.ft_plan_stats_get(plan).k_parts > 1
    ref, refabs = oc.matmul(p["A"], p["B"], si.F16, want_abs=True)
    A = torch.zeros(M * K + 8, dtype=torch.int16, device="cuda")
    A[4:4 + M * K] = dev_bits(p["A"]).reshape(-1)            # 8 bytes past a 16-byte boundary
    B = dev_bits(p["B"])
    buf = alloc_out(M * N)
    ft.ft_launch(plan, A.data_ptr() + 8, B.data_ptr(), buf.data_ptr() + 4 * GUARD, stream())
    torch.cuda.synchronize()
    check(out_view(buf, M * N), ref, refabs, "misaligned A")


def test_split_plan_through_the_timing_entry_points_and_a_graph():
    """Back-to-back launches of one split plan on rotating buffers, eagerly and as a replayed HIP
    graph (the arrival counters are reset by the kernel itself, no memset node): every buffer set
    holds the same bits as a single eager launch."""
    M, N, K = 528, 768, 3072
    p = si.config1_problem(M, N, K)
    op = matmul_op(N, K, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
    assert ft.ft_plan_stats_get(plan).k_parts > 1
    ref, refabs = oc.matmul(p["A"], p["B"], si.F16, want_abs=True)
    single = run(plan, p["A"], p["B"], M * N)
    check(single, ref, refabs, "single launch")
    side = torch.cuda.Stream()
    n_sets = 3
    A = [dev_bits(p["A"]) for _ in range(n_sets)]
    B = [dev_bits(p["B"]) for _ in range(n_sets)]
    for use_graph in (False, True, True):
        bufs = [alloc_out(M * N) for _ in range(n_sets)]
        torch.cuda.synchronize()
        ms = ft.ft_launch_timed(plan, [t.data_ptr() for t in A], [t.data_ptr() for t in B],
                                [b.data_ptr() + 4 * GUARD for b in bufs], side.cuda_stream, 7, graph=use_graph)
        torch.cuda.synchronize()
        assert 0.0 < ms < 10.0
        for b in bufs:
            assert np.array_equal(out_view(b, M * N), single), f"timed launches, graph={use_graph}"
        assert np.array_equal(run(plan, p["A"], p["B"], M * N), single), "eager launch between timed runs"


def test_relaunch_with_other_inputs_sees_no_stale_partials():
    """The workspace slabs are reused by every launch of a plan: launches with different operands,
    back to back on one stream without host synchronisation in between, must each give their own
    result (a partial tile left over from the previous launch, in any cache, would show)."""
    M, N, K = 528, 768, 3072
    op = matmul_op(N, K, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
    assert ft.ft_plan_stats_get(plan).k_parts > 1
    g = np.random.default_rng(77)
    sets = []
    for i in range(3):
        A = si.normal_bits(g, (M, K), 1.0 + i, ft.FT_F16)
        B = si.normal_bits(g, (K, N), 0.02 * (i + 1), ft.FT_F16)
        sets.append((A, B, dev_bits(A), dev_bits(B), alloc_out(M * N)))
    stream = torch.cuda.current_stream().cuda_stream
    for rep in range(4):                       # 12 launches, operands changing every launch
        for (_, _, dA, dB, buf) in sets:
            ft.ft_launch(plan, dA.data_ptr(), dB.data_ptr(), buf.data_ptr() + 4 * GUARD, stream)
    torch.cuda.synchronize()
    for i, (A, B, _, _, buf) in enumerate(sets):
        ref, refabs = oc.matmul(A, B, si.F16, want_abs=True)
        check(out_view(buf, M * N), ref, refabs, f"operand set {i} after interleaved launches")


@pytest.mark.parametrize("M,N,K,forced", [(64, 64, 65536, 0), (40, 128, 16384, 0), (256, 256, 4096, 64), (100, 72, 4104, 64)])
def test_extreme_reduce_extents_and_part_counts(M, N, K, forced):
    """Very long reduce axes on one or two tiles (the planner splits as far as its rules allow) and
    the largest part count a caller may force: 64 parts of a single k-tile each (65 k-tiles with a
    tail of 8 in the last case, so the last part holds the zero-filled tail alone)."""
    g = np.random.default_rng(M + K)
    A = si.normal_bits(g, (M, K), 1.0, ft.FT_BF16)
    B = si.normal_bits(g, (K, N), 0.05, ft.FT_BF16)
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_BF16, n=N, k=K, m_lo=0, m_hi=4096))
    s = ft.ft_ukernels_derive(op)
    if forced:
        infos = [ft.ft_ukset_get(s, i) for i in range(ft.ft_ukset_size(s))]
        Hp = -(-M // 16) * 16
        u = next(u for u in infos if Hp % u.tm == 0 and u.acc_regs <= P.KPART_ACC_MAX)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED,
                                 ft.ft_forced_program(k1=u.id, count1=Hp // u.tm, k_parts=forced))
        nk = -(-K // 64)
        per = -(-nk // min(forced, nk))
        assert ft.ft_plan_stats_get(plan).k_parts == -(-nk // per)
    else:
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
        assert ft.ft_plan_stats_get(plan).k_parts > 1
    ref, refabs = oc.matmul(A, B, si.BF16, want_abs=True)
    got = run(plan, A, B, M * N)
    check(got, ref, refabs, f"{M}x{N}x{K} forced {forced}")
    assert np.array_equal(run(plan, A, B, M * N), got)


@pytest.mark.parametrize("M,N,K", [(1600, 768, 3072), (1232, 3072, 768), (80, 768, 768), (16, 4096, 4096)])
def test_table_order_gives_the_same_bits(M, N, K):
    """FT_PLAN_TABLE_ORDER: workgroups read their descriptors (dealt to the XCDs in chunks) instead
    of deriving them from the tile grids; with and without a reduce-axis split the output must be
    bit-identical to the default order's (same tiles, same summation order)."""
    g = np.random.default_rng(M * 3 + N + K)
    A = si.normal_bits(g, (M, K), 1.0, ft.FT_F16)
    B = si.normal_bits(g, (K, N), 0.02, ft.FT_F16)
    op = matmul_op(N, K, ft.FT_F16)
    s = ft.ft_ukernels_derive(op)
    default = ft.ft_plan_create(op, s, ft.ft_shape(m=M))
    table = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_TABLE_ORDER)
    sd, stt = ft.ft_plan_stats_get(default), ft.ft_plan_stats_get(table)
    assert (sd.table_order, stt.table_order) == (0, 1) and sd.k_parts == stt.k_parts
    assert ft.ft_plan_descriptors(default) == ft.ft_plan_descriptors(table)
    order = ft.ft_plan_launch_order(table)
    assert sorted(t for t in order if t != 0xFFFFFFFF) == list(range(stt.n_tiles))
    ref, refabs = oc.matmul(A, B, si.F16, want_abs=True)
    got = run(default, A, B, M * N)
    check(got, ref, refabs, f"{M}x{N}x{K}")
    assert np.array_equal(run(table, A, B, M * N), got)
