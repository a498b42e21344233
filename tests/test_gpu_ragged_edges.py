"""GPU parity of the LDS-DMA bodies on operands whose rows end inside a 16-byte chunk or start at any
2-byte aligned address: K and / or N not multiples of 8, odd row pitches, operands at odd element
offsets inside buffers whose every other element is a NaN (whatever a body reads beyond a row's end
must not reach an output).  Both layouts of B, every four-wave standard body, batched P V of odd
lengths, grouped launches.  Same oracle and tolerance as the other parity tests."""
import numpy as np
import pytest
import torch

import paper_2407_21418_amd as ft
import synth_inputs as si
from oracle import contraction as oc
from oracle import planner as P

from gpu_util import GUARD, alloc_out, check, out_view, stream

pytestmark = pytest.mark.gpu

NAN16 = {ft.FT_F16: 0x7e00, ft.FT_BF16: 0x7fc0}
STANDARD_BODIES = [(wm, wn, gm, gn) for (wm, wn, _) in P.wave_tiles() for (gm, gn, gk) in P.WAVE_GRIDS
                   if gk == 1 and gm * gn == 4]


def poisoned(bits, dtype, offset):
    """The operand at element `offset` of a buffer that holds NaNs everywhere else; returns (buffer, pointer)."""
    flat = np.ascontiguousarray(bits).reshape(-1)
    buf = torch.full((flat.size + offset + 64,), NAN16[dtype], dtype=torch.int16, device="cuda")
    buf[offset:offset + flat.size] = torch.from_numpy(flat.view(np.int16)).cuda()
    return buf, buf.data_ptr() + 2 * offset


def run_poisoned(plan, A_bits, B_bits, n_out, dtype, off_a=3, off_b=5):
    keep_a, pa = poisoned(A_bits, dtype, off_a)
    keep_b, pb = poisoned(B_bits, dtype, off_b)
    buf = alloc_out(n_out)
    ft.ft_launch(plan, pa, pb, buf.data_ptr() + 4 * GUARD, stream())
    torch.cuda.synchronize()
    return out_view(buf, n_out)


@pytest.mark.parametrize("layout", [ft.FT_B_KN, ft.FT_B_NK], ids=["kn", "nk"])
@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
@pytest.mark.parametrize("body", STANDARD_BODIES, ids=lambda b: "w%dx%d_g%dx%d" % b)
def test_every_standard_body_on_ragged_rows(body, dtype, layout):
    """Each four-wave body alone as a forced program, 2 x 4 tiles with ragged tails on M and an odd N;
    reduce extents that end inside a chunk: several k-tiles, less than one k-tile, one chunk and a bit."""
    wm, wn, gm, gn = body
    tm, tn = wm * gm, wn * gn
    for K in (203, 71, 9):
        N, M = 4 * tn - 3, 2 * tm - 5
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dtype, n=N, k=K, m_lo=0, m_hi=1 << 16, b_layout=layout))
        s = ft.ft_ukernels_derive(op)
        infos = [ft.ft_ukset_get(s, i) for i in range(ft.ft_ukset_size(s))]
        ids = [u.id for u in infos if (u.tm, u.tn, u.wm, u.wn, u.gm, u.gn, u.gk) == (tm, tn, wm, wn, gm, gn, 1)]
        if not ids:
            continue            # the workload filters of this operator dropped the shape
        g = np.random.default_rng(wm * 3 + wn + gm + K + dtype + layout)
        A = si.normal_bits(g, (M, K), 1.0, dtype)
        B = si.normal_bits(g, (K, N), 1.0, dtype)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED, ft.ft_forced_program(k1=ids[0], count1=2))
        ref, refabs = oc.matmul(A, B, dtype, want_abs=True)
        Bm = B if layout == ft.FT_B_KN else np.ascontiguousarray(B.T)
        check(run_poisoned(plan, A, Bm, M * N, dtype), ref, refabs, f"ragged body {body} K {K} dtype {dtype} layout {layout}")


SPLIT_K_TILES = [(16, 16), (16, 32), (16, 64), (32, 32), (32, 64), (64, 32), (64, 64)]


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
@pytest.mark.parametrize("tile", SPLIT_K_TILES, ids=lambda t: "%dx%d" % t)
def test_every_split_k_body_on_ragged_rows(tile, dtype):
    """The split-k wave grid (each wave a quarter of the k-tiles, private rings): the wave that holds the
    operand's last k-tile fixes the ragged chunks up itself.  Reduce extents whose last k-tile falls to
    each of the four waves, and shorter than four k-tiles."""
    tm, tn = tile
    for K in (203, 267, 331, 395, 71, 9):
        N, M = 4 * tn - 3, 2 * tm - 5
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dtype, n=N, k=K, m_lo=0, m_hi=1 << 16))
        s = ft.ft_ukernels_derive(op)
        infos = [ft.ft_ukset_get(s, i) for i in range(ft.ft_ukset_size(s))]
        ids = [u.id for u in infos if (u.tm, u.tn, u.gk) == (tm, tn, 4)]
        if not ids:
            continue
        g = np.random.default_rng(tm * 3 + tn + K + dtype)
        A = si.normal_bits(g, (M, K), 1.0, dtype)
        B = si.normal_bits(g, (K, N), 1.0, dtype)
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), ft.FT_PLAN_FORCED, ft.ft_forced_program(k1=ids[0], count1=2))
        ref, refabs = oc.matmul(A, B, dtype, want_abs=True)
        check(run_poisoned(plan, A, B, M * N, dtype), ref, refabs, f"ragged split-k body {tile} K {K} dtype {dtype}")


@pytest.mark.parametrize("M,N,K", [(100, 203, 331), (77, 768, 331), (300, 1000, 776), (1, 8, 8), (33, 9, 4095), (2048, 333, 513)])
@pytest.mark.parametrize("layout", [ft.FT_B_KN, ft.FT_B_NK], ids=["kn", "nk"])
def test_planner_plans_on_ragged_shapes(M, N, K, layout):
    dtype = ft.FT_BF16
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dtype, n=N, k=K, m_lo=0, m_hi=8192, b_layout=layout))
    s = ft.ft_ukernels_derive(op)
    g = np.random.default_rng(M + N + K)
    A = si.normal_bits(g, (M, K), 1.0, dtype)
    B = si.normal_bits(g, (K, N), K ** -0.5, dtype)
    ref, refabs = oc.matmul(A, B, dtype, want_abs=True)
    Bm = B if layout == ft.FT_B_KN else np.ascontiguousarray(B.T)
    for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
        plan = ft.ft_plan_create(op, s, ft.ft_shape(m=M), mode)
        for off_a, off_b in ((3, 5), (0, 0), (8, 1)):
            check(run_poisoned(plan, A, Bm, M * N, dtype, off_a, off_b), ref, refabs, f"ragged plan {M}x{N}x{K} mode {mode} layout {layout}")


@pytest.mark.parametrize("dtype", [ft.FT_F16, ft.FT_BF16])
def test_attention_of_odd_lengths_both_operators(dtype):
    """P V with P's odd row pitch and odd reduce extent (batch strides odd too), and Q K^T with K^T's
    odd row pitch: the lengths at and above 8 run the LDS-DMA bodies, the shorter ones the general ones."""
    pv = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=dtype, n=64, m_lo=0, m_hi=512, k_lo=0, k_hi=512, batch_hi=768))
    qk = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=dtype, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512, batch_hi=768))
    spv, sqk = ft.ft_ukernels_derive(pv), ft.ft_ukernels_derive(qk)
    for nb, L in ((12, 9), (12, 77), (24, 255), (12, 313), (3, 511), (7, 8), (5, 15), (12, 5), (4, 1)):
        g = np.random.default_rng(L + nb + dtype)
        Pm = si.normal_bits(g, (nb, L, L), 0.1, dtype)
        V = si.normal_bits(g, (nb, L, 64), 1.0, dtype)
        plan = ft.ft_plan_create(pv, spv, ft.ft_shape(batch=nb, m=L, k=L))
        ref, refabs = oc.bmm(Pm, V, dtype, want_abs=True)
        check(run_poisoned(plan, Pm, V, nb * L * 64, dtype), ref, refabs, f"PV batch {nb} L {L} dtype {dtype}")
        Q = si.normal_bits(g, (nb, L, 64), 1.0, dtype)
        Kt = si.normal_bits(g, (nb, 64, L), 1.0, dtype)
        plan = ft.ft_plan_create(qk, sqk, ft.ft_shape(batch=nb, m=L, n=L))
        ref, refabs = oc.bmm(Q, Kt, dtype, want_abs=True)
        check(run_poisoned(plan, Q, Kt, nb * L * L, dtype), ref, refabs, f"QK^T batch {nb} L {L} dtype {dtype}")


@pytest.mark.parametrize("lengths", [[77, 9, 128, 0, 257, 33, 100, 511, 16], [5, 77, 3, 128, 1, 257, 2, 40], [77, 128, 5], [300, 1, 1]],
                         ids=["all-at-least-8", "short-ones-inside", "short-one-last", "ones-last"])
def test_ragged_pv_grouped_on_odd_lengths(lengths):
    """Grouped P V of odd lengths on the LDS-DMA bodies, sequences shorter than 8 included (their rows are
    fetched together with what follows them in the packed buffer and cleared in LDS); with such a
    sequence at the very end of the buffer the launch takes the general bodies.  Either way every
    group matches the oracle, with NaNs around the buffers."""
    dtype = ft.FT_F16
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=dtype, n=64, m_lo=0, m_hi=512, k_lo=0, k_hi=512, batch_hi=768))
    s = ft.ft_ukernels_derive(op)
    groups = [ft.ft_shape(batch=3, m=L, k=L) for L in lengths]
    plan = ft.ft_plan_create_grouped(op, s, groups, ft.FT_PLAN_PATCHWORK)
    na, nb, nc = ft.ft_plan_group_layout(plan, len(groups))
    g = np.random.default_rng(41)
    A = si.normal_bits(g, (max(na, 1),), 0.1, dtype)
    B = si.normal_bits(g, (max(nb, 1),), 1.0, dtype)
    Cout = run_poisoned(plan, A, B, nc, dtype)
    for gi, L in enumerate(lengths):
        if L == 0:
            continue
        oa, ob, oc_ = ft.ft_plan_group_layout(plan, gi)
        ref, refabs = oc.bmm(A[oa:oa + 3 * L * L].reshape(3, L, L), B[ob:ob + 3 * L * 64].reshape(3, L, 64), dtype, want_abs=True)
        check(Cout[oc_:oc_ + 3 * L * 64], ref, refabs, f"grouped PV L {L}")
