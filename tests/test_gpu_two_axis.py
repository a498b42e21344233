"""GPU parity of plans with second-axis strips (both space axes of a batched Matmul dynamic):
up to four uKernel shapes in one launch, walked in table order.  Same oracle and tolerance as
everywhere; the plan itself must be the oracle's, byte for byte."""
import numpy as np
import pytest

import paper_2407_21418_amd as ft
import synth_inputs as si
from oracle import contraction as oc
from oracle import planner as P

from gpu_util import check, run

pytestmark = pytest.mark.gpu

# (M, N, batch): the planner's pick depends on the batch count (it multiplies the tile count)
SHAPES = [(133, 133, 96), (141, 141, 96), (390, 390, 96), (415, 415, 96), (450, 450, 96),
          (133, 281, 96), (313, 415, 96), (183, 313, 96), (136, 280, 96), (312, 416, 96),
          (183, 183, 768), (281, 281, 768), (313, 313, 768), (141, 141, 768)]


def _ops():
    d = ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512, batch_hi=768)
    o = P.Op(P.OP_BMM, P.F16, k=64, m_range=(0, 512), n_range=(0, 512), batch_hi=768)
    return ft.ft_op_register(d), o


def _tuning():
    """The strips are off by default (measured slower on this device, where the fp32 score matrix is
    bound by its own write): switched on for these tests, in the library and in the oracle."""
    t = ft.ft_tuning_default()
    t.second_axis_strips = 1
    return t, dict(P.default_tuning(), second_axis_strips=1)


@pytest.mark.parametrize("M,N,NB", SHAPES, ids=lambda v: str(v))
def test_attention_scores_with_strips(M, N, NB):
    op, oop = _ops()
    lt, ot = _tuning()
    s = ft.ft_ukernels_derive(op, None, lt)
    ouk = P.derive_ukernels(oop, t=ot)
    g = np.random.default_rng(M * 1000 + N)
    A = si.normal_bits(g, (NB, M, 64), 1.0, si.F16)
    B = si.normal_bits(g, (NB, 64, N), 1.0, si.F16)
    plan = ft.ft_plan_create(op, s, ft.ft_shape(batch=NB, m=M, n=N))
    want = P.plan(oop, ouk, (NB, M, N, 64), t=ot)
    assert ft.ft_plan_descriptors(plan) == b"".join(d.pack() for d in want.descs)
    st = ft.ft_plan_stats_get(plan)
    ref, refabs = oc.bmm(A, B, si.F16, want_abs=True)
    check(run(plan, A, B, NB * M * N), ref, refabs, f"{M}x{N} strips {list(st.strip_ukernel_id)}")


def test_the_shapes_above_do_exercise_strips():
    op, _ = _ops()
    s = ft.ft_ukernels_derive(op, None, _tuning()[0])
    kinds = set()
    for M, N, NB in SHAPES:
        st = ft.ft_plan_stats_get(ft.ft_plan_create(op, s, ft.ft_shape(batch=NB, m=M, n=N), ft.FT_PLAN_HOST_ONLY))
        n_strips = sum(st.strip_ukernel_id[i] != 0xFFFFFFFF for i in range(2))
        kinds.add((st.tau, n_strips, (M * 2) % 16 == 0 and (N * 2) % 16 == 0))
    assert any(k[1] == 1 for k in kinds) and any(k[1] == 2 for k in kinds)          # one and two strips
    assert any(k[0] == 1 and k[1] > 0 for k in kinds)                                # main axis = columns
    assert any(k[1] > 0 and k[2] for k in kinds) and any(k[1] > 0 and not k[2] for k in kinds)   # LDS-DMA and general bodies
