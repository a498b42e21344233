"""Pins of the planner oracle: the paper's printed worked examples (tests/golden), closed
forms of Eq. 2-4, brute-force enumeration of decompositions, and the exact-cover invariant
of every emitted plan.  CPU only."""
import itertools
import os

import numpy as np
import pytest

from oracle import planner as P


def read_golden(golden_dir, name):
    out = {}
    with open(os.path.join(golden_dir, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [int(v) for v in vals]
    return out


def test_paper_combination_example(golden_dir):
    gdn = read_golden(golden_dir, "combination_example.txt")
    H, k1, k2 = gdn["H"][0], gdn["K1"][0], gdn["K2"][0]
    trace = []
    progs = P.combin_search(H, [k1, k2], trace=trace)
    assert progs[0] == [(k1, gdn["NUM1"][0]), (k2, gdn["NUM2"][0])]
    assert trace[0] == (k1, gdn["FIRST_REDUCED_H"][0])
    # the gfx950 reading (last success) gives the same decomposition on this example
    pool = P.build_pool([k1, k2], H)
    assert [(0, gdn["NUM1"][0]), (1, gdn["NUM2"][0])] in pool
    for prog in pool:
        assert sum([k1, k2][i] * c for i, c in prog) == H


def test_paper_prime_rule(golden_dir):
    gdn = read_golden(golden_dir, "regtile_prime_example.txt")
    n = gdn["LENGTH"][0]
    want = set()
    for m in gdn["NEIGHBOURS"]:
        want |= {d for d in range(1, m + 1) if m % d == 0}
    assert P.reg_tile_rule_factors(n) == sorted(want)
    assert P.reg_tile_rule_factors(12) == [1, 2, 3, 4, 6, 12]


def test_paper_occupancy_example(golden_dir):
    gdn = read_golden(golden_dir, "occupancy_example.txt")
    assert P.occ_fraction(gdn["BLOCKS"][0], gdn["CORES"][0]) == (gdn["OCC_NUM"][0], gdn["OCC_DEN"][0])
    for t in range(1, 400):
        n, d = P.occ_fraction(t, 80)
        assert 0 < n <= d and (n == d) == (t % 80 == 0)


def test_paper_crosspick_sweep(golden_dir):
    gdn = read_golden(golden_dir, "crosspick_sweep.txt")
    t = P.default_tuning()
    for key, name in [("EPS_MIN", "eps_min_pm"), ("EPS_MAX", "eps_max_pm"), ("EPS_STEP", "eps_step_pm"),
                      ("LAM_MAX", "lam_max_pm"), ("LAM_MIN", "lam_min_pm"), ("LAM_STEP", "lam_step_pm")]:
        assert t[name] == gdn[key][0]
    pts = P.sweep_points(t)
    assert len(pts) == gdn["POINTS"][0]
    assert pts[0] == (gdn["EPS_MIN"][0], gdn["LAM_MAX"][0])
    assert pts[-1] == (gdn["LAST_EPS"][0], gdn["LAST_LAM"][0])
    # staircase semantics on hand-made fractions
    assert P.cross_pick((1, 2), (95, 100), t)            # pad 0.50, occ 0.95: first step
    assert not P.cross_pick((49, 100), (1, 1), t)        # pad below eps_min never passes
    assert P.cross_pick((1, 1), (905, 1000), t)          # occ 0.905 passes only at the last step
    assert not P.cross_pick((1, 1), (904, 1000), t)
    assert not P.cross_pick((94, 100), (905, 1000), t)   # needs eps=0.95 for lam=0.905
    assert P.cross_pick((60, 100), (94, 100), t)         # step 10: eps 0.60, lam 0.94


def test_pad_fraction_closed_form():
    assert P.pad_fraction(77 * 768, 80 * 768) == (77 * 768, 80 * 768)
    n, d = P.pad_fraction(64 * 64, 64 * 64)
    assert n == d


def test_default_hyper_parameters_from_paper():
    t = P.default_tuning()
    assert t["zeta"] == 2 and (t["c0"], t["c1"], t["c2"]) == (1, 1, 1)


def test_sia_product_form_by_hand():
    """One uKernel, one shape, every factor recomputed from its definition."""
    op = P.Op(P.OP_MATMUL, P.F16, n=3072, k=768, m_range=(1, 8192))
    uks = P.derive_ukernels(op)
    hw, t = P.default_hw(), P.default_tuning()
    assert t["sia_form"] == P.SIA_PRODUCT
    cap = max(max(u.cmr_q, u.cmr2_q) for u in uks)
    assert cap == P.cmr_cap(uks)
    u = next(u for u in uks if (u.tm, u.tn, u.gk) == (128, 128, 1))
    p = P.evaluate([(u.id, 5)], uks, 1, 630, 3072, 0, hw, t, cap)          # H' = 640 = 5 * 128
    T = 5 * 24                                                              # 120 tiles <= 256 CUs:
    assert p.block_bound == 1                                               # one workgroup per CU
    cmr = (min(u.cmr_q, cap) << 20) // cap                                  # -> the solo value
    pad = ((630 * 3072) << 20) // (T * 128 * 128)
    occ = (T << 20) // 256
    assert p.sia_q == ((((cmr * pad) >> 20) * occ) >> 20)
    # two uKernels: harmonic mean of the two per-uKernel products, each on its own rows,
    # weighted by the useful elements each produces (work / summed time);
    # 96 + 384 tiles > 256 CUs: block.bound = 2, and both uKernels can share a CU
    # (capacity >= 2), so both take the shared-CU value
    v = next(x for x in uks if (x.tm, x.tn, x.gk) == (16, 64, 1))
    p2 = P.evaluate([(u.id, 4), (v.id, 8)], uks, 1, 630, 3072, 0, hw, t, cap)   # 512 + 128 rows
    assert p2.block_bound == 2 and u.max_wg_per_cu >= 2 and v.max_wg_per_cu >= 2
    cmr_u2 = (min(u.cmr2_q, cap) << 20) // cap
    s_u = ((((cmr_u2 * (1 << 20)) >> 20) * ((4 * 24 << 20) // 256)) >> 20)
    cmr_v = (min(v.cmr2_q, cap) << 20) // cap
    pad_v = ((118 * 3072) << 20) // (8 * 48 * 16 * 64)
    s_v = ((((cmr_v * pad_v) >> 20) * ((8 * 48 << 20) // 512)) >> 20)
    u1, u2 = 512 * 3072, 118 * 3072
    assert p2.sia_q == ((u1 + u2) * s_u * s_v) // (u1 * s_v + u2 * s_u)
    assert abs(p2.sia_q - (u1 + u2) / (u1 / s_u + u2 / s_v)) < 1
    # the printed linear form is still available
    p3 = P.evaluate([(u.id, 5)], uks, 1, 630, 3072, 0, hw, dict(t, sia_form=P.SIA_LINEAR), cap)
    assert p3.sia_q == p3.cmr_q + p3.pad_q + p3.occ_q


def test_resource_closed_forms():
    op = P.Op(P.OP_BMM, P.F16, n=768, k=768, m_range=(1, 100))     # too small to ever fill the device:
    uks = P.derive_ukernels(op)                                     # the workload filters are skipped
    by = {(u.tm, u.tn, u.wm, u.wn): u for u in uks}
    assert by[(32, 32, 32, 32)].gk == 4 and by[(32, 32, 32, 32)].stages == 5 and by[(32, 32, 32, 32)].max_wg_per_cu == 1
    u = by[(256, 256, 128, 128)]
    assert u.lds_bytes == 131072 and u.acc_regs == 256 and u.max_wg_per_cu == 1
    assert u.regs == 328 and u.reg_budget == 512
    u = by[(128, 128, 64, 64)]
    assert u.lds_bytes == 65536 and u.acc_regs == 64 and u.max_wg_per_cu == 2
    assert u.regs == 136 and u.reg_budget == 256 and u.stages == 2   # 2 waves/SIMD by registers, 2 workgroups by LDS
    assert by[(64, 128, 32, 64)].reg_budget == 128
    assert by[(16, 64, 16, 16)].stages == 8 and by[(64, 64, 32, 32)].stages == 5
    assert by[(128, 256, 64, 128)].reg_budget == 256
    for u in uks:
        share = 81920 if u.gk == 1 else 163840 // 4
        assert 2 <= u.stages <= 8 and u.stages == max(2, min(8, share // ((u.tm + u.tn) * 128)))
        assert u.lds_bytes == u.gk * u.stages * (u.tm + u.tn) * u.tk * 2 <= 163840
        assert u.acc_regs * 64 == u.wm * u.wn
        assert u.tm == u.gm * u.wm and u.tn == u.gn * u.wn and u.gm * u.gn * u.gk == 4
        assert 768 % u.tn == 0                              # static axis divided evenly
        assert u.tk % (16 if u.mfma == 0 else 32) == 0
        assert (u.mfma == 1) == (u.wm == 16)
    # canonical order: non-increasing area, ids consecutive
    areas = [u.tm * u.tn for u in uks]
    assert areas == sorted(areas, reverse=True)
    assert [u.id for u in uks] == list(range(len(uks)))
    assert len({(u.tm, u.tn, u.tk, u.wm, u.wn) for u in uks}) == len(uks)


def test_workload_filters_crosspick_and_eq5():
    """A uKernel survives iff some shape of the workload, tiled by it alone, reaches
    zeta x NumCores tiles and passes the CrossPick staircase (checked here by enumerating
    every M of a range whose samples are all its multiples of 16)."""
    hw, t = P.default_hw(), P.default_tuning()
    op = P.Op(P.OP_MATMUL, P.F16, n=768, k=768, m_range=(1, 4096))
    assert P.axis_samples(1, 4096, 256) == [1] + list(range(16, 4097, 16))
    assert P.axis_samples(1, 8192, 256)[:3] == [1, 16, 48] and P.axis_samples(1, 8192, 256)[-1] == 8192
    assert P.axis_samples(5, 3, 256) == [] and P.axis_samples(0, 7, 256) == [1, 7]
    got = {(u.tm, u.tn, u.wm, u.wn) for u in P.derive_ukernels(op)}
    for tm, tn in [(256, 256), (128, 128), (128, 64), (64, 64), (16, 64), (256, 32)]:
        want = False
        for M in range(1, 4097):
            T = -(-M // tm) * (768 // tn)
            if T >= 512 and P.cross_pick((M * 768, T * tm * tn), P.occ_fraction(T, 256), t):
                want = True
                break
        assert any(k[:2] == (tm, tn) for k in got) == want, (tm, tn)
    # 256x256 on N = 768 never reaches 512 tiles for M <= 4096; 64x64 does
    assert not any(k[:2] == (256, 256) for k in got) and any(k[:2] == (64, 64) for k in got)


def test_compute_eff_closed_form():
    hw = P.default_hw()
    # 128x128 tile, 2x2 waves, K = 768: t_c = 2*128*128*768 flop at 4096 flop/clk = 6144 clk;
    # t_g = (256*768*2 + 128*128*4) B / 64 = 7168 clk; t_s = (393216 + 768*2*512) B / 256 = 4608 clk;
    # k-loop latency 400 clk x 12 k-tiles = 4800 clk
    #   alone on the CU:  K_mem = t_c + 50 % of t_g + latency = 6144 + 3584 + 4800
    n, d = P.compute_eff(128, 128, 2, 2, 768, hw)
    assert n * (6144 + 3584 + 4800) == d * 6144
    #   two workgroups share the CU:  K_mem = max(t_c, t_g, t_s) + latency / 2 = 7168 + 2400
    n, d = P.compute_eff(128, 128, 2, 2, 768, hw, residents=2)
    assert n * (7168 + 2400) == d * 6144
    # split-k grid: the four waves share the 12 k-tiles
    n4, d4 = P.compute_eff(32, 32, 1, 1, 768, hw, gk=4)
    t_c, t_g = 2 * 32 * 32 * 768 / 4096, (64 * 768 * 2 + 32 * 32 * 4) / 64
    assert abs(n4 / d4 - t_c / (t_c + t_g / 2 + 400 * 12 / 4)) < 1e-12
    n4, d4 = P.compute_eff(32, 32, 1, 1, 768, hw, gk=4, residents=3)
    t_s = (64 * 768 * 2 + 768 * 2 * 64) / 256
    assert abs(n4 / d4 - t_c / (max(t_c, t_g, t_s) + 400 * 12 / 4 / 3)) < 1e-12
    # a split-k grid on a single k-tile (K = 64) leaves three of its four waves idle: the MFMA
    # phase lasts 4 x t_c and the one working wave pays the full k-tile latency
    n1, d1 = P.compute_eff(32, 32, 1, 1, 64, hw, gk=4)
    t_c1, t_g1 = 2 * 32 * 32 * 64 / 4096, (64 * 64 * 2 + 32 * 32 * 4) / 64
    assert abs(n1 / d1 - t_c1 / (4 * t_c1 + t_g1 / 2 + 400)) < 1e-12
    # K = 576 (nine k-tiles): a wave of the split-k grid walks ceil(9 / 4) = 3 of them
    n9, d9 = P.compute_eff(32, 32, 1, 1, 576, hw, gk=4)
    t_c9, t_g9 = 2 * 32 * 32 * 576 / 4096, (64 * 576 * 2 + 32 * 32 * 4) / 64
    assert abs(n9 / d9 - t_c9 / (t_c9 * 12 / 9 + t_g9 / 2 + 400 * 3)) < 1e-12
    # a bigger tile is more compute-intensive; the ratio is an efficiency, never above 1
    n1, d1 = P.compute_eff(128, 128, 2, 2, 768, hw)
    n2, d2 = P.compute_eff(256, 256, 2, 2, 768, hw)
    assert n2 * d1 > n1 * d2 and n2 <= d2
    assert P.compute_eff(256, 256, 2, 2, 1 << 20, dict(hw, ktile_latency_clk=0), residents=2)[0] == \
           P.compute_eff(256, 256, 2, 2, 1 << 20, dict(hw, ktile_latency_clk=0), residents=2)[1]   # MFMA bound: 1


def brute_decompositions(H, extents):
    out = set()
    for (i1, e1), (i2, e2) in itertools.permutations(list(enumerate(extents)), 2):
        for n1 in range(1, H // e1 + 1):
            rem = H - n1 * e1
            if rem > 0 and rem % e2 == 0:
                out.add((i1, n1, i2, rem // e2))
    return out


@pytest.mark.parametrize("extents", [[7, 8], [16, 32, 48, 64], [5, 9, 12], [16, 64, 256]])
def test_pool_against_brute_force(extents):
    for H in range(1, 200):
        pool = P.build_pool(extents, H)
        brute = brute_decompositions(H, extents)
        for prog in pool:
            assert sum(extents[i] * c for i, c in prog) == H and all(c >= 1 for _, c in prog)
        for i1, e1 in enumerate(extents):
            mine = [p for p in pool if p[0][0] == i1]
            if H % e1 == 0:
                assert mine == [[(i1, H // e1)]]
                continue
            feas = [d for d in brute if d[0] == i1]
            if not feas:
                assert mine == []
                continue
            n1max = max(d[1] for d in feas)
            want = sorted((i1, n1, i2, n2) for (_, n1, i2, n2) in feas if n1 == n1max)
            got = sorted((p[0][0], p[0][1], p[1][0], p[1][1]) for p in mine)
            assert got == want


SHAPES = [(1, 77, 768, 768), (1, 1, 768, 768), (1, 15, 768, 768), (1, 16, 768, 768),
          (1, 17, 768, 768), (1, 1232, 3072, 768), (1, 2048, 768, 3072), (1, 8191, 768, 768)]


@pytest.mark.parametrize("mode", [P.PLAN_PATCHWORK, P.PLAN_PAD_BASELINE])
@pytest.mark.parametrize("shape", SHAPES)
def test_matmul_plans_cover_exactly_once(shape, mode):
    _, M, N, K = shape
    op = P.Op(P.OP_MATMUL, P.F16, n=N, k=K, m_range=(1, 8192))
    uks = P.derive_ukernels(op)
    pl = P.plan(op, uks, shape, mode)
    cnt = P.exact_cover_counts(pl, uks)
    assert cnt.min() == 1 and cnt.max() == 1
    check_plan_invariants(pl, uks, mode)


def check_plan_invariants(pl, uks, mode):
    prog = pl.program
    tau_ext = lambda u: u.tm if pl.tau == 0 else u.tn
    H = pl.M if pl.tau == 0 else pl.N
    total = sum(tau_ext(uks[i]) * c for i, c in prog.parts)
    if mode == P.PLAN_PATCHWORK:
        assert total == P.ceil_by(H, 16)                 # zero padding on tau up to the granule
        assert len(prog.parts) <= 2
    else:
        assert prog.parts[0][0] == 0 and total == P.ceil_by(H, tau_ext(uks[0]))
    seen = set()
    area = 0
    for d in pl.descs:
        u = uks[d.ukernel_id]
        assert d.m0 % 16 == 0 and d.n0 % 16 == 0
        assert d.m_valid == min(u.tm, pl.M - d.m0) and d.n_valid == min(u.tn, pl.N - d.n0)
        assert d.m_valid > 0 and d.n_valid > 0
        assert d.flags == (1 if (d.m_valid < u.tm or d.n_valid < u.tn) else 0)
        key = (d.batch, d.m0, d.n0)
        assert key not in seen
        seen.add(key)
        area += u.tm * u.tn
    assert area == pl.covered and pl.useful == pl.batch * pl.M * pl.N
    order = [(d.ukernel_id, d.batch, d.m0, d.n0) for d in pl.descs]
    assert order == sorted(order)
    assert prog.pad_q == (pl.useful << 20) // pl.covered
    assert len(pl.descs[0].pack()) == 24


def test_bmm_two_dynamic_axes_and_dynamic_k():
    qk = P.Op(P.OP_BMM, P.F16, k=64, m_range=(1, 512), n_range=(1, 512))
    pv = P.Op(P.OP_BMM, P.F16, n=64, m_range=(1, 512), k_range=(1, 512))
    uq, up = P.derive_ukernels(qk), P.derive_ukernels(pv)
    assert all(u.tn in (16, 32, 64) for u in up)
    for L in (1, 7, 16, 33, 100, 257, 512):
        for op, uks, shape in ((qk, uq, (3, L, L, 64)), (pv, up, (3, L, 64, L))):
            for mode in (P.PLAN_PATCHWORK, P.PLAN_PAD_BASELINE):
                pl = P.plan(op, uks, shape, mode)
                cnt = P.exact_cover_counts(pl, uks)
                assert cnt.min() == 1 and cnt.max() == 1
                check_plan_invariants(pl, uks, mode)


def test_main_axis_choice():
    both = P.Op(P.OP_BMM, P.F16, k=64, m_range=(1, 512), n_range=(1, 512))
    assert P.main_axis(both, 100, 100) == 0 and P.main_axis(both, 10, 100) == 1
    only_n = P.Op(P.OP_BMM, P.F16, m=64, k=64, n_range=(1, 512))
    assert P.main_axis(only_n, 64, 7) == 1
    uks = P.derive_ukernels(only_n)
    pl = P.plan(only_n, uks, (2, 64, 77, 64))
    assert pl.tau == 1
    cnt = P.exact_cover_counts(pl, uks)
    assert cnt.min() == 1 and cnt.max() == 1
    check_plan_invariants(pl, uks, P.PLAN_PATCHWORK)


def test_conv_shape_mapping_and_cover():
    op = P.Op(P.OP_CONV2D, P.F16, c_in=64, c_out=128, r=3, s=3, stride=1, pad=1, m_range=(1, 1 << 20))
    uks = P.derive_ukernels(op)
    assert all(128 % u.tn == 0 for u in uks)
    shape = P.resolve_shape(op, img_n=8, img_h=37, img_w=37)
    assert shape == (1, 8 * 37 * 37, 128, 576)
    pl = P.plan(op, uks, shape)
    cnt = P.exact_cover_counts(pl, uks)
    assert cnt.min() == 1 and cnt.max() == 1
    check_plan_invariants(pl, uks, P.PLAN_PATCHWORK)


def test_empty_shapes_give_empty_plans():
    op = P.Op(P.OP_BMM, P.F16, k=64, m_range=(0, 512), n_range=(0, 512))
    uks = P.derive_ukernels(op)
    for shape in [(0, 5, 5, 64), (2, 0, 5, 64), (2, 5, 0, 64)]:
        pl = P.plan(op, uks, shape)
        assert pl.descs == [] and pl.program is None


def test_pad_baseline_wastes_at_least_as_much_as_patchwork():
    op = P.Op(P.OP_MATMUL, P.F16, n=768, k=768, m_range=(1, 8192))
    uks = P.derive_ukernels(op)
    for M in [1, 5, 77, 80, 100, 272, 528, 1000, 1232, 1600, 2048, 4097]:
        a = P.plan(op, uks, (1, M, 768, 768), P.PLAN_PATCHWORK)
        b = P.plan(op, uks, (1, M, 768, 768), P.PLAN_PAD_BASELINE)
        assert a.covered <= b.covered
        assert a.covered == P.ceil_by(M, 16) * 768       # only granule padding is left


def test_sia_is_the_weighted_sum_and_top1_is_max():
    op = P.Op(P.OP_MATMUL, P.F16, n=3072, k=768, m_range=(1, 8192))
    uks = P.derive_ukernels(op)
    hw, t = P.default_hw(), P.default_tuning()
    t2 = dict(t, c0=3, c1=5, c2=7, sia_form=P.SIA_LINEAR)
    cap = P.cmr_cap(uks)
    shape = (1, 528, 3072, 768)
    pool = [P.evaluate(p, uks, 1, 528, 3072, 0, hw, t2, cap)
            for p in P.build_pool([u.tm for u in uks], 528, kinds=[P.eight_waves(u) for u in uks])]
    for p in pool:
        assert p.sia_q == 3 * p.cmr_q + 5 * p.pad_q + 7 * p.occ_q
        assert 0 <= p.cmr_q <= 1 << 20 and 0 < p.pad_q <= 1 << 20 and 0 < p.occ_q <= 1 << 20
    pl = P.plan(op, uks, shape, hw=hw, t=t2)
    cands = [p for p in pool if p.in_bound] or pool
    assert pl.program.sia_q == max(p.sia_q for p in cands)


# --------------------------------------------------------------------------------------
# reduce-axis split over workgroups (occupancy rescue)
# --------------------------------------------------------------------------------------
def test_compute_eff_of_one_part_closed_form():
    """One part of a split tile: 128x128, 2x2 waves, its share of the reduce axis 1024 (16 k-tiles),
    12 bytes of global traffic per output element (fp32 C + the partial written and read once) and
    4000 clk of exchange latency.  t_c = 2*128*128*1024 / 4096 = 8192 clk;
    t_g = (256*1024*2 + 128*128*12) / 64 = 11264 clk; t_s = (524288 + 1024*2*512) / 256 = 6144 clk;
    t_l = 400 * 16 = 6400 clk."""
    hw = P.default_hw()
    n, d = P.compute_eff(128, 128, 2, 2, 1024, hw, out_bytes=12, exchange_clk=4000)
    assert n * (8192 + 5632 + 6400 + 4000) == d * 8192             # alone: t_c + t_g/2 + t_l + X
    n, d = P.compute_eff(128, 128, 2, 2, 1024, hw, residents=2, out_bytes=12, exchange_clk=4000)
    assert n * (11264 + (6400 + 4000) // 2) == d * 8192             # shared: max(..) + (t_l + X)/2
    # without the exchange arguments nothing changes
    assert P.compute_eff(128, 128, 2, 2, 1024, hw, exchange_clk=0) == P.compute_eff(128, 128, 2, 2, 1024, hw)


def test_part_tiles_and_split_rules():
    hw, t = P.default_hw(), P.default_tuning()
    assert P.part_tiles(3072, 64, 3) == 16 and P.part_tiles(712, 64, 5) == 3 and P.part_tiles(0, 64, 1) == 1
    op = P.Op(P.OP_MATMUL, P.F16, n=768, k=3072, m_range=(0, 8192))
    uks = P.derive_ukernels(op)
    by = {(u.tm, u.tn, u.gk): u for u in uks}
    small = by[(64, 128, 1)]                        # 32 accumulator registers, two workgroups per CU
    assert small.acc_regs <= P.KPART_ACC_MAX and small.max_wg_per_cu >= 2
    parts = [(small.id, 25)]                        # M = 1600: 25 x 6 = 150 tiles
    ok = lambda kp, tiles=150, K=3072, tt=t: P.split_allowed(parts, uks, K, kp, tt, hw, tiles)
    assert ok(1) and ok(2) and ok(3)
    assert not ok(4)                                # 600 workgroups > 256 CUs x 2
    assert ok(4, tiles=128) and not ok(4, tiles=129)
    assert not ok(8, tiles=10)                      # 48 k-tiles / 8 = 6 < k_part_min_tiles
    assert ok(8, tiles=10, tt=dict(t, k_part_min_tiles=6))
    assert not ok(2, tt=dict(t, k_parts_max=1))
    assert not ok(5, tiles=10, K=712)               # 12 k-tiles in runs of 3 make 4 parts, not 5
    assert not ok(2, K=768)                         # 12 k-tiles / 2 = 6 < 8
    big = max(uks, key=lambda u: u.acc_regs)
    if big.acc_regs > P.KPART_ACC_MAX:
        assert not P.split_allowed([(big.id, 1)], uks, 3072, 2, t, hw, 1)
    # a uKernel that owns its CU (split-k wave grid) offers one slot per CU
    solo = next(u for u in uks if u.gk == 4 and u.max_wg_per_cu == 1 and u.acc_regs <= P.KPART_ACC_MAX)
    assert P.split_allowed([(solo.id, 1)], uks, 3072, 2, t, hw, 128)
    assert not P.split_allowed([(solo.id, 1)], uks, 3072, 2, t, hw, 129)


def test_split_program_counts_workgroups():
    """Eq. 3, Eq. 5 and SetBound on tiles x k_parts workgroups; Eq. 2 unchanged."""
    hw, t = P.default_hw(), P.default_tuning()
    op = P.Op(P.OP_MATMUL, P.F16, n=768, k=3072, m_range=(0, 8192))
    uks = P.derive_ukernels(op)
    u = next(u for u in uks if (u.tm, u.tn, u.gk) == (64, 128, 1))
    cap = P.cmr_cap(uks)
    whole = P.evaluate([(u.id, 25)], uks, 1, 1600, 768, 0, hw, t, cap)
    split = P.evaluate([(u.id, 25)], uks, 1, 1600, 768, 0, hw, t, cap, 3, 3072, 4)
    assert (whole.num_tiles, whole.block_bound, whole.occ_q) == (150, 1, (150 << 20) // 256)
    assert (split.num_tiles, split.block_bound, split.occ_q) == (150, 2, (450 << 20) // 512)
    assert split.pad_q == whole.pad_q == 1 << 20 and split.k_parts == 3
    # its compute_eff is Eq. 6 on 16 k-tiles with the exchange, two workgroups per CU, normalised
    # exchange: 2000 clk of round trips + 3 partial tiles of 64 x 128 fp32 read at 16 bytes per clock
    assert (hw["part_exchange_clk"], hw["part_exchange_bytes_per_clk"]) == (2000, 16)
    n, d = P.compute_eff(64, 128, u.gm, u.gn, 1024, hw, residents=2, out_bytes=12, exchange_clk=2000 + 3 * 64 * 128 * 4 // 16)
    assert split.cmr_q == (min((n << 20) // d, cap) << 20) // cap
    assert split.sia_q == (((split.cmr_q * split.pad_q) >> 20) * split.occ_q) >> 20


@pytest.mark.parametrize("M,N,K,expect_split", [(528, 768, 3072, True), (1600, 768, 768, False),
                                                (16, 4096, 4096, True), (8192, 4096, 4096, False)])
def test_plans_split_only_where_the_device_is_underfilled(M, N, K, expect_split):
    hw, t = P.default_hw(), P.default_tuning()
    op = P.Op(P.OP_MATMUL, P.BF16, n=N, k=K, m_range=(1, 8192))
    uks = P.derive_ukernels(op)
    pl = P.plan(op, uks, (1, M, N, K))
    assert (pl.k_parts > 1) == expect_split
    nk = -(-K // 64)
    assert (pl.k_parts - 1) * pl.k_part_tiles < nk <= pl.k_parts * pl.k_part_tiles      # no empty part
    if pl.k_parts > 1:
        per_cu = min([t["zeta"]] + [uks[i].max_wg_per_cu for i, _ in pl.program.parts])
        assert pl.program.num_tiles * pl.k_parts <= hw["num_cus"] * per_cu
        assert pl.k_part_tiles >= t["k_part_min_tiles"]
        assert all(uks[i].acc_regs <= P.KPART_ACC_MAX for i, _ in pl.program.parts)
    # switching the rescue off gives a plan of whole tiles, never a better-scored one
    off = P.plan(op, uks, (1, M, N, K), t=dict(t, k_parts_max=1))
    assert off.k_parts == 1 and off.program.sia_q <= pl.program.sia_q
    # BMM and the pad baseline never split
    assert P.plan(op, uks, (1, M, N, K), P.PLAN_PAD_BASELINE).k_parts == 1


# --------------------------------------------------------------------------------------
# second-axis strips (two dynamic space axes, Fig. 4(d))
# --------------------------------------------------------------------------------------
def _qk():
    op = P.Op(P.OP_BMM, P.F16, k=64, m_range=(0, 512), n_range=(0, 512), batch_hi=768)
    return op, P.derive_ukernels(op)


def test_strip_choices_against_brute_force():
    op, uks = _qk()
    for Wp in (16, 48, 112, 144, 208, 272, 464, 512):
        for u in uks:
            got = P.strip_choices(u, uks, Wp, 0)
            e = u.tn
            if Wp % e == 0 or e > Wp:
                assert got == []
                continue
            n_full, rem = divmod(Wp, e)
            ok = [v for v in uks if v.tm == u.tm and v.tn < e and -(-rem // v.tn) * v.tn < e]
            ok.sort(key=lambda v: (-v.tn, v.id))
            assert got == [(v.id, n_full, -(-rem // v.tn)) for v in ok[:P.STRIP_CHOICES]]
            for sid, a, b in got:                       # the strip closes the gap and pads less than one more K1 tile
                assert a * e + b * uks[sid].tn >= Wp > a * e + (b - 1) * uks[sid].tn
                assert a * e + b * uks[sid].tn < (a + 1) * e
    # along the other main axis the roles of tm and tn swap
    u = next(u for u in uks if (u.tm, u.tn) == (128, 128))
    for sid, a, b in P.strip_choices(u, uks, 208, 1):
        assert uks[sid].tn == 128 and uks[sid].tm < 128 and a == 1


def test_strip_variants_order_and_count():
    op, uks = _qk()
    by = {(u.tm, u.tn, u.gk): u for u in uks}
    parts = [(by[(64, 64, 1)].id, 1), (by[(16, 64, 1)].id, 3)]          # L = 100: H' = W' = 112 = 64 + 3*16
    c0 = P.strip_choices(uks[parts[0][0]], uks, 112, 0)
    c1 = P.strip_choices(uks[parts[1][0]], uks, 112, 0)
    assert c0 and c1
    var = P.strip_variants(parts, uks, 112, 0)
    assert len(var) == (1 + len(c0)) * (1 + len(c1)) - 1
    none0, none1 = (-1, 2, 0), (-1, 2, 0)
    assert var[0] == [none0, c1[0]]                                  # first part varies slowest, 'none' first
    assert var[len(c1)] == [c0[0], none1]
    assert all(any(s[0] >= 0 for s in v) for v in var)
    # a program whose tiles divide W' has no variants
    assert P.strip_variants([(by[(16, 16, 4)].id, 7)], uks, 112, 0) == []


def test_constituents_and_harmonic_mean_of_three_regions_by_hand():
    from fractions import Fraction
    op, uks = _qk()
    hw, t = P.default_hw(), P.default_tuning()
    by = {(u.tm, u.tn, u.gk): u for u in uks}
    k1, k2, ks = by[(64, 64, 1)], by[(16, 64, 1)], by[(64, 16, 1)]
    parts = sorted([(k1.id, 1), (k2.id, 3)])
    strips = [(ks.id, 1, 3) if uid == k1.id else (-1, 2, 0) for uid, _ in parts]
    cons = P.constituents(parts, strips, uks, 1, 100, 100, 0)
    want = {k1.id: (1, 64 * 64, 64 * 64), ks.id: (3, 64 * 36, 3 * 64 * 16), k2.id: (6, 36 * 100, 6 * 16 * 64)}
    assert {c[0]: c[1:] for c in cons} == want and sum(c[2] for c in cons) == 100 * 100
    cap = P.cmr_cap(uks)
    p = P.evaluate(parts, uks, 12, 100, 100, 0, hw, t, cap, strips=strips)
    assert p.num_tiles == 12 * 10 and p.area == 64 * 64 + 3 * 64 * 16 + 6 * 16 * 64
    # score = sum u_i / sum (u_i / x_i) with x_i = CMR * Pad * Occ of region i in q20 steps
    xs = []
    for uid, tiles, useful, area in cons:
        u = uks[uid]
        x = (min(P.cmr_at(u, p.block_bound), cap) << 20) // cap
        x = (x * ((useful << 20) // area)) >> 20
        T = 12 * tiles
        x = (x * ((T << 20) // (256 * -(-T // 256)))) >> 20
        xs.append((useful, x))
    exact = Fraction(sum(u for u, _ in xs)) / sum(Fraction(u, x) for u, x in xs)
    assert p.sia_q == int(exact)                        # floor of the exact ratio


def test_every_strip_variant_is_an_exact_cover_and_pads_no_more():
    op, uks = _qk()
    hw, t = P.default_hw(), P.default_tuning()
    cap = P.cmr_cap(uks)
    checked = 0
    for L in (33, 100, 141, 257):
        Hp = P.ceil_by(L, 16)
        for parts in P.build_pool([u.tm for u in uks], Hp, kinds=[P.eight_waves(u) for u in uks])[::7]:
            whole = P.evaluate(parts, uks, 2, L, L, 0, hw, t, cap)
            for strips in P.strip_variants(parts, uks, Hp, 0):
                p = P.evaluate(parts, uks, 2, L, L, 0, hw, t, cap, strips=strips)
                assert p.area <= whole.area
                descs = P.emit(p.parts, uks, 2, L, L, 0, p.strips)
                assert len(descs) == p.num_tiles
                assert [(d.ukernel_id, d.batch, d.m0, d.n0) for d in descs] == sorted((d.ukernel_id, d.batch, d.m0, d.n0) for d in descs)
                pl = P.Plan(2, L, L, 64, 0, p, descs)
                assert (P.exact_cover_counts(pl, uks) == 1).all(), (L, parts, strips)
                assert sum(uks[d.ukernel_id].tm * uks[d.ukernel_id].tn for d in descs) == 2 * p.area
                checked += 1
    assert checked > 50
    # main axis = columns (more columns than rows): strips run down the rows
    pl = P.plan(op, uks, (2, 100, 141, 64), t=dict(t, second_axis_strips=1))
    assert pl.tau == 1 and (P.exact_cover_counts(pl, uks) == 1).all()


def test_strips_only_when_asked_for_and_with_two_dynamic_axes():
    op, uks = _qk()
    on = dict(P.default_tuning(), second_axis_strips=1)
    picked = 0
    for L in (97, 133, 183, 281, 313, 390, 415, 450):
        pl = P.plan(op, uks, (768, L, L, 64), t=on)
        picked += bool(pl.program.strips)
        assert (P.exact_cover_counts(P.plan(op, uks, (1, L, L, 64), t=on), uks) == 1).all()
        assert P.plan(op, uks, (768, L, L, 64)).program.strips == []          # off by default
    assert picked >= 3                                   # the planner does use them
    one_axis = P.Op(P.OP_BMM, P.F16, n=64, m_range=(0, 512), k_range=(0, 512), batch_hi=768)
    assert P.plan(one_axis, P.derive_ukernels(one_axis), (96, 141, 64, 141), t=on).program.strips == []
    mm = P.Op(P.OP_MATMUL, P.F16, n=768, k=768, m_range=(0, 8192))
    assert P.plan(mm, P.derive_ukernels(mm), (1, 1232, 768, 768), t=on).program.strips == []


def test_eq6_threshold_is_dropped_only_when_nothing_reaches_it():
    """Eq. 6: with a reduce axis of a few elements every loop is latency and no uKernel reaches psi;
    the set must not come out empty (the threshold is then not applied).  Where some reach it, those
    that do not are still filtered out."""
    hw, t = P.default_hw(), P.default_tuning()
    below = lambda u, k: (lambda n, d: n * t["psi_den"] < t["psi_num"] * d)(
        *P.compute_eff(u.tm, u.tn, u.gm, u.gn, k, hw, u.gk, u.tk, out_bytes=4))
    tiny = P.derive_ukernels(P.Op(P.OP_MATMUL, P.BF16, n=304, k=12, m_range=(0, 1024)))
    assert tiny and all(below(u, 12) for u in tiny)
    assert P.plan(P.Op(P.OP_MATMUL, P.BF16, n=304, k=12, m_range=(0, 1024)), tiny, (1, 543, 304, 12)).descs
    usual = P.derive_ukernels(P.Op(P.OP_MATMUL, P.F16, n=768, k=768, m_range=(0, 8192)))
    assert usual and not any(below(u, 768) for u in usual)


def test_grouped_table_covers_every_group_exactly_once_heaviest_first():
    """plan_grouped: brute-force cover of every group's outputs by its own descriptors (each element
    of each batch entry exactly once, nothing from another group's shape), offsets by hand, and the
    order of the table."""
    op = P.Op(P.OP_BMM, P.F16, m_range=(0, 512), n_range=(0, 512), k_range=(0, 512), batch_hi=64)
    uks = P.derive_ukernels(op)
    shapes = [(2, 37, 50, 9), (3, 100, 7, 300), (0, 64, 64, 64), (1, 129, 257, 300), (2, 0, 40, 8), (4, 16, 16, 16)]
    table, offsets = P.plan_grouped(op, uks, shapes)
    # offsets: running sums of batch * M * K, batch * K * N, batch * M * N in the order given
    assert offsets[0] == (0, 0, 0) and offsets[1] == (2 * 37 * 9, 2 * 9 * 50, 2 * 37 * 50)
    assert offsets[-1] == (sum(b * m * k for b, m, n, k in shapes), sum(b * k * n for b, m, n, k in shapes),
                           sum(b * m * n for b, m, n, k in shapes))
    # order: reduce extent descending, then output size descending; empty groups contribute nothing
    seen = []
    for g, _ in table:
        if not seen or seen[-1] != g:
            seen.append(g)
    assert seen == [3, 1, 5, 0]          # K = 300 twice (the larger output first), then K = 16, then K = 9
    for g, (b, M, N, K) in enumerate(shapes):
        count = [[[0] * N for _ in range(M)] for _ in range(b)]
        for gg, d in table:
            if gg != g:
                continue
            u = uks[d.ukernel_id]
            assert d.batch < b and d.m_valid == min(u.tm, M - d.m0) and d.n_valid == min(u.tn, N - d.n0)
            for i in range(d.m0, d.m0 + d.m_valid):
                for j in range(d.n0, d.n0 + d.n_valid):
                    count[d.batch][i][j] += 1
        assert all(c == 1 for e in count for row in e for c in row), g
    # the launch's batch: 12 entries -> 16; a group planned alone at its own batch may differ, at 16 it may not
    b, M, N, K = shapes[1]
    own = [d for g, d in table if g == 1]
    at_launch = [d for d in P.plan(op, uks, (16, M, N, K)).descs if d.batch < b]
    assert [d.pack() for d in own] == [d.pack() for d in at_launch]
