"""A second, independently written evaluation of the planner's scores, in exact rational arithmetic
(fractions.Fraction; no common denominators, no shared helpers), checked for equality against both
the planner oracle and the library on seeded (operator, shape, program) triples.

What is evaluated, from the definitions:
  Eq. 2  Pad  = useful output elements / elements covered by the tiles
  Eq. 3  Occ  = workgroups / ceil_by(workgroups, NumCores)
  Eq. 6-7 compute_eff = t_c / K_mem with t_c = FLOPs / FLOPS, t_g = (data_R + data_W) / bw_G,
         t_s = (data_transW + data_transR) / bw_S and K_mem read as the time of the k loop:
           a workgroup alone on its CU:  K_mem = t_ce + exposed * t_g + t_l
           workgroups sharing a CU:      K_mem = max(t_ce, t_g, t_s) + t_l / residents
           eight-wave grid alone:        K_mem = max(t_c, 2 t_s) + exposed / 2 * t_g + 2/3 t_l
           two teams (gk = 2):           K_mem = max(t_c, t_g, t_s) + phase latency * nk / residents
         t_ce = t_c * gk * ceil(nk / gk) / nk, t_l = k-tile latency * ceil(nk / gk) (+ the exchange of a
         reduce-axis split), nk = ceil(K / tk)
  Eq. 1  in product form: per constituent x = CMRn^c0 * Pad^c1 * Occ^c2 on its own sub-workload, two
         constituents combined by the harmonic mean weighted with their useful outputs.
Quantisation (part of the definition, so that plans are reproducible): every metric is the floor of
its exact value times 2^20; CMRn = floor(min(cmr, cap) * 2^20 / cap) on those integers; a product of
two such numbers is floor(x * y / 2^20); the mean is the floor of the exact ratio of the integers.
"""
import math
import random
from fractions import Fraction as Fr

import pytest

import paper_2407_21418_amd as ft
from oracle import planner as P

ONE = 1 << 20


def fl(x):
    return math.floor(x)


def second_compute_eff(u, k_extent, residents, out_bytes, hw, exchange=0):
    """Eq. 6 as an exact Fraction for uKernel u over a reduce extent of k_extent."""
    flops = Fr(2 * u.tm * u.tn * k_extent)
    t_c = flops / hw["mfma_flops_per_clk_per_cu"]
    data_r = (u.tm + u.tn) * k_extent * 2
    data_w = u.tm * u.tn * out_bytes
    t_g = Fr(data_r + data_w, hw["bw_global_bytes_per_clk_per_cu"])
    # what the copies write into LDS, plus what the waves read back: every wave column re-reads the A
    # rows of its wave row and every wave row the B columns of its wave column
    data_tw = data_r
    data_tr = k_extent * 2 * (u.tm * u.gn + u.tn * u.gm)
    t_s = Fr(data_tw + data_tr, hw["bw_lds_bytes_per_clk_per_cu"])
    nk = -(-k_extent // u.tk)
    res = residents
    if u.gm * u.gn == 8 and u.gk == 1 and residents < 2:
        t_l = Fr(hw["ktile_latency_clk"] * nk + exchange)
        k_mem = max(t_c, 2 * t_s) + Fr(hw["solo_copy_exposed_pct"], 200) * t_g + Fr(2, 3) * t_l
        return t_c / k_mem
    if u.gk == 2:
        k_mem = max(t_c, t_g, t_s) + Fr(hw["phase_latency_clk"] * nk + exchange, res)
        return t_c / k_mem
    nk_w = -(-nk // u.gk)
    t_ce = t_c * u.gk * nk_w / nk
    t_l = Fr(hw["ktile_latency_clk"] * nk_w + exchange)
    if res >= 2:
        k_mem = max(t_ce, t_g, t_s) + t_l / res
    else:
        k_mem = t_ce + Fr(hw["solo_copy_exposed_pct"], 100) * t_g + t_l
    return t_c / k_mem


def second_opinion(parts, uks, op, batch, M, N, K, tau, hw, t, k_parts=1):
    """Scores of the program `parts` = [(uKernel index, tiles along tau), ...] on shape (batch, M, N, K)."""
    parts = sorted(parts)
    H, W = (M, N) if tau == 0 else (N, M)
    W16 = 16 * (-(-W // 16))
    regions, offset = [], 0
    for uid, count in parts:
        u = uks[uid]
        e_tau, e_other = (u.tm, u.tn) if tau == 0 else (u.tn, u.tm)
        rows = max(0, min(H - offset, count * e_tau))
        offset += count * e_tau
        tiles = count * (-(-W16 // e_other))
        regions.append((u, tiles, rows * W, tiles * u.tm * u.tn))
    tiles_all = batch * sum(r[1] for r in regions)
    wgs = tiles_all * k_parts
    cores = hw["num_cus"]
    block_bound = min(max(1, -(-wgs // cores)), t["zeta"])
    # (an eight-wave grid brings two waves per SIMD with one workgroup: it counts twice against block.bound)
    out = {"block_bound": block_bound,
           "in_bound": all(r[0].max_wg_per_cu * (2 if r[0].gm * r[0].gn == 8 else 1) >= block_bound for r in regions),
           "pad_q": fl(Fr(M * N, sum(r[3] for r in regions)) * ONE),
           "occ_q": fl(Fr(wgs, cores * (-(-wgs // cores))) * ONE)}
    k_ref = op.k_ref()
    cap = max(max(fl(second_compute_eff(u, k_ref, 1, op.out_bytes, hw) * ONE),
                  fl(second_compute_eff(u, k_ref, 2, op.out_bytes, hw) * ONE)) for u in uks)

    def cmr_q(u):
        shared = min(u.max_wg_per_cu, block_bound) >= 2
        if k_parts == 1:
            v = second_compute_eff(u, k_ref, 2 if shared else 1, op.out_bytes, hw)
        else:
            nk = max(-(-K // u.tk), 1)
            k_one = -(-nk // k_parts) * u.tk
            rate = hw["part_exchange_bytes_per_clk"]
            exchange = hw["part_exchange_clk"] + ((k_parts * u.tm * u.tn * 4) // rate if rate else 0)
            v = second_compute_eff(u, k_one, 2 if shared else 1, op.out_bytes + 8, hw, exchange)
        return (min(fl(v * ONE), cap) * ONE) // cap

    out["cmr_q"] = sum(cmr_q(r[0]) for r in regions) // len(regions)
    terms = []
    for u, tiles, useful, area in regions:
        wg = batch * tiles * k_parts
        x = ONE
        for q, c in ((cmr_q(u), t["c0"]), (fl(Fr(useful, area) * ONE), t["c1"]),
                     (fl(Fr(wg, cores * (-(-wg // cores))) * ONE), t["c2"])):
            for _ in range(c):
                x = (x * q) // ONE
        terms.append((useful, x))
    if len(terms) > 1:
        weighted = [(w, x) for w, x in terms if w > 0]
        terms = weighted if weighted else terms[:1]
    if any(x == 0 for _, x in terms):
        out["sia_q"] = 0
    elif len(terms) == 1:
        out["sia_q"] = terms[0][1]
    else:
        out["sia_q"] = fl(Fr(sum(w for w, _ in terms)) / sum(Fr(w, x) for w, x in terms))
    return out


def _cases():
    rnd = random.Random(240721418)
    ops = []
    for (N, K) in ((768, 768), (3072, 768), (768, 3072), (4096, 4096), (1024, 2304), (11008, 4096), (304, 64)):
        for out_bytes in (4, 2):
            ops.append(P.Op(P.OP_MATMUL, P.F16, n=N, k=K, m_range=(1, 8192), out_bytes=out_bytes))
    ops.append(P.Op(P.OP_BMM, P.F16, k=64, m_range=(1, 512), n_range=(1, 512), batch_hi=768))
    ops.append(P.Op(P.OP_BMM, P.F16, n=64, m_range=(1, 512), k_range=(1, 512), batch_hi=768))
    ops.append(P.Op(P.OP_CONV2D, P.F16, c_in=64, c_out=128, r=3, s=3, stride=1, pad=1, m_range=(1, 1 << 22)))
    cases = []
    for op in ops:
        for _ in range(6):
            if op.kind == P.OP_MATMUL:
                shape = (1, rnd.choice([1, 16, 77, 80, 272, 300, 528, 1024, 1232, 1600, 2048, 4000, 8192, rnd.randint(1, 8192)]), op.n, op.k)
            elif op.kind == P.OP_BMM:
                L = rnd.randint(1, 512)
                shape = (rnd.choice([12, 96, 768]), L, op.n or L, op.k or L)
            else:
                res = rnd.choice([5, 28, 37, 56, 112])
                shape = (1, 8 * res * res, 128, 576)
            cases.append((op, shape))
    return cases


def _oracle_side(op, two_team):
    hw, t = P.default_hw(), P.default_tuning()
    if two_team:
        t["two_team_bodies"] = 1
    return hw, t, P.derive_ukernels(op, hw, t)


@pytest.mark.parametrize("two_team", [False, True], ids=["four-wave", "with-two-team"])
def test_second_opinion_equals_oracle_and_library(two_team):
    rnd = random.Random(7)
    n_checked = n_split = n_two = n_shared = 0
    for op, (batch, M, N, K) in _cases():
        hw, t, uks = _oracle_side(op, two_team)
        tau = P.main_axis(op, M, N)
        Hp = P.ceil_by(M if tau == 0 else N, P.GRANULE)
        pool = P.build_pool([P._ext(u, tau) for u in uks], Hp, kinds=[P.eight_waves(u) for u in uks])
        if not pool:
            continue
        cap_q = P.cmr_cap(uks)
        picks = rnd.sample(pool, min(8, len(pool)))
        for parts in picks:
            base = P.evaluate(parts, uks, batch, M, N, tau, hw, t, cap_q, out_bytes=op.out_bytes)
            mine = second_opinion(parts, uks, op, batch, M, N, K, tau, hw, t)
            got = dict(block_bound=base.block_bound, in_bound=base.in_bound, pad_q=base.pad_q, occ_q=base.occ_q,
                       cmr_q=base.cmr_q, sia_q=base.sia_q)
            assert mine == got, (op, (batch, M, N, K), parts)
            n_checked += 1
            n_two += len(parts) == 2
            n_shared += base.block_bound >= 2
            if op.kind == P.OP_MATMUL:
                for kp in (2, 3, 4, 6, 8):
                    if not P.split_allowed(parts, uks, K, kp, t, hw, base.num_tiles):
                        continue
                    sp = P.evaluate(parts, uks, batch, M, N, tau, hw, t, cap_q, k_parts=kp, K=K, out_bytes=op.out_bytes)
                    mine = second_opinion(parts, uks, op, batch, M, N, K, tau, hw, t, k_parts=kp)
                    assert mine == dict(block_bound=sp.block_bound, in_bound=sp.in_bound, pad_q=sp.pad_q, occ_q=sp.occ_q,
                                        cmr_q=sp.cmr_q, sia_q=sp.sia_q), (op, (batch, M, N, K), parts, kp)
                    n_split += 1
    assert n_checked >= 200 and n_split >= 20 and n_two >= 50 and n_shared >= 50, (n_checked, n_split, n_two, n_shared)


def test_second_opinion_equals_the_library_pool_scores():
    """The same evaluation against what the library reports for every program of its pools."""
    n = 0
    for (N, K, M) in ((768, 768, 1232), (3072, 768, 528), (768, 3072, 2048), (4096, 4096, 300), (768, 768, 77)):
        oop = P.Op(P.OP_MATMUL, P.F16, n=N, k=K, m_range=(1, 8192))
        hw, t, uks = _oracle_side(oop, False)
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=N, k=K, m_lo=1, m_hi=8192))
        s = ft.ft_ukernels_derive(op)
        for e in ft.ft_plan_pool(op, s, ft.ft_shape(m=M)):
            parts = [(e.k1, e.count1)] + ([(e.k2, e.count2)] if e.k2 != 0xFFFFFFFF else [])
            mine = second_opinion(parts, uks, oop, 1, M, N, K, 0, hw, t)
            assert (mine["pad_q"], mine["occ_q"], mine["cmr_q"], mine["sia_q"]) == (e.pad_q20, e.occ_q20, e.cmr_q20, e.sia_q20), (N, K, M, parts)
            assert mine["in_bound"] == bool(e.flags & 1)
            n += 1
    assert n >= 100
