"""Host-side checks of libftuner.so that need no GPU: every declared symbol is exported, the
uKernel table and every plan are bit-identical to the planner oracle's, error codes."""
import os
import re

import numpy as np
import pytest

import paper_2407_21418_amd as ft
from oracle import planner as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST = ft.FT_PLAN_HOST_ONLY


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "ftuner.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ft_[a-z0-9_]+)\s*\(", hdr))
    assert declared, "no declarations parsed"
    lib = ft.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in ftuner.h but not exported"
    assert declared == set(ft.SYMBOLS), (declared ^ set(ft.SYMBOLS))


def to_lib_op(op: P.Op):
    d = ft.ft_op_desc(kind=op.kind, dtype=op.dtype, m=op.m, n=op.n, k=op.k,
                      m_lo=op.m_range[0], m_hi=op.m_range[1], n_lo=op.n_range[0], n_hi=op.n_range[1],
                      k_lo=op.k_range[0], k_hi=op.k_range[1], c_in=op.c_in, c_out=op.c_out, r=op.r, s=op.s,
                      stride=op.stride, pad=op.pad,
                      out_dtype=ft.FT_OUT_SAME if op.out_bytes == 2 else ft.FT_OUT_F32, batch_hi=op.batch_hi,
                      b_layout=ft.FT_B_NK if op.b_nk else ft.FT_B_KN)
    return ft.ft_op_register(d)


OPS = {
    "dense768": P.Op(P.OP_MATMUL, P.F16, n=768, k=768, m_range=(0, 8192)),
    "dense3072": P.Op(P.OP_MATMUL, P.F16, n=3072, k=768, m_range=(0, 8192)),
    "dense768k3072": P.Op(P.OP_MATMUL, P.F16, n=768, k=3072, m_range=(0, 8192)),
    "llm11008": P.Op(P.OP_MATMUL, P.BF16, n=11008, k=4096, m_range=(1, 8192)),
    "llm4096": P.Op(P.OP_MATMUL, P.BF16, n=4096, k=4096, m_range=(1, 8192)),
    "qk": P.Op(P.OP_BMM, P.F16, k=64, m_range=(0, 512), n_range=(0, 512)),
    "qk_b768": P.Op(P.OP_BMM, P.F16, k=64, m_range=(0, 512), n_range=(0, 512), batch_hi=768),
    "pv": P.Op(P.OP_BMM, P.F16, n=64, m_range=(0, 512), k_range=(0, 512)),
    "onlyn": P.Op(P.OP_BMM, P.F16, m=64, k=64, n_range=(1, 512)),
    "conv": P.Op(P.OP_CONV2D, P.F16, c_in=64, c_out=128, r=3, s=3, stride=1, pad=1, m_range=(0, 1 << 22)),
    "qk_nk": P.Op(P.OP_BMM, P.F16, k=64, m_range=(0, 512), n_range=(0, 512), batch_hi=768, b_nk=True),
    "dense768_nk": P.Op(P.OP_MATMUL, P.F16, n=768, k=768, m_range=(0, 8192), b_nk=True),
    "odd_static_n": P.Op(P.OP_MATMUL, P.F16, n=1000, k=100, m_range=(1, 4096)),
    "dense3072_out16": P.Op(P.OP_MATMUL, P.F16, n=3072, k=768, m_range=(0, 8192), out_bytes=2),
    "tiny_k": P.Op(P.OP_MATMUL, P.BF16, n=304, k=12, m_range=(0, 1024)),
}


def teams_on():
    lt = ft.ft_tuning_default()
    lt.two_team_bodies = 1
    return lt, dict(P.default_tuning(), two_team_bodies=1)


TEAM_OPS = ["dense768+teams", "dense3072+teams", "dense768k3072+teams", "llm4096+teams", "conv+teams", "tiny_k+teams", "qk+teams"]


@pytest.mark.parametrize("name", sorted(OPS) + TEAM_OPS)
def test_ukernel_table_matches_oracle(name):
    lib_t, ora_t = (None, None)
    if name.endswith("+teams"):
        name = name[:-len("+teams")]
        lib_t, ora_t = teams_on()
    op = OPS[name]
    want = P.derive_ukernels(op, t=ora_t)
    lop = to_lib_op(op)
    s = ft.ft_ukernels_derive(lop, None, lib_t)
    if lib_t is not None:       # two-team uKernels: Matmul and Conv2d with at least four k-tiles, never batched Matmul
        assert any(w.gk == 2 for w in want) == (op.kind != P.OP_BMM and op.k_ref() > 192)
    assert ft.ft_ukset_size(s) == len(want)
    for i, w in enumerate(want):
        g = ft.ft_ukset_get(s, i)
        got = (g.id, g.tm, g.tn, g.tk, g.wm, g.wn, g.gm, g.gn, g.gk, g.mfma, g.stages, g.lds_bytes, g.acc_regs,
               g.regs, g.reg_budget, g.max_wg_per_cu, g.cmr_q20, g.cmr_shared_q20)
        assert got == (w.id, w.tm, w.tn, w.tk, w.wm, w.wn, w.gm, w.gn, w.gk, w.mfma, w.stages, w.lds_bytes,
                       w.acc_regs, w.regs, w.reg_budget, w.max_wg_per_cu, w.cmr_q, w.cmr2_q)


def shapes_for(name):
    if name in ("qk", "qk_b768", "qk_nk"):
        return [dict(batch=b, m=L, n=L) for b in (1, 12, 96) for L in (1, 7, 16, 33, 77, 100, 257, 512)] + \
               [dict(batch=768, m=L, n=L) for L in (133, 141, 183, 281, 313, 390, 415, 450)] + \
               [dict(batch=96, m=313, n=200), dict(batch=96, m=200, n=313), dict(batch=96, m=133, n=281), dict(batch=96, m=313, n=415)] + \
               [dict(batch=3, m=100, n=40), dict(batch=3, m=40, n=100), dict(batch=0, m=5, n=5), dict(batch=2, m=0, n=0)]
    if name == "pv":
        return [dict(batch=b, m=L, k=L) for b in (1, 12) for L in (1, 7, 16, 33, 77, 100, 257, 512)]
    if name == "onlyn":
        return [dict(batch=2, n=L) for L in (1, 15, 16, 17, 77, 500)]
    if name == "conv":
        return [dict(img_n=8, img_h=h, img_w=h) for h in (1, 5, 28, 37, 56, 91)] + [dict(img_n=2, img_h=9, img_w=13)]
    ms = [1, 2, 15, 16, 17, 31, 32, 33, 77, 80, 100, 128, 272, 528, 1000, 1024, 1232, 1600, 2048, 4095, 8192]
    if name.startswith("dense"):
        ms = [0] + ms
    if name == "odd_static_n":
        ms = [1, 77, 1000, 4096]
    if name == "llm4096":
        ms = [1, 16, 45, 128, 300, 512, 1024, 2048, 8192]
    if name == "tiny_k":
        ms = [1, 77, 543, 1024]
    return [dict(m=m) for m in ms]


def oracle_shape(op, kw):
    return P.resolve_shape(op, batch=kw.get("batch", 1), m=kw.get("m", 0), n=kw.get("n", 0), k=kw.get("k", 0),
                           img_n=kw.get("img_n", 0), img_h=kw.get("img_h", 0), img_w=kw.get("img_w", 0))


def strips_on():
    """(library tuning, oracle tuning) with the second-axis strips switched on (off by default)."""
    lt = ft.ft_tuning_default()
    lt.second_axis_strips = 1
    return lt, dict(P.default_tuning(), second_axis_strips=1)


@pytest.mark.parametrize("mode", [P.PLAN_PATCHWORK, P.PLAN_PAD_BASELINE])
@pytest.mark.parametrize("name", sorted(OPS) + ["qk_b768+strips"] + TEAM_OPS)
def test_plans_bit_identical_to_oracle(name, mode):
    lib_t, ora_t = (None, None)
    if name.endswith("+strips"):
        name = name[:-len("+strips")]
        lib_t, ora_t = strips_on()
    if name.endswith("+teams"):
        name = name[:-len("+teams")]
        lib_t, ora_t = teams_on()
    op = OPS[name]
    uks = P.derive_ukernels(op, t=ora_t)
    lop = to_lib_op(op)
    s = ft.ft_ukernels_derive(lop, None, lib_t)
    for kw in shapes_for(name):
        shape = oracle_shape(op, kw)
        if op.kind != P.OP_BMM:
            shape = (1,) + tuple(shape[1:])
        want = P.plan(op, uks, shape, mode, t=ora_t)
        pl = ft.ft_plan_create(lop, s, ft.ft_shape(**kw), mode | HOST)
        got = ft.ft_plan_descriptors(pl)
        assert got == b"".join(d.pack() for d in want.descs), (name, kw)
        st = ft.ft_plan_stats_get(pl)
        assert (st.batch, st.m, st.n, st.k) == tuple(shape) and st.tau == want.tau
        assert st.n_tiles == len(want.descs) and st.useful_elems == want.useful
        if want.program is None:
            assert st.n_ukernels == 0
            continue
        pr = want.program
        assert st.covered_elems == want.covered
        assert st.n_ukernels == len(pr.parts)
        assert [(st.ukernel_id[i], st.count_tau[i]) for i in range(st.n_ukernels)] == list(pr.parts)
        assert (st.pad_q20, st.occ_q20, st.cmr_q20, st.sia_q20) == (pr.pad_q, pr.occ_q, pr.cmr_q, pr.sia_q)
        assert st.block_bound == pr.block_bound and st.level == want.level and st.pool_size == want.pool_size
        used = [i for i, _ in pr.parts] + [sid for sid, _, _ in pr.strips if sid >= 0]
        assert st.lds_bytes == max(uks[i].lds_bytes for i in used)
        assert (st.k_parts, st.k_part_tiles) == (want.k_parts, want.k_part_tiles), (name, kw)
        # second-axis strips: per part (strip uKernel or none, own tiles across the other axis, strip tiles)
        Wp = P.ceil_by(shape[2] if want.tau == 0 else shape[1], 16)
        for i, (uid, _) in enumerate(pr.parts):
            sid, n_full, n_strip = pr.strips[i] if pr.strips else (-1, P.ceil_div(Wp, uks[uid].tn if want.tau == 0 else uks[uid].tm), 0)
            assert (st.strip_ukernel_id[i], st.main_tiles[i], st.strip_tiles[i]) == (sid if sid >= 0 else 0xFFFFFFFF, n_full, n_strip), (name, kw)
        # the kernels' closed form of the descriptors held for every workgroup of every plan without strips
        assert st.table_order == (1 if pr.strips else 0), (name, kw)
        slab = max(uks[i].tm * uks[i].tn for i, _ in pr.parts)
        assert st.workspace_bytes == (st.n_tiles * st.k_parts * slab * 4 if st.k_parts > 1 else 0)


def test_some_plans_carry_second_axis_strips():
    """The attention shapes of the bit-identity test include plans with strips on both main axes;
    such a plan is launched in table order."""
    op = OPS["qk_b768"]
    lop = to_lib_op(op)
    s = ft.ft_ukernels_derive(lop, None, strips_on()[0])
    s_default = ft.ft_ukernels_derive(lop)
    seen = set()
    for kw in shapes_for("qk_b768"):
        if kw.get("batch", 1) == 0 or kw["m"] == 0:
            continue
        pl = ft.ft_plan_create(lop, s, ft.ft_shape(**kw), HOST)
        st = ft.ft_plan_stats_get(pl)
        has = any(st.strip_ukernel_id[i] != 0xFFFFFFFF for i in range(2))
        seen.add((st.tau, has))
        off = ft.ft_plan_stats_get(ft.ft_plan_create(lop, s_default, ft.ft_shape(**kw), HOST))
        assert all(off.strip_ukernel_id[i] == 0xFFFFFFFF for i in range(2))         # off unless asked for
        if has:
            # table order in chunks of 16 descriptors per XCD; idle workgroups pad the last round
            order = ft.ft_plan_launch_order(pl)
            assert len(order) % (8 * 16) == 0 and len(order) - st.n_tiles < 8 * 16
            busy = [t for t in order if t != 0xFFFFFFFF]
            assert sorted(busy) == list(range(st.n_tiles))
            for b, t in enumerate(order):
                want_t = ((b // 8 // 16) * 8 + b % 8) * 16 + (b // 8) % 16
                assert t == (want_t if want_t < st.n_tiles else 0xFFFFFFFF)
    assert (0, True) in seen and (1, True) in seen and (0, False) in seen


def test_some_plans_split_the_reduce_axis_like_the_oracle():
    """The shapes of the bit-identity test above include plans with k_parts > 1 (few tiles, long
    reduce axis) and the switch that turns the rescue off is honoured."""
    seen = set()
    for name in ("dense768k3072", "llm4096", "dense768"):
        op = OPS[name]
        uks = P.derive_ukernels(op)
        lop = to_lib_op(op)
        s = ft.ft_ukernels_derive(lop)
        t_off = ft.ft_tuning_default()
        t_off.k_parts_max = 1
        s_off = ft.ft_ukernels_derive(lop, None, t_off)
        for kw in shapes_for(name):
            if kw["m"] == 0:
                continue
            st = ft.ft_plan_stats_get(ft.ft_plan_create(lop, s, ft.ft_shape(**kw), HOST))
            want = P.plan(op, uks, (1,) + tuple(oracle_shape(op, kw)[1:]))
            assert st.k_parts == want.k_parts
            seen.add((name, st.k_parts > 1))
            off = ft.ft_plan_stats_get(ft.ft_plan_create(lop, s_off, ft.ft_shape(**kw), HOST))
            assert off.k_parts == 1 and off.workspace_bytes == 0
    assert ("dense768k3072", True) in seen and ("llm4096", True) in seen and ("dense768", True) not in seen


@pytest.mark.parametrize("name", ["dense768", "qk", "conv"])
def test_pool_scores_match_oracle(name):
    op = OPS[name]
    uks = P.derive_ukernels(op)
    lop = to_lib_op(op)
    s = ft.ft_ukernels_derive(lop)
    hw, t = P.default_hw(), P.default_tuning()
    cap = P.cmr_cap(uks)
    for kw in shapes_for(name)[:10]:
        b, M, N, K = oracle_shape(op, kw)
        if b == 0 or M == 0 or N == 0:
            continue
        tau = P.main_axis(op, M, N)
        Hp = P.ceil_by(M if tau == 0 else N, 16)
        want = P.build_pool([u.tm if tau == 0 else u.tn for u in uks], Hp, kinds=[P.eight_waves(u) for u in uks])
        got = ft.ft_plan_pool(lop, s, ft.ft_shape(**kw))
        assert len(got) == len(want)
        for g, parts in zip(got, want):
            p = P.evaluate(parts, uks, b, M, N, tau, hw, t, cap)
            k2 = parts[1][0] if len(parts) > 1 else 0xFFFFFFFF
            c2 = parts[1][1] if len(parts) > 1 else 0
            assert (g.k1, g.count1, g.k2, g.count2) == (parts[0][0], parts[0][1], k2, c2)
            assert (g.pad_q20, g.occ_q20, g.cmr_q20, g.sia_q20, g.n_tiles) == (p.pad_q, p.occ_q, p.cmr_q, p.sia_q, p.num_tiles)
            assert g.flags == (1 if p.in_bound else 0) | (2 if p.cross else 0) | (4 if p.saturated else 0)


def test_custom_tuning_and_hw_are_honoured():
    op = OPS["dense3072"]
    hw, t = P.default_hw(), P.default_tuning()
    hw2 = dict(hw, num_cus=80, bw_lds_bytes_per_clk_per_cu=128, ktile_latency_clk=0)
    t2 = dict(t, c0=1, c1=2, c2=6, zeta=1, rest_regs=96, psi_num=1, psi_den=5, sia_form=P.SIA_LINEAR)
    uks = P.derive_ukernels(op, hw2, t2)
    lhw = ft.ft_hw_default_gfx950(); lhw.num_cus = 80; lhw.bw_lds_bytes_per_clk_per_cu = 128
    lhw.ktile_latency_clk = 0
    lt = ft.ft_tuning_default(); lt.c1 = 2; lt.c2 = 6; lt.zeta = 1; lt.rest_regs = 96; lt.psi_den = 5
    lt.sia_form = ft.FT_SIA_LINEAR
    lop = to_lib_op(op)
    s = ft.ft_ukernels_derive(lop, lhw, lt)
    assert ft.ft_ukset_size(s) == len(uks)
    for M in (77, 528, 1232, 2048):
        want = P.plan(op, uks, (1, M, 3072, 768), hw=hw2, t=t2)
        pl = ft.ft_plan_create(lop, s, ft.ft_shape(m=M), HOST)
        assert ft.ft_plan_descriptors(pl) == b"".join(d.pack() for d in want.descs)


def test_product_form_with_exponents_matches_oracle():
    op = OPS["llm11008"]
    t2 = dict(P.default_tuning(), c0=2, c1=0, c2=3, sia_form=P.SIA_PRODUCT)
    uks = P.derive_ukernels(op, None, t2)
    lt = ft.ft_tuning_default(); lt.c0 = 2; lt.c1 = 0; lt.c2 = 3
    lop = to_lib_op(op)
    s = ft.ft_ukernels_derive(lop, None, lt)
    for M in (1, 45, 300, 1000, 4096, 8192):
        want = P.plan(op, uks, (1, M, 11008, 4096), t=t2)
        pl = ft.ft_plan_create(lop, s, ft.ft_shape(m=M), HOST)
        assert ft.ft_plan_descriptors(pl) == b"".join(d.pack() for d in want.descs)
        assert ft.ft_plan_stats_get(pl).sia_q20 == want.program.sia_q
    lt.c0 = 5
    with pytest.raises(ft.FtError) as e:
        ft.ft_ukernels_derive(lop, None, lt)
    assert e.value.status == ft.FT_ERR_INVALID_ARG


def test_forced_program_mode():
    op = OPS["dense768"]
    uks = P.derive_ukernels(op)
    lop = to_lib_op(op)
    s = ft.ft_ukernels_derive(lop)
    by = {(u.tm, u.tn, u.wm): u.id for u in uks}
    k1, k2 = by[(64, 64, 32)], by[(16, 64, 16)]
    pl = ft.ft_plan_create(lop, s, ft.ft_shape(m=77), ft.FT_PLAN_FORCED | HOST,
                           ft.ft_forced_program(k1=k1, count1=1, k2=k2, count2=1))
    want = P.emit([(k1, 1), (k2, 1)], uks, 1, 77, 768, 0)
    assert ft.ft_plan_descriptors(pl) == b"".join(d.pack() for d in want)
    with pytest.raises(ft.FtError) as e:
        ft.ft_plan_create(lop, s, ft.ft_shape(m=77), ft.FT_PLAN_FORCED | HOST,
                          ft.ft_forced_program(k1=k1, count1=2, k2=k2, count2=1))
    assert e.value.status == ft.FT_ERR_NO_COVER


def test_eight_wave_grids_are_for_plain_gemms_only():
    """Eight-wave grids (gm * gn = 8) have bodies for the plain GEMM walk only: a convolution or a batched
    operator gets none; a large dense operator gets the three tile shapes."""
    def grids(name):
        s = ft.ft_ukernels_derive(to_lib_op(OPS[name]))
        return {(u.tm, u.tn) for u in (ft.ft_ukset_get(s, i) for i in range(ft.ft_ukset_size(s))) if u.gm * u.gn == 8}
    assert grids("conv") == set() and grids("qk") == set() and grids("pv") == set()
    assert grids("llm4096") == {(256, 256), (128, 256), (256, 128)}
    assert {(u.tm, u.tn) for u in P.derive_ukernels(OPS["conv"]) if u.gm * u.gn == 8} == set()


def test_b_layout_of_an_operator():
    """FT_B_NK: Matmul and BMM only; the set holds four-wave standard grids only, like the oracle's."""
    with pytest.raises(ft.FtError) as e:
        ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_CONV2D, dtype=ft.FT_F16, c_in=64, c_out=128, r=3, s=3, stride=1, pad=1,
                                        m_lo=0, m_hi=1 << 22, b_layout=ft.FT_B_NK))
    assert e.value.status == ft.FT_ERR_INVALID_ARG
    with pytest.raises(ft.FtError) as e:
        ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=64, k=64, m_lo=0, m_hi=64, b_layout=2))
    assert e.value.status == ft.FT_ERR_INVALID_ARG
    for name in ("qk_nk", "dense768_nk"):
        s = ft.ft_ukernels_derive(to_lib_op(OPS[name]))
        us = [ft.ft_ukset_get(s, i) for i in range(ft.ft_ukset_size(s))]
        assert us and all(u.gk == 1 and u.gm * u.gn == 4 for u in us)


def test_launch_order_fetches_no_more_than_any_group_height():
    """Single-uKernel plans of the encoder sweep: the bytes the eight private L2s must fetch under the
    library's launch order (each XCD reads once the A row panels and B column panels of its tiles;
    workgroup b -> XCD b % 8, every XCD a contiguous run of the walk) are those of the best group
    height 1..16, found here by walking the tile grid with every height."""
    import synth_inputs as si
    dt = np.dtype([("uk", "<u4"), ("batch", "<u4"), ("m0", "<u4"), ("n0", "<u4"), ("mv", "<u2"), ("nv", "<u2"), ("flags", "<u4")])
    nx, checked = 8, 0
    sets = {}
    for M, N, K in si.config1_shapes():
        if (N, K) not in sets:
            lop = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=N, k=K, m_lo=1, m_hi=8192))
            sets[(N, K)] = (lop, ft.ft_ukernels_derive(lop))
        lop, s = sets[(N, K)]
        pl = ft.ft_plan_create(lop, s, ft.ft_shape(m=M), ft.FT_PLAN_PATCHWORK | HOST)
        desc = np.frombuffer(ft.ft_plan_descriptors(pl), dtype=dt)
        if len(set(desc["uk"].tolist())) != 1:
            continue
        n = len(desc)
        cols = len(set(desc["n0"].tolist()))
        rows = n // cols
        tm, tn = int(desc["mv"].max()), int(desc["nv"].max())
        if rows < 2 or cols < 2 or n > 8 * 32:        # (one round: all tiles of an XCD run together)
            continue

        def fetched(tiles_of_xcd):
            return sum(len({t // cols for t in ts}) * tm + len({t % cols for t in ts}) * tn for ts in tiles_of_xcd)

        order = ft.ft_plan_launch_order(pl)
        lib = fetched([[t for b, t in enumerate(order) if b % nx == x] for x in range(nx)])
        q, r = divmod(n, nx)
        best = None
        for g in range(1, min(16, rows) + 1):
            walk = []                                   # tile indices in the order of the grouped walk
            for first in range(0, rows, g):
                gr = min(g, rows - first)
                walk += [(first + w % gr) * cols + w // gr for w in range(gr * cols)]
            assert sorted(walk) == list(range(n))
            slices = [walk[x * q + min(x, r): x * q + min(x, r) + q + (1 if x < r else 0)] for x in range(nx)]
            f = fetched(slices)
            best = f if best is None else min(best, f)
        assert lib == best, (M, N, K, rows, cols, lib, best)
        checked += 1
    assert checked >= 8


def test_launch_order_is_a_balanced_permutation():
    """Every workgroup takes a distinct descriptor; each XCD (workgroup b -> XCD b % 8) gets an
    equal share (+-1) of EACH constituent's tiles, as contiguous slices of the table."""
    import struct
    cases = [("dense3072", 1232, None), ("dense3072", 1600, None), ("dense768", 77, None), ("qk", None, (8, 77, 77)),
             ("conv", None, None), ("llm11008", 300, None)]
    for name, m, bmm in cases:
        op = OPS[name]
        lop = to_lib_op(op)
        s = ft.ft_ukernels_derive(lop)
        if name == "conv":
            shape = ft.ft_shape(batch=2, img_h=37, img_w=37)
        elif bmm:
            shape = ft.ft_shape(batch=bmm[0], m=bmm[1], n=bmm[2])
        else:
            shape = ft.ft_shape(m=m)
        for mode in (ft.FT_PLAN_PATCHWORK, ft.FT_PLAN_PAD_BASELINE):
            pl = ft.ft_plan_create(lop, s, shape, mode | HOST)
            st = ft.ft_plan_stats_get(pl)
            order = ft.ft_plan_launch_order(pl)
            assert sorted(order) == list(range(st.n_tiles)), (name, mode)
            raw = ft.ft_plan_descriptors(pl)
            uk_of = [struct.unpack_from("<IIIIHHI", raw, 24 * i)[0] for i in range(st.n_tiles)]
            ids = sorted(set(uk_of))
            for uk in ids:
                per_xcd = [sum(1 for b, t in enumerate(order) if b % 8 == x and uk_of[t] == uk) for x in range(8)]
                assert max(per_xcd) - min(per_xcd) <= 1, (name, mode, uk, per_xcd)
                for x in range(8):
                    mine = sorted(t for b, t in enumerate(order) if b % 8 == x and uk_of[t] == uk)
                    # a slice of the constituent's block: walked in 2-D groups, so not sorted, but
                    # its tiles are exactly a contiguous run of the grouped sequence -> same count
                    assert len(mine) == per_xcd[x]
            # the larger constituent is started first inside every XCD
            if len(ids) == 2:
                first_uk = uk_of[0]
                for x in range(8):
                    seq = [uk_of[t] for b, t in enumerate(order) if b % 8 == x]
                    if first_uk in seq and seq.count(first_uk) < len(seq):
                        last_first = max(i for i, u in enumerate(seq) if u == first_uk)
                        assert all(u == first_uk for u in seq[:last_first + 1]), (name, x, seq)


def test_error_codes():
    lop = to_lib_op(OPS["dense768"])
    s = ft.ft_ukernels_derive(lop)
    with pytest.raises(ft.FtError) as e:
        ft.ft_plan_create(lop, s, ft.ft_shape(m=8193), HOST)
    assert e.value.status == ft.FT_ERR_OUT_OF_RANGE
    with pytest.raises(ft.FtError) as e:
        ft.ft_plan_create(lop, s, ft.ft_shape(m=5, n=512), HOST)       # static n contradicted
    assert e.value.status == ft.FT_ERR_INVALID_ARG
    bad = ft.ft_shape(m=5)
    bad.struct_size = 3
    with pytest.raises(ft.FtError) as e:
        ft.ft_plan_create(lop, s, bad, HOST)
    assert e.value.status == ft.FT_ERR_INVALID_ARG
    with pytest.raises(ft.FtError) as e:
        ft.ft_op_register(ft.ft_op_desc(kind=7))
    assert e.value.status == ft.FT_ERR_INVALID_ARG
    with pytest.raises(ft.FtError) as e:
        ft.ft_op_register(ft.ft_op_desc(kind=0, m_lo=5, m_hi=1, n=8, k=8))
    assert e.value.status == ft.FT_ERR_INVALID_ARG
    other = to_lib_op(OPS["dense3072"])
    with pytest.raises(ft.FtError) as e:
        ft.ft_plan_create(other, s, ft.ft_shape(m=5), HOST)              # set derived for another op
    assert e.value.status == ft.FT_ERR_INVALID_ARG
    # a hardware model whose LDS holds no tile leaves no uKernel
    hw = ft.ft_hw_default_gfx950(); hw.lds_bytes_per_cu = 1024
    with pytest.raises(ft.FtError) as e:
        ft.ft_ukernels_derive(lop, hw, None)
    assert e.value.status == ft.FT_ERR_NO_COVER
    assert ft.ft_status_string(ft.FT_ERR_NO_COVER) == "FT_ERR_NO_COVER"
    # host-only plans cannot be launched, and need no GPU to find that out
    pl = ft.ft_plan_create(lop, s, ft.ft_shape(m=16), HOST)
    with pytest.raises(ft.FtError) as e:
        ft.ft_launch(pl, 16, 16, 16, 0)
    assert e.value.status == ft.FT_ERR_INVALID_ARG


def test_limits_are_reported():
    """Shapes beyond the 32-bit offset arithmetic of the kernels are refused at plan time."""
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, k=64, m_lo=1, m_hi=64, n_lo=1, n_hi=1 << 21))
    s = ft.ft_ukernels_derive(op)
    with pytest.raises(ft.FtError) as e:
        ft.ft_plan_create(op, s, ft.ft_shape(batch=1, m=16, n=1 << 20), HOST)
    assert e.value.status == ft.FT_ERR_UNSUPPORTED
    ft.ft_plan_create(op, s, ft.ft_shape(batch=1, m=16, n=(1 << 20) - 16), HOST)


def test_batch_bound_of_a_batched_workload():
    """Without a batch bound the workload filters are skipped for BMM; with one, the tile count of
    the workload scales with it (a single 512 x 512 entry cannot fill the device with large tiles,
    768 of them can)."""
    full = P.derive_ukernels(P.Op(P.OP_BMM, P.F16, k=64, m_range=(1, 512), n_range=(1, 512)))
    one = P.derive_ukernels(P.Op(P.OP_BMM, P.F16, k=64, m_range=(1, 512), n_range=(1, 512), batch_hi=1))
    many = P.derive_ukernels(P.Op(P.OP_BMM, P.F16, k=64, m_range=(1, 512), n_range=(1, 512), batch_hi=768))
    key = lambda us: {(u.tm, u.tn, u.gk) for u in us}
    assert key(many) == key(full) and len(one) < len(full)
    assert (128, 128, 1) in key(many) and (128, 128, 1) not in key(one)
    for bh, want in ((0, full), (1, one), (768, many)):
        lop = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, k=64, m_lo=1, m_hi=512, n_lo=1, n_hi=512, batch_hi=bh))
        s = ft.ft_ukernels_derive(lop)
        assert ft.ft_ukset_size(s) == len(want)


def test_plan_cache_returns_the_same_plan_per_shape_and_flags():
    op = OPS["dense768"]
    lop = to_lib_op(op)
    s = ft.ft_ukernels_derive(lop)
    a = ft.ft_plan_cached(lop, s, ft.ft_shape(m=1232), HOST)
    b = ft.ft_plan_cached(lop, s, ft.ft_shape(m=1232), HOST)
    c = ft.ft_plan_cached(lop, s, ft.ft_shape(m=1233), HOST)
    d = ft.ft_plan_cached(lop, s, ft.ft_shape(m=1232), HOST | ft.FT_PLAN_PAD_BASELINE)
    assert a.ptr == b.ptr and len({a.ptr, c.ptr, d.ptr}) == 3
    fresh = ft.ft_plan_create(lop, s, ft.ft_shape(m=1232), HOST)
    assert ft.ft_plan_descriptors(a) == ft.ft_plan_descriptors(fresh)
    sa, sf = ft.ft_plan_stats_get(a), ft.ft_plan_stats_get(fresh)
    assert (sa.n_tiles, sa.sia_q20, sa.k_parts) == (sf.n_tiles, sf.sia_q20, sf.k_parts)
    with pytest.raises(ft.FtError):                      # forced programs are not cached
        ft.ft_plan_cached(lop, s, ft.ft_shape(m=1232), HOST | ft.FT_PLAN_FORCED)
    with pytest.raises(ft.FtError):                      # errors of ft_plan_create pass through, nothing is cached
        ft.ft_plan_cached(lop, s, ft.ft_shape(m=9000), HOST)
    # many threads asking for the same new shape get one plan
    import threading
    got = []
    def ask():
        got.append(ft.ft_plan_cached(lop, s, ft.ft_shape(m=777), HOST).ptr)
    th = [threading.Thread(target=ask) for _ in range(8)]
    [t.start() for t in th]
    [t.join() for t in th]
    assert len(set(got)) == 1


def _random_ops(n=90, seed=515):
    """Seeded random operators of the three kinds with a few runtime shapes each (static extents from
    tiny to LLM sized, 16-bit outputs, strips on for some batched ones)."""
    import random
    rnd = random.Random(seed)
    ext = [1, 2, 5, 8, 12, 16, 24, 40, 64, 100, 128, 304, 768, 1000, 1536, 4096, 11008]
    out = []
    for i in range(n):
        kind = rnd.choice([P.OP_MATMUL, P.OP_MATMUL, P.OP_BMM, P.OP_BMM, P.OP_CONV2D])
        dt, ob = rnd.choice([P.F16, P.BF16]), rnd.choice([4, 4, 2])
        strips = False
        if kind == P.OP_MATMUL:
            lo, hi = rnd.choice([0, 1]), rnd.choice([64, 1024, 8192])
            op = P.Op(kind, dt, n=rnd.choice(ext), k=rnd.choice(ext), m_range=(lo, hi), out_bytes=ob)
            shapes = [dict(m=rnd.randint(lo, hi)) for _ in range(3)]
        elif kind == P.OP_BMM:
            which, bh = rnd.choice(["qk", "pv", "all"]), rnd.choice([0, 12, 768])
            strips = rnd.random() < 0.4
            kw = dict(m_range=(0, 512), batch_hi=bh, out_bytes=ob)
            if which == "qk":
                kw.update(k=rnd.choice([16, 64, 128]), n_range=(0, 512))
            elif which == "pv":
                kw.update(n=rnd.choice([16, 64, 128]), k_range=(0, 512))
            else:
                kw.update(n_range=(0, 512), k_range=(0, 512))
            op = P.Op(kind, dt, **kw)
            shapes = []
            for _ in range(3):
                L = rnd.randint(0, 512)
                sh = dict(batch=rnd.randint(0, bh or 96), m=L)
                if which != "pv":
                    sh["n"] = rnd.choice([L, rnd.randint(0, 512)])
                if which != "qk":
                    sh["k"] = rnd.choice([L, rnd.randint(0, 512)])
                shapes.append(sh)
        else:
            r, pad = rnd.choice([1, 3, 5]), rnd.choice([0, 1, 2])
            op = P.Op(kind, dt, c_in=rnd.choice([3, 8, 12, 64, 72]), c_out=rnd.choice([1, 8, 100, 128]), r=r, s=r,
                      stride=rnd.choice([1, 2]), pad=pad, m_range=(0, 1 << 20), out_bytes=ob)
            lo = max(1, r - 2 * pad)
            shapes = [dict(img_n=rnd.randint(1, 8), img_h=rnd.randint(lo, 60), img_w=rnd.randint(lo, 60)) for _ in range(3)]
        out.append((i, op, shapes, strips))
    return out


@pytest.mark.parametrize("case", _random_ops(), ids=lambda c: "r%d_kind%d" % (c[0], c[1].kind))
def test_random_operators_match_the_oracle(case):
    """uKernel table and descriptor table of the library equal the oracle's, field by field and byte
    by byte, for operators and shapes nobody picked by hand."""
    _, op, shapes, strips = case
    lib_t, ora_t = strips_on() if strips else (None, None)
    uks = P.derive_ukernels(op, t=ora_t)
    lop = to_lib_op(op)
    s = ft.ft_ukernels_derive(lop, None, lib_t)
    assert ft.ft_ukset_size(s) == len(uks)
    for i, w in enumerate(uks):
        g = ft.ft_ukset_get(s, i)
        assert (g.tm, g.tn, g.gk, g.stages, g.max_wg_per_cu, g.cmr_q20, g.cmr_shared_q20) == \
               (w.tm, w.tn, w.gk, w.stages, w.max_wg_per_cu, w.cmr_q, w.cmr2_q)
    for kw in shapes:
        shape = oracle_shape(op, kw)
        if op.kind != P.OP_BMM:
            shape = (1,) + tuple(shape[1:])
        want = P.plan(op, uks, shape, t=ora_t)
        pl = ft.ft_plan_create(lop, s, ft.ft_shape(**kw), HOST)
        assert ft.ft_plan_descriptors(pl) == b"".join(d.pack() for d in want.descs), kw
        st = ft.ft_plan_stats_get(pl)
        assert st.n_tiles == len(want.descs)
        if want.program is not None:
            assert (st.sia_q20, st.k_parts, st.k_part_tiles) == (want.program.sia_q, want.k_parts, want.k_part_tiles), kw


# ---- grouped plans: one launch over groups of different shapes (Sec. 1 / Fig. 1(b): ragged batches) ----
GROUPED = {
    "qk": (OPS["qk_b768"], [dict(batch=12, m=L, n=L) for L in (77, 5, 128, 0, 257, 33, 100, 512)]),
    "pv": (OPS["pv"], [dict(batch=12, m=L, k=L) for L in (77, 5, 128, 257, 1, 100)]),
    "one": (OPS["qk"], [dict(batch=3, m=100, n=40)]),
}


@pytest.mark.parametrize("mode", [P.PLAN_PATCHWORK, P.PLAN_PAD_BASELINE])
@pytest.mark.parametrize("name", sorted(GROUPED))
def test_grouped_plan_is_the_concatenation_of_the_groups_plans(name, mode):
    """Descriptor table = the oracle's plans of the groups one after the other (heaviest first), each descriptor tagged
    with its group (flags bits 12..31; bits 1..11 name the compiled body and its ring depth and are the
    library's own);
    operands packed group after group."""
    op, groups = GROUPED[name]
    uks = P.derive_ukernels(op)
    lop = to_lib_op(op)
    s = ft.ft_ukernels_derive(lop)
    pl = ft.ft_plan_create_grouped(lop, s, [ft.ft_shape(**kw) for kw in groups], mode | HOST)
    got = np.frombuffer(ft.ft_plan_descriptors(pl), dtype=np.dtype(
        [("uk", "<u4"), ("batch", "<u4"), ("m0", "<u4"), ("n0", "<u4"), ("mv", "<u2"), ("nv", "<u2"), ("flags", "<u4")]))
    shapes = [oracle_shape(op, kw) for kw in groups]
    table, offsets = P.plan_grouped(op, uks, shapes, mode)
    for gi in range(len(groups) + 1):
        assert ft.ft_plan_group_layout(pl, gi) == offsets[gi], (name, gi)
    assert len(got) == len(table)
    ref = np.frombuffer(b"".join(d.pack() for _, d in table), dtype=got.dtype)
    for f in ("uk", "batch", "m0", "n0", "mv", "nv"):
        assert (got[f] == ref[f]).all(), (name, f)
    assert ((got["flags"] & 1) == (ref["flags"] & 1)).all()
    assert (got["flags"] >> 12).tolist() == [g for g, _ in table]
    at = len(table)
    useful = sum(b * m * n for b, m, n, k in shapes)
    st = ft.ft_plan_stats_get(pl)
    tile_area = {u.id: u.tm * u.tn for u in uks}
    covered = sum(tile_area[d.ukernel_id] for _, d in table)
    assert (st.n_tiles, st.useful_elems, st.covered_elems, st.k_parts, st.table_order) == (at, useful, covered, 1, 1)
    order = ft.ft_plan_launch_order(pl)
    assert sorted(t for t in order if t != 0xFFFFFFFF) == list(range(at))


def test_grouped_plan_argument_checks():
    lop = to_lib_op(OPS["qk"])
    s = ft.ft_ukernels_derive(lop)
    with pytest.raises(ft.FtError) as e:                       # a Matmul operator has no groups
        mm = to_lib_op(OPS["dense768"])
        ft.ft_plan_create_grouped(mm, ft.ft_ukernels_derive(mm), [ft.ft_shape(m=5)], HOST)
    assert e.value.status == ft.FT_ERR_UNSUPPORTED
    with pytest.raises(ft.FtError) as e:                       # a group outside the registered range
        ft.ft_plan_create_grouped(lop, s, [ft.ft_shape(batch=1, m=5, n=5), ft.ft_shape(batch=1, m=513, n=5)], HOST)
    assert e.value.status == ft.FT_ERR_OUT_OF_RANGE
    with pytest.raises(ft.FtError):                            # forced programs are per shape
        ft.ft_plan_create_grouped(lop, s, [ft.ft_shape(batch=1, m=5, n=5)], ft.FT_PLAN_FORCED | HOST)
    empty = ft.ft_plan_create_grouped(lop, s, [], HOST)
    assert ft.ft_plan_stats_get(empty).n_tiles == 0 and ft.ft_plan_group_layout(empty, 0) == (0, 0, 0)
    with pytest.raises(ft.FtError):
        ft.ft_plan_group_layout(empty, 1)
