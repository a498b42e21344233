"""Planner oracle (TEST INFRASTRUCTURE ONLY): uKernel-set derivation and runtime covering.

Pure Python, integers only (Python ints are unbounded, so nothing can overflow), written
from the paper's algorithms in the paper's order and notation:

  * uKernel data structure: reg_tile, smem_tile, padding_threshold (Pad), usage_eff (Occ),
    compute_eff (CMR)                                        -- Fig. 6 caption, Table 1
  * HardwareAlign / RegTileRule / SmemTileRule                -- Sec. 4.1, Alg. 1
  * mem.IsOverflow, Eq. 4 (register bound, block.bound)       -- Sec. 4.2, Alg. 1
  * Pad (Eq. 2), Occ (Eq. 3), CrossPick epsilon/lambda sweep  -- Sec. 4.2
  * space-axis saturation (Eq. 5), compute_eff (Eq. 6, 7)     -- Sec. 4.3
  * CombinSearch on the main axis tau (Alg. 2)                -- Sec. 5.1
  * SIA score (Eq. 1), Top-1                                  -- Sec. 5.2

The paper's device is an NVIDIA GPU with fp32 CUDA cores; here its terms are re-based on
gfx950 resources (CU, wave64, LDS, unified VGPR/AGPR file, MFMA shapes).  The readings
taken where the paper is silent or loose are listed next to each function.

Shares no code with the GPU library.  Fixed-point scores are floor(x * 2**20) of exact
rationals so that a second implementation can reproduce every decision bit for bit.
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

Q = 20                      # fixed-point fraction bits of the cached metrics
ONE = 1 << Q
GRANULE = 16                # smallest MFMA output extent on gfx950 (16x16x32)

OP_MATMUL, OP_BMM, OP_CONV2D = 0, 1, 2
F16, BF16 = 0, 1
PLAN_PATCHWORK, PLAN_PAD_BASELINE = 0, 1
SIA_LINEAR, SIA_PRODUCT = 0, 1


def default_hw():
    """Hardware description 'script' (Sec. 8): bandwidth per memory level, clock, cores."""
    return dict(num_cus=256, simds_per_cu=4, wave_size=64, regs_per_lane=512,
                max_waves_per_simd=8, lds_bytes_per_cu=163840, clock_mhz=2400,
                mfma_flops_per_clk_per_cu=4096, bw_global_bytes_per_clk_per_cu=64,
                bw_lds_bytes_per_clk_per_cu=256, ktile_latency_clk=400, solo_copy_exposed_pct=50,
                part_exchange_clk=2000,
                part_exchange_bytes_per_clk=16, phase_latency_clk=150,
                hbm_gbytes_per_s=8000, num_xcds=8)


def default_tuning():
    """Hyper-parameters (Sec. 4.2: epsilon 50%..95% step 1%, lambda 95%..90% step 0.1%,
    zeta = 2; Sec. 5.2: c0 = c1 = c2 = 1).  Per-mille units; psi is never given a value in
    the paper, 1/64 here."""
    return dict(eps_min_pm=500, eps_max_pm=950, eps_step_pm=10,
                lam_max_pm=950, lam_min_pm=900, lam_step_pm=1,
                zeta=2, rest_regs=72, psi_num=1, psi_den=64, c0=1, c1=1, c2=1, sia_form=SIA_PRODUCT,
                k_parts_max=8, k_part_min_tiles=8, second_axis_strips=0, two_team_bodies=1)


# --------------------------------------------------------------------------------------
# small closed-form pieces
# --------------------------------------------------------------------------------------
def ceil_div(a, b):
    return -((-a) // b)


def ceil_by(x, m):
    """ceil_by of Eq. 3: x rounded up to a multiple of m."""
    return m * ceil_div(x, m)


def occ_fraction(num_tiles, slots):
    """Eq. 3 as an exact fraction (numerator, denominator): (wkl/K) / ceil_by(wkl/K, slots)."""
    return num_tiles, ceil_by(num_tiles, slots)


def pad_fraction(base, padded_total):
    """Eq. 2 as an exact fraction: base / (pad + base), both counted in multiply-accumulates
    per unit of the reduce axis (the reduce extent is common to numerator and denominator)."""
    return base, padded_total


def sweep_points(t):
    """Lock-step epsilon/lambda staircase of CrossPick (Alg. 1, 'Forward' = one stride of
    both): starts at (eps_min, lam_max), stops when either bound is passed."""
    pts = []
    eps, lam = t["eps_min_pm"], t["lam_max_pm"]
    while eps <= t["eps_max_pm"] and lam >= t["lam_min_pm"]:
        pts.append((eps, lam))
        eps += t["eps_step_pm"]
        lam -= t["lam_step_pm"]
    return pts


def cross_pick(pad, occ, t):
    """CrossPick test for one candidate: kept iff at some step of the staircase
    K.pad >= eps_i and K.occ >= lam_j (exact integer comparison of fractions)."""
    pn, pd = pad
    on, od = occ
    for eps, lam in sweep_points(t):
        if 1000 * pn >= eps * pd and 1000 * on >= lam * od:
            return True
    return False


def factors(n):
    return [d for d in range(1, n + 1) if n % d == 0]


def reg_tile_rule_factors(length):
    """RegTileRule as printed (Sec. 4.1): all factors of the dynamic-axis length; for a
    prime length the factors of the two neighbours instead.  On gfx950 the register tile
    is a multiple of an MFMA shape, so this form survives only for its worked example."""
    def is_prime(n):
        return n > 1 and all(n % d for d in range(2, int(n ** 0.5) + 1))
    if is_prime(length):
        return sorted(set(factors(length - 1)) | set(factors(length + 1)))
    return factors(length)


def combin_search(H, extents, trace=None):
    """Alg. 2 on bare main-axis extents, paper form (first success): for each K1 in set
    order, a single-uKernel program if K1 divides H; otherwise H is reduced by K1 once per
    search round until some other extent K2 divides what is left:
        H = Num1*K1 + Num2*K2.
    Returns a list of programs [(K1, Num1)] or [(K1, Num1), (K2, Num2)], one per K1 that
    admits one (first K2 in set order).  trace, if a list, receives (K1, H) for every
    reduced H the search visits."""
    progs = []
    for k1 in extents:
        if H % k1 == 0:
            progs.append([(k1, H // k1)])
            continue
        left, n1 = H, 0
        found = None
        while left - k1 > 0 and found is None:
            left -= k1
            n1 += 1
            if trace is not None:
                trace.append((k1, left))
            for k2 in extents:
                if k2 != k1 and left % k2 == 0:
                    found = [(k1, n1), (k2, left // k2)]
                    break
        if found:
            progs.append(found)
    return progs


# --------------------------------------------------------------------------------------
# uKernel set (compile stage, Sec. 4)
# --------------------------------------------------------------------------------------
@dataclass
class UKernel:
    tm: int
    tn: int
    tk: int
    wm: int          # reg_tile: per-wave accumulator tile
    wn: int
    gm: int          # wave grid inside the workgroup: rows, columns, reduce axis
    gn: int
    gk: int
    mfma: int        # 0 = 32x32x16, 1 = 16x16x32
    stages: int
    lds_bytes: int
    acc_regs: int
    regs: int
    reg_budget: int  # register allocation of the kernel the body is compiled into
    max_wg_per_cu: int
    cmr_q: int       # compute_eff alone on its CU, floor(x * 2^20)
    cmr2_q: int      # compute_eff when two or more workgroups share the CU
    id: int = -1


@dataclass
class Op:
    kind: int
    dtype: int
    # GEMM view; a static extent is > 0, a dynamic one is 0 with its [lo, hi] range
    m: int = 0
    n: int = 0
    k: int = 0
    m_range: Tuple[int, int] = (1, 1)
    n_range: Tuple[int, int] = (1, 1)
    k_range: Tuple[int, int] = (1, 1)
    # conv only (NHWC, RSCK)
    c_in: int = 0
    c_out: int = 0
    r: int = 0
    s: int = 0
    stride: int = 1
    pad: int = 0
    out_bytes: int = 4   # bytes per output element: fp32, or 2 when C has the inputs' 16-bit type
    batch_hi: int = 0    # BMM: largest batch count of the workload (the batch itself is a runtime
                         # value); 0 = unknown: the workload filters cannot be evaluated and are skipped
    b_nk: bool = False   # operand B stored as [N][K] (k contiguous): four-wave standard grids only

    def gemm_static(self):
        if self.kind == OP_CONV2D:
            return 0, self.c_out, self.r * self.s * self.c_in
        return self.m, self.n, self.k

    def k_ref(self):
        _, _, k = self.gemm_static()
        return k if k > 0 else self.k_range[1]


def wave_tiles():
    """RegTileRule on gfx950: per-wave accumulator tiles are power-of-two multiples of an
    MFMA output shape, at most 128 on a side.  Rows of 16 use the 16x16x32 instruction
    (columns up to 64); everything else the 32x32x16 one with aspect ratio within 2."""
    out = []
    sizes = (16, 32, 64, 128)
    for wm in sizes:
        for wn in sizes:
            if wm == 16 and wn <= 64:
                out.append((wm, wn, 1))
            elif wm >= 32 and wn >= 32 and wm <= 2 * wn and wn <= 2 * wm:
                out.append((wm, wn, 0))
    return out


# four wave64 per workgroup, one per SIMD, arranged over (rows, columns, reduce axis); in the
# split-k grid every wave owns the whole tile and a quarter of k.  gk = 2: the standard grids again
# with eight waves, two teams of four (two waves per SIMD) that take alternate k-tiles of the tile
# (tuning two_team_bodies; Matmul and Conv2d): while one team runs its MFMAs the other copies.
# gm * gn = 8 (gk = 1): eight waves, two per SIMD, on the same k-tiles -- the largest tiles at half the
# accumulator registers per wave; compiled for the wave tiles in EIGHT_WAVE_FAMILY only.
WAVE_GRIDS = ((1, 4, 1), (2, 2, 1), (4, 1, 1), (1, 1, 4), (1, 4, 2), (2, 2, 2), (4, 1, 2), (2, 4, 1), (4, 2, 1))
EIGHT_WAVE_FAMILY = {(128, 64, 2, 4), (64, 128, 4, 2), (64, 64, 2, 4), (64, 64, 4, 2)}      # (wm, wn, gm, gn)


def eight_waves(u):
    """Workgroups of eight waves (two teams, or an eight-wave grid) run in kernels of their own: the
    uKernels of one launch are all of one kind."""
    return u.gk == 2 or u.gm * u.gn == 8
TWO_TEAM_STAGE_MAX = 40960                  # both teams' rings of two stages fit the LDS
TWO_TEAM_ACC_MAX = 64                       # accumulator registers per lane of a two-team wave
TK_CHOICES = (64,)                          # 64 16-bit elements = one 128-byte line
MIN_STAGES, MAX_STAGES = 2, 8
ELT = 2


def waves_bound(u):
    """What a uKernel offers against block.bound (Alg. 1: workgroups a CU should hold): its residency,
    doubled for an eight-wave grid, whose one workgroup already puts two waves on every SIMD.  A
    two-team workgroup also has eight waves, but its teams alternate on the k-tiles: it counts once."""
    return u.max_wg_per_cu * (2 if u.gm * u.gn == 8 else 1)


def compute_eff(tm, tn, gm, gn, k_ref, hw, gk=1, tk=64, residents=1, out_bytes=4, exchange_clk=0):
    """Eq. 6 / Eq. 7: (FLOPs / FLOPS) : K_mem, with K_mem read on gfx950 as the time the
    uKernel's k loop needs, so the ratio is the fraction of that time the MFMA pipes are busy.
    t_c = FLOPs / FLOPS, t_g = global bytes / bw_G, t_s = LDS bytes / bw_S (Eq. 7's data terms).
    A wave walks through nk_w = ceil(nk / gk) of the nk = ceil(K / tk) k-tiles (all of them in a
    standard grid, every gk-th in a split-k grid): the MFMA phase lasts t_ce = t_c * gk * nk_w / nk
    (= t_c unless a split-k grid leaves waves idle) and the loop pays t_l = ktile_latency_clk * nk_w.
      * residents >= 2 (workgroups sharing a CU, Alg. 1's block.bound): a SIMD holds several
        waves, copy, LDS and MFMA phases of different waves overlap:
            K_mem = max(t_ce, t_g, t_s) + t_l / residents
      * residents == 1: the one wave of a SIMD issues its global->LDS copies and its MFMAs
        itself; a fraction solo_copy_exposed_pct of the copy time is not hidden:
            K_mem = t_ce + exposed * t_g + t_l
      * an eight-wave grid (gm * gn == 8) alone on its CU: the two waves of a SIMD pass the
        workgroup's barriers together; they read their fragments at the same time (t_s at half the
        LDS rate), half of the solo share of the copy time stays exposed, and the k-tile latency
        is shared by the two waves but not hidden:
            K_mem = max(t_c, 2 t_s) + exposed / 2 * t_g + 2/3 t_l
      * two teams (gk == 2): a SIMD holds one wave of each team, copies and MFMAs of the two overlap
        and every k-tile ends with one barrier:
            K_mem = max(t_c, t_g, t_s) + phase_latency_clk * nk / residents
    exchange_clk: a fixed time added to K_mem (divided by residents like t_l): the round trips of
    a workgroup that hands its partial tile to the others of a reduce-axis split.
    Returns (numerator, denominator) of the exact ratio."""
    F, G, S = hw["mfma_flops_per_clk_per_cu"], hw["bw_global_bytes_per_clk_per_cu"], hw["bw_lds_bytes_per_clk_per_cu"]
    flops = 2 * tm * tn * k_ref
    gbytes = (tm + tn) * k_ref * ELT + tm * tn * out_bytes    # data_r + data_w
    sbytes = (tm + tn) * k_ref * ELT + k_ref * ELT * (tm * gn + tn * gm)   # data_tw + data_tr
    nk = ceil_div(k_ref, tk)
    r = residents
    if gm * gn == 8 and gk == 1 and residents < 2:
        # over the common denominator F * G * S * 600
        c8 = flops * G * S * 600
        return c8, (max(c8, sbytes * F * G * 1200) + gbytes * F * S * 3 * hw["solo_copy_exposed_pct"]
                    + (hw["ktile_latency_clk"] * nk + exchange_clk) * F * G * S * 400)
    if gk == 2:
        # over the common denominator F * G * S * r
        c2 = flops * G * S * r
        return c2, max(c2, gbytes * F * S * r, sbytes * F * G * r) + (hw["phase_latency_clk"] * nk + exchange_clk) * F * G * S
    nk_w = ceil_div(nk, gk)
    ed = 100
    # everything over the common denominator F * G * S * nk * r * ed
    c = flops * G * S * nk * r * ed
    ce = flops * G * S * gk * nk_w * r * ed
    lt = (hw["ktile_latency_clk"] * nk_w + exchange_clk) * F * G * S * nk * ed
    if r >= 2:
        g = gbytes * F * S * nk * r * ed
        s = sbytes * F * G * nk * r * ed
        return c, max(ce, g, s) + lt
    g = gbytes * F * S * nk * hw["solo_copy_exposed_pct"]
    return c, ce + g + lt


def reg_budget(regs, hw):
    """Registers are granted per wave in power-of-two fractions of the file that a whole
    number of waves can share: regs_per_lane / 4, / 2, / 1 (128, 256, 512 on gfx950).  The
    budget of a uKernel is the smallest such fraction holding reg_tile + RestRegs; it is
    the K.RegsInBlock / lanes of Eq. 4."""
    b = hw["regs_per_lane"] // 4
    while b < regs:
        b *= 2
    return b


def axis_samples(lo, hi, cap):
    """Shapes of the workload ('every possible shape', Sec. 4) along one dynamic axis: both ends
    of the registered range and the multiples of the granule between them, thinned to about cap
    points by a fixed stride."""
    lo = max(lo, 1)
    if hi < lo:
        return []
    pts = {lo, hi}
    first = ceil_by(lo, GRANULE)
    if first <= hi:
        n_mult = (hi - first) // GRANULE + 1
        stride = max(1, ceil_div(n_mult, cap)) * GRANULE
        pts.update(range(first, hi + 1, stride))
    return sorted(pts)


def workload_shapes(op: Op):
    """(M, N) pairs the compile stage evaluates a uKernel on."""
    m_s, n_s, _ = op.gemm_static()
    both = m_s == 0 and n_s == 0
    cap = 48 if both else 256
    ms = [m_s] if m_s else axis_samples(op.m_range[0], op.m_range[1], cap)
    ns = [n_s] if n_s else axis_samples(op.n_range[0], op.n_range[1], cap)
    return [(m, n) for m in ms for n in ns]


def passes_workload(tm, tn, shapes, hw, t, batch=1):
    """CrossPick (Alg. 1) and the space-axis test (Eq. 5) for one uKernel K over the workload:
    kept iff for some shape, composed of K alone (padding where K does not divide), K.pad and
    K.occ pass the staircase and the number of uKernels reaches Active Blocks = zeta x NumCores.
    SetBound's K.IsInBound depends on block.bound = min(K.wkl.block, zeta), which is known
    only per shape: it is applied at the runtime stage.  batch: the largest batch count of the
    workload (every batch entry is tiled alike, so it multiplies the number of uKernels)."""
    for M, N in shapes:
        T = batch * ceil_div(M, tm) * ceil_div(N, tn)
        if T < t["zeta"] * hw["num_cus"]:
            continue                                                # Eq. 5
        if cross_pick(pad_fraction(M * N, T * tm * tn), occ_fraction(T, hw["num_cus"]), t):
            return True
    return False


def derive_ukernels(op: Op, hw=None, t=None) -> List[UKernel]:
    """Compile stage: HardwareAlign, then the filters of Alg. 1 and Sec. 4.3 over the workload
    (IsOverflow, Eq. 4 at block.bound = 1, CrossPick, Eq. 5, Eq. 6), in the canonical set order: larger
    smem_tile area first.  If no uKernel survives the workload filters (ranges too small to
    ever fill the device), the set before them is kept; likewise Eq. 6's threshold psi is not applied
    when no uKernel reaches it (a reduce axis of a few elements: every loop is latency)."""
    hw = hw or default_hw()
    t = t or default_tuning()
    m_s, n_s, _ = op.gemm_static()
    k_ref = op.k_ref()
    shapes = workload_shapes(op)
    cand = []
    kept = []
    psi_ok = []
    for wm, wn, mfma in wave_tiles():
        for gm, gn, gk in WAVE_GRIDS:
            if op.b_nk and (gk != 1 or gm * gn != 4):
                continue
            if gk == 4 and not (256 <= wm * wn <= 4096):
                continue
            if gk == 2 and (not t.get("two_team_bodies", 0) or op.kind == OP_BMM or ceil_div(k_ref, TK_CHOICES[0]) < 4):
                continue                            # (each team wants at least two k-tiles)
            if gm * gn == 8 and (not t.get("two_team_bodies", 0) or op.kind != OP_MATMUL or (wm, wn, gm, gn) not in EIGHT_WAVE_FAMILY):
                continue
            waves_per_simd = 2 if (gk == 2 or gm * gn == 8) else 1    # 4 waves on 4 SIMDs, or 8
            for tk in TK_CHOICES:
                tm, tn = gm * wm, gn * wn
                if gk == 2 and ((tm + tn) * tk * ELT > TWO_TEAM_STAGE_MAX or wm * wn // 64 > TWO_TEAM_ACC_MAX):
                    continue
                # static space axes are divided evenly (after rounding to the MFMA granule,
                # the gfx950 form of "factors of the neighbours")
                if m_s > 0 and ceil_by(m_s, GRANULE) % tm:
                    continue
                if n_s > 0 and ceil_by(n_s, GRANULE) % tn:
                    continue
                # LDS ring depth: the k-tiles that fit in one workgroup's share of the LDS when
                # zeta workgroups are resident, between 2 and 8
                # (a split-k workgroup keeps one ring per wave and is meant to own the CU's LDS)
                stage_bytes = (tm + tn) * tk * ELT
                if gk == 1:
                    stages = (hw["lds_bytes_per_cu"] // t["zeta"]) // stage_bytes
                else:
                    stages = hw["lds_bytes_per_cu"] // (gk * stage_bytes)
                stages = max(MIN_STAGES, min(MAX_STAGES, stages))
                lds = gk * stages * stage_bytes
                if lds > hw["lds_bytes_per_cu"]:
                    continue                                        # mem.IsOverflow
                acc = wm * wn // hw["wave_size"]
                regs = acc + t["rest_regs"]
                if regs * waves_per_simd > hw["regs_per_lane"]:
                    continue                                        # Eq. 4, block.bound = 1
                budget = reg_budget(regs, hw)
                cn, cd = compute_eff(tm, tn, gm, gn, k_ref, hw, gk, tk, out_bytes=op.out_bytes)
                psi_ok.append(cn * t["psi_den"] >= t["psi_num"] * cd)          # Eq. 6
                cap = min(hw["lds_bytes_per_cu"] // lds, hw["regs_per_lane"] // budget // waves_per_simd,
                          hw["max_waves_per_simd"] // waves_per_simd)
                cn2, cd2 = compute_eff(tm, tn, gm, gn, k_ref, hw, gk, tk, residents=2, out_bytes=op.out_bytes)
                cand.append(UKernel(tm, tn, tk, wm, wn, gm, gn, gk, mfma, stages, lds, acc, regs,
                                    budget, cap, (cn << Q) // cd, (cn2 << Q) // cd2))
                if op.kind == OP_BMM:
                    # the tile count of a batched workload scales with a batch only known at run time
                    kept.append(op.batch_hi == 0 or passes_workload(tm, tn, shapes, hw, t, op.batch_hi))
                else:
                    kept.append(passes_workload(tm, tn, shapes, hw, t))
    if any(psi_ok):
        cand, kept = [u for u, ok in zip(cand, psi_ok) if ok], [k for k, ok in zip(kept, psi_ok) if ok]
    if any(kept):
        cand = [u for u, k in zip(cand, kept) if k]
    cand.sort(key=lambda u: (-(u.tm * u.tn), -u.tm, -u.tn, -u.tk, -u.wm, -u.wn, u.gk, -u.gm))
    for i, u in enumerate(cand):
        u.id = i
    return cand


# --------------------------------------------------------------------------------------
# runtime stage (Sec. 5)
# --------------------------------------------------------------------------------------
@dataclass
class Desc:
    ukernel_id: int
    batch: int
    m0: int
    n0: int
    m_valid: int
    n_valid: int
    flags: int

    def pack(self):
        import struct
        return struct.pack("<IIIIHHI", self.ukernel_id, self.batch, self.m0, self.n0,
                           self.m_valid, self.n_valid, self.flags)


@dataclass
class Program:
    parts: List[Tuple[int, int]]            # (ukernel id, count along tau), ascending id
    num_tiles: int = 0
    area: int = 0                           # sum of tm*tn over one batch entry's tiles
    block_bound: int = 1
    in_bound: bool = True
    cross: bool = False
    saturated: bool = False
    pad_q: int = 0
    occ_q: int = 0
    cmr_q: int = 0
    sia_q: int = 0
    k1: int = -1
    k2: int = -1
    k_parts: int = 1                        # workgroups per tile along the reduce axis
    # second-axis strips (two dynamic space axes): per part (strip ukernel id or -1, tiles of the
    # part's own uKernel across the other axis, tiles of the strip uKernel after them)
    strips: List[Tuple[int, int, int]] = field(default_factory=list)


@dataclass
class Plan:
    batch: int
    M: int
    N: int
    K: int
    tau: int                                # 0: rows (M) are the main axis, 1: columns (N)
    program: Optional[Program]
    descs: List[Desc] = field(default_factory=list)
    pool_size: int = 0
    level: int = 0
    useful: int = 0
    covered: int = 0
    k_parts: int = 1                        # workgroups per tile along the reduce axis
    k_part_tiles: int = 0                   # k-tiles per part (the last part may get fewer)


def resolve_shape(op: Op, batch=1, m=0, n=0, k=0, img_n=0, img_h=0, img_w=0):
    """Runtime shape -> GEMM view (batch, M, N, K); conv maps space (n,p,q) to rows."""
    if op.kind == OP_CONV2D:
        P = (img_h + 2 * op.pad - op.r) // op.stride + 1
        Qo = (img_w + 2 * op.pad - op.s) // op.stride + 1
        return 1, img_n * P * Qo, op.c_out, op.r * op.s * op.c_in
    ms, ns, ks = op.gemm_static()
    return batch, (ms or m), (ns or n), (ks or k)


def main_axis(op: Op, M, N):
    """Main axis tau = the largest dynamic space axis (tie: rows); rows if none is dynamic."""
    ms, ns, _ = op.gemm_static()
    dyn_m, dyn_n = ms == 0, ns == 0
    if dyn_m and dyn_n:
        return 0 if M >= N else 1
    if dyn_n and not dyn_m:
        return 1
    return 0


def _ext(u: UKernel, axis):
    return u.tm if axis == 0 else u.tn


def build_pool(extents, Hp, kinds=None):
    """Alg. 2 over the main-axis extents of the uKernel set (extents[i] belongs to uKernel
    i) on the main-axis size Hp.  kinds[i], if given, is the workgroup size class of uKernel i: one
    launch has one workgroup size, so K2 must be of K1's kind.  For each K1 in set order: a single-uKernel program when
    K1 divides Hp; otherwise Hp = Num1*K1 + Num2*K2 with a second uKernel K2.
    Reading: on gfx950 every extent is a multiple of the 16-row granule, so the *first*
    success of the printed search (smallest Num1) is always Num1 = 1 followed by a long run
    of granule tiles; the search is therefore run from the other end and stops at its
    *last* success (largest Num1 whose positive remainder some K2 divides), and every K2
    dividing that remainder yields a program.  On the paper's worked example the success
    is unique, so both readings give 53 = 3*7 + 4*8."""
    pool = []
    for i1, e1 in enumerate(extents):
        if Hp % e1 == 0:
            pool.append([(i1, Hp // e1)])
            continue
        for n1 in range(Hp // e1, 0, -1):
            rem = Hp - n1 * e1
            found = [(i2, rem // e2) for i2, e2 in enumerate(extents)
                     if e2 != e1 and rem % e2 == 0 and (kinds is None or kinds[i2] == kinds[i1])]
            if found:
                pool.extend([(i1, n1), f] for f in found)
                break
    return pool


K_PART_CHOICES = (1, 2, 3, 4, 6, 8)    # workgroups per tile along the reduce axis the planner considers
KPART_ACC_MAX = 128                    # uKernels with more accumulator registers per lane are never split


def part_tiles(K, tk, k_parts):
    """k-tiles per part when the nk = ceil(K / tk) k-tiles are dealt out in equal runs."""
    return ceil_div(max(ceil_div(K, tk), 1), k_parts)


def split_allowed(parts, uks, K, k_parts, t, hw, tiles):
    """May every tile of this program (tiles of them) be split over k_parts workgroups along the
    reduce axis?  One part is always allowed.  More need: room in the registers of every
    constituent for the exchange, at least k_part_min_tiles k-tiles per part, no empty part, and
    all tiles * k_parts workgroups resident at once (the split is there to fill a device the
    tiles alone leave partly idle, not to queue more rounds of workgroups)."""
    if k_parts == 1:
        return True
    if k_parts > t.get("k_parts_max", 1):
        return False
    if any(uks[uid].acc_regs > KPART_ACC_MAX or eight_waves(uks[uid]) for uid, _ in parts):
        return False                                   # (four-wave bodies only)
    per_cu = min([t["zeta"]] + [uks[uid].max_wg_per_cu for uid, _ in parts])
    if tiles * k_parts > hw["num_cus"] * per_cu:
        return False
    tk = uks[parts[0][0]].tk
    nk = max(ceil_div(K, tk), 1)
    per = ceil_div(nk, k_parts)
    return nk // k_parts >= max(t.get("k_part_min_tiles", 1), 1) and ceil_div(nk, per) == k_parts


STRIP_CHOICES = 3       # strip uKernels tried per part (the widest ones that pad less than one more K1 tile)


def strip_choices(u, uks, Wp, tau):
    """Second-axis combination for one part (Fig. 4(d): both space axes of a batched Matmul are
    dynamic): along the other axis sigma a part of uKernel K1 places Num1 = floor(W' / K1.ext)
    whole tiles and covers the rest with Num2 tiles of a narrower uKernel K2 that has K1's extent
    along tau (so the rows of the two line up): W' = Num1*K1 + Num2*K2 - padding, Alg. 2's form
    with K1 given.  Candidates for K2: every narrower uKernel with that tau extent whose Num2 tiles
    pad less than one more K1 tile would, widest first (ties: lower index), at most STRIP_CHOICES
    of them.  None if K1 divides W' or is wider than W'.
    Returns a list of (K2 id, Num1, Num2)."""
    e = _ext(u, 1 - tau)
    n_full, rem = Wp // e, Wp % e
    if n_full < 1 or rem == 0:
        return []
    cands = [v for v in uks
             if _ext(v, tau) == _ext(u, tau) and _ext(v, 1 - tau) < e and ceil_by(rem, _ext(v, 1 - tau)) < e
             and eight_waves(v) == eight_waves(u)]
    cands.sort(key=lambda v: (-_ext(v, 1 - tau), v.id))
    return [(v.id, n_full, ceil_div(rem, _ext(v, 1 - tau))) for v in cands[:STRIP_CHOICES]]


def strip_variants(parts, uks, Wp, tau):
    """Every way to give the parts of a program a strip or none (at least one strip), in a fixed
    order: the choices of the first part vary slowest, 'no strip' comes first."""
    per_part = []
    for uid, _ in parts:
        u = uks[uid]
        per_part.append([(-1, ceil_div(Wp, _ext(u, 1 - tau)), 0)] + strip_choices(u, uks, Wp, tau))
    out = [[]]
    for choices in per_part:
        out = [prev + [c] for prev in out for c in choices]
    return [v for v in out if any(c[0] >= 0 for c in v)]


def constituents(parts, strips, uks, batch, M, N, tau):
    """The uKernel-homogeneous regions of a program in placement order: for each one
    (ukernel id, tiles per batch entry, useful output elements per batch entry, area per batch entry)."""
    H = M if tau == 0 else N
    W = N if tau == 0 else M
    Wp = ceil_by(W, GRANULE)
    off, out = 0, []
    for i, (uid, cnt) in enumerate(parts):
        u = uks[uid]
        e = _ext(u, tau)
        rows = max(0, min(H - off, cnt * e))
        off += cnt * e
        if strips is None or strips[i][0] < 0:
            across = ceil_div(Wp, _ext(u, 1 - tau))
            out.append((uid, cnt * across, rows * W, cnt * across * u.tm * u.tn))
        else:
            sid, n_full, n_strip = strips[i]
            v = uks[sid]
            w_main = min(W, n_full * _ext(u, 1 - tau))
            out.append((uid, cnt * n_full, rows * w_main, cnt * n_full * u.tm * u.tn))
            out.append((sid, cnt * n_strip, rows * (W - w_main), cnt * n_strip * v.tm * v.tn))
    return out


def evaluate(parts, uks, batch, M, N, tau, hw, t, cap_q, k_parts=1, K=0, out_bytes=4, strips=None):
    """Cached-metric evaluation of one program (Sec. 5.2) on the actual shape.  With k_parts > 1
    every tile is worked on by k_parts workgroups (occupancy rescue, see split_allowed): the
    workgroup count of Eq. 3, Eq. 5 and SetBound is k_parts times the tile count, and compute_eff
    is taken on one part of the reduce axis."""
    order = sorted(range(len(parts)), key=lambda i: parts[i])
    parts_sorted = [parts[i] for i in order]
    strips_sorted = [strips[i] for i in order] if strips is not None else None
    cons = constituents(parts_sorted, strips_sorted, uks, batch, M, N, tau)
    tiles_per_batch = sum(c[1] for c in cons)
    area = sum(c[3] for c in cons)
    T = batch * tiles_per_batch
    Wg = T * k_parts
    p = Program(parts=parts_sorted, num_tiles=T, area=area, k_parts=k_parts,
                strips=strips_sorted if strips_sorted is not None else [])
    p.k1 = parts[0][0]
    p.k2 = parts[1][0] if len(parts) > 1 else -1
    # SetBound (Alg. 1): block.bound = min(K.wkl.block, zeta)
    p.block_bound = min(max(1, ceil_div(Wg, hw["num_cus"])), t["zeta"])
    ids = [c[0] for c in cons]
    p.in_bound = all(waves_bound(uks[uid]) >= p.block_bound for uid in ids)
    occ = occ_fraction(Wg, hw["num_cus"])
    pad = pad_fraction(M * N, area)
    p.occ_q = (occ[0] << Q) // occ[1]
    p.pad_q = (pad[0] << Q) // pad[1]
    p.cross = cross_pick(pad, occ, t)
    p.saturated = Wg >= t["zeta"] * hw["num_cus"]                # Eq. 5
    # compute_eff is normalised by the set's best; a two-uKernel program takes the average of
    # its constituents (Sec. 5.2).  Each constituent contributes the value cached for the number
    # of workgroups that share a CU on this shape: min(its capacity, block.bound)
    acc = 0
    for uid in ids:
        acc += (min(cmr_split(uks[uid], p.block_bound, k_parts, K, hw, out_bytes), cap_q) << Q) // cap_q
    p.cmr_q = acc // len(ids)
    if t.get("sia_form", SIA_LINEAR) == SIA_LINEAR:
        p.sia_q = t["c0"] * p.cmr_q + t["c1"] * p.pad_q + t["c2"] * p.occ_q   # Eq. 1 as printed
    else:
        p.sia_q = sia_product(cons, uks, batch, hw, t, cap_q, p.block_bound, k_parts, K, out_bytes)
    return p


def cmr_cap(uks):
    """Normaliser of the CMR term: the best compute_eff cached anywhere in the set."""
    return max(max(u.cmr_q, u.cmr2_q) for u in uks)


def cmr_at(u, block_bound):
    """The cached compute_eff of uKernel u when block_bound workgroups per CU are wanted."""
    return u.cmr2_q if min(u.max_wg_per_cu, block_bound) >= 2 else u.cmr_q


def cmr_split(u, block_bound, k_parts, K, hw, out_bytes):
    """compute_eff of uKernel u on this shape: the cached value when a tile is one workgroup; for
    a reduce-axis split, Eq. 6 re-evaluated on one part: its share of the k-tiles, 8 more bytes of
    global traffic per output element (the fp32 partial written once and read once) and the
    exchange: its round trips (part_exchange_clk) plus the time the workgroup that arrives last
    needs to read the k_parts fp32 partial tiles (tm * tn * 4 bytes each) at
    part_exchange_bytes_per_clk (0 switches this term off)."""
    if k_parts == 1:
        return cmr_at(u, block_bound)
    r = 2 if min(u.max_wg_per_cu, block_bound) >= 2 else 1
    k_part = part_tiles(K, u.tk, k_parts) * u.tk
    rate = hw["part_exchange_bytes_per_clk"]
    exchange = hw["part_exchange_clk"] + ((k_parts * u.tm * u.tn * 4) // rate if rate else 0)
    cn, cd = compute_eff(u.tm, u.tn, u.gm, u.gn, k_part, hw, u.gk, u.tk, residents=r,
                         out_bytes=out_bytes + 8, exchange_clk=exchange)
    return (cn << Q) // cd


def sia_product(cons, uks, batch, hw, t, cap_q, block_bound, k_parts=1, K=0, out_bytes=4):
    """Eq. 1 in its multiplicative (log-domain) form, evaluated per uKernel from the metrics
    cached in each uKernel's data structure (Sec. 5.2): each constituent K (a region of the
    program tiled by one uKernel, see constituents()) gets CMR^c0 * Pad^c1 * Occ^c2 from its own
    sub-workload -- the outputs it covers, its own tile count.  The product is what a throughput
    estimate looks like (fraction of cores busy x fraction of useful work x per-core efficiency);
    a weighted sum of the logarithms of the three metrics ranks single-uKernel programs
    identically.  The paper averages the constituents of a program without saying how; here it is
    the harmonic mean weighted by the useful output elements u_i each constituent produces,
        score = sum(u_i) / sum(u_i / x_i),
    i.e. total work over the time the constituents need at their own rates (an unweighted mean
    lets a 16-row tail decide the fate of a program whose other constituent does 95 % of the
    work; an arithmetic mean hides a slow constituent).  Fixed point: every multiply is
    floor(x * y / 2^20); the mean is floor of the exact ratio of the q20 values, computed as
    (sum u_i) * prod x_i / sum_i (u_i * prod_{j != i} x_j).  A constituent with no useful output
    (a strip or tail that lies wholly in the padding) carries no weight."""
    terms = []
    for uid, tiles, useful, area in cons:
        u = uks[uid]
        T = batch * tiles * k_parts                         # workgroups of this constituent
        cmr_q = (min(cmr_split(u, block_bound, k_parts, K, hw, out_bytes), cap_q) << Q) // cap_q
        pad_q = (useful << Q) // area
        on, od = occ_fraction(T, hw["num_cus"])
        occ_q = (on << Q) // od
        x = ONE
        for q, c in ((cmr_q, t["c0"]), (pad_q, t["c1"]), (occ_q, t["c2"])):
            for _ in range(c):
                x = (x * q) >> Q
        terms.append((useful, x))
    if len(terms) > 1:
        terms = [(u_, x) for u_, x in terms if u_ > 0] or terms[:1]
    if any(x == 0 for _, x in terms):
        return 0
    if len(terms) == 1:
        return terms[0][1]
    prod_all = 1
    for _, x in terms:
        prod_all *= x
    den = sum(u_ * (prod_all // x) for u_, x in terms)
    return (sum(u_ for u_, _ in terms) * prod_all) // den


def emit(parts, uks, batch, M, N, tau, strips=None):
    """Tile descriptors in canonical order: uKernel id, batch, m0, n0 ascending.  Along tau
    the part with the lower id (larger tile) comes first; along the other axis a part's own tiles
    come first, then its strip's."""
    descs = []
    off = 0
    Wp = ceil_by(N if tau == 0 else M, GRANULE)
    order = sorted(range(len(parts)), key=lambda i: parts[i])
    for i in order:
        uid, cnt = parts[i]
        u = uks[uid]
        e_tau = _ext(u, tau)
        if strips is None or not strips or strips[i][0] < 0:
            runs = [(u, 0, ceil_div(Wp, _ext(u, 1 - tau)))]
        else:
            sid, n_full, n_strip = strips[i]
            runs = [(u, 0, n_full), (uks[sid], n_full * _ext(u, 1 - tau), n_strip)]
        for v, start, count in runs:
            along = [off + j * e_tau for j in range(cnt)]
            across = [start + j * _ext(v, 1 - tau) for j in range(count)]
            m_list, n_list = (along, across) if tau == 0 else (across, along)
            for b in range(batch):
                for m0 in m_list:
                    for n0 in n_list:
                        mv, nv = min(v.tm, M - m0), min(v.tn, N - n0)
                        descs.append(Desc(v.id, b, m0, n0, mv, nv, 1 if (mv < v.tm or nv < v.tn) else 0))
        off += cnt * e_tau
    descs.sort(key=lambda d: (d.ukernel_id, d.batch, d.m0, d.n0))
    return descs


def plan(op: Op, uks: List[UKernel], shape, mode=PLAN_PATCHWORK, hw=None, t=None) -> Plan:
    """Runtime stage: pool construction (Alg. 2), evaluation (Eq. 1-3, 5), Top-1, descriptors.

    mode PLAN_PAD_BASELINE instead pads every dynamic axis up to a multiple of the single
    largest uKernel of the set (the 'optimized kernel in the manual library', Fig. 2)."""
    hw = hw or default_hw()
    t = t or default_tuning()
    batch, M, N, K = shape
    if not uks:
        raise ValueError("empty uKernel set")
    tau = main_axis(op, M, N)
    pl = Plan(batch, M, N, K, tau, None, useful=batch * M * N)
    if batch == 0 or M == 0 or N == 0:
        return pl
    cap_q = cmr_cap(uks)
    if mode == PLAN_PAD_BASELINE:
        u = uks[0]
        Hp = ceil_by(M if tau == 0 else N, _ext(u, tau))
        parts = [(0, Hp // _ext(u, tau))]
        prog = evaluate(parts, uks, batch, M, N, tau, hw, t, cap_q)
        pl.pool_size, pl.level = 1, 0 if prog.in_bound else 1
    else:
        Hp = ceil_by(M if tau == 0 else N, GRANULE)
        covers = build_pool([_ext(u, tau) for u in uks], Hp, kinds=[eight_waves(u) for u in uks])
        if not covers:
            # Alg. 2 found nothing (the main axis is shorter than every extent the static
            # axes admit): pad it up to the uKernel with the smallest main-axis extent
            e_min = min(_ext(u, tau) for u in uks)
            u = next(u for u in uks if _ext(u, tau) == e_min)
            covers = [[(u.id, ceil_div(Hp, e_min))]]
        pl.pool_size = len(covers)
        # Occupancy rescue (Matmul): every program is also scored with its tiles split over
        # 2, 3, ... workgroups along the reduce axis, where that is allowed
        # (the split runs in the LDS-DMA bodies only: rows of 16-byte chunks, K and N multiples of 8)
        choices = K_PART_CHOICES if op.kind == OP_MATMUL and K % 8 == 0 and N % 8 == 0 else (1,)
        # Two dynamic space axes: every program is also scored with second-axis strips
        ms, ns, _ = op.gemm_static()
        two_axes = ms == 0 and ns == 0 and t.get("second_axis_strips", 0) != 0
        Wp = ceil_by(N if tau == 0 else M, GRANULE)
        pool = []
        for parts in covers:
            whole = evaluate(parts, uks, batch, M, N, tau, hw, t, cap_q)
            pool.append(whole)
            pool.extend(evaluate(parts, uks, batch, M, N, tau, hw, t, cap_q, kp, K, op.out_bytes)
                        for kp in choices[1:] if split_allowed(parts, uks, K, kp, t, hw, whole.num_tiles))
            if two_axes:
                pool.extend(evaluate(parts, uks, batch, M, N, tau, hw, t, cap_q, strips=strips)
                            for strips in strip_variants(parts, uks, Wp, tau))
        # runtime stage: the programs whose uKernels fit block.bound workgroups per CU on this
        # shape (SetBound); all of them if none does
        cands = [p for p in pool if p.in_bound]
        pl.level = 0
        if not cands:
            cands, pl.level = pool, 1
        # Top-1 by SIA; ties: fewer parts, fewer tiles, no strips, then lower K1 index, then lower K2 index
        # (two strip variants of one program that tie: the one listed first by strip_variants)
        prog = min(enumerate(cands), key=lambda ip: (-ip[1].sia_q, ip[1].k_parts, ip[1].num_tiles, len(ip[1].strips) > 0,
                                                     ip[1].k1, ip[1].k2, ip[0]))[1]
    pl.program = prog
    pl.descs = emit(prog.parts, uks, batch, M, N, tau, prog.strips or None)
    pl.covered = batch * prog.area
    pl.k_parts = prog.k_parts
    pl.k_part_tiles = part_tiles(K, uks[prog.parts[0][0]].tk, prog.k_parts)
    assert len(pl.descs) == prog.num_tiles
    return pl


def exact_cover_counts(pl: Plan, uks: List[UKernel]):
    """Paint every descriptor's valid region into an integer count array [batch, M, N];
    a correct plan gives all ones.  Independent of emit(): uses only the descriptors."""
    import numpy as np
    cnt = np.zeros((pl.batch, pl.M, pl.N), dtype=np.int32)
    for d in pl.descs:
        cnt[d.batch, d.m0:d.m0 + d.m_valid, d.n0:d.n0 + d.n_valid] += 1
    return cnt


def plan_grouped(op: Op, uks: List[UKernel], shapes, mode=PLAN_PATCHWORK, hw=None, t=None):
    """Groups of batched Matmuls of different shapes in one launch (the motivation of Sec. 1 /
    Fig. 1(b): sequences of one batch differ in length, and padding them to the longest wastes most
    of the work).  shapes: one (batch, M, N, K) per group.  Returns (table, offsets):

    offsets[g] = element offsets (A, B, C) of group g in buffers that pack the groups one after the
    other in the order given, each group densely packed like a plain batched problem; one more
    entry holds the totals.

    table = list of (group, Desc).  The groups share the device, so a group's program is the one
    plan() picks for its shape at the batch of the whole launch -- the sum of the groups' batches
    rounded up to a power of two, at most batch_hi -- and the group contributes the descriptors of
    its own batch entries of that plan.  The table lists the groups with the longest reduce axis
    first, then the larger outputs (ties keep the given order): the workgroups with the most work
    start first."""
    offsets, off = [], (0, 0, 0)
    for b, M, N, K in shapes:
        offsets.append(off)
        off = (off[0] + b * M * K, off[1] + b * K * N, off[2] + b * M * N)
    offsets.append(off)
    launch_batch = 1
    while launch_batch < sum(s[0] for s in shapes):
        launch_batch *= 2
    if op.batch_hi:
        launch_batch = min(launch_batch, op.batch_hi)
    table = []
    for g in sorted(range(len(shapes)), key=lambda i: (-shapes[i][3], -shapes[i][1] * shapes[i][2])):
        b, M, N, K = shapes[g]
        if b == 0:
            continue
        whole = plan(op, uks, (max(b, launch_batch), M, N, K), mode, hw, t)
        table += [(g, d) for d in whole.descs if d.batch < b]
    return table, offsets

