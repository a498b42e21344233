// Host half of the library: hardware model, uKernel-set generator (compile stage, Sec. 4) and
// runtime planner (Sec. 5).  Integer arithmetic throughout: every cached metric is the floor of
// an exact rational times 2^20, so plans are reproducible bit for bit.
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "family.h"
#include "ft_internal.h"
#include "tile_order.h"

namespace {

typedef unsigned __int128 u128;
constexpr uint32_t QBITS = 20;
constexpr uint32_t GRANULE = 16;      // smallest MFMA output extent (16x16x32)
constexpr uint32_t ELT = 2;           // bytes per input element
constexpr uint32_t MIN_STAGES = 2, MAX_STAGES = 8;

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
inline uint64_t ceil_by(uint64_t x, uint64_t m) { return m * ceil_div(x, m); }

void hw_defaults(ft_hw_model *h) {
    std::memset(h, 0, sizeof(*h));
    h->struct_size = sizeof(*h);
    h->num_cus = 256;
    h->simds_per_cu = 4;
    h->wave_size = 64;
    h->regs_per_lane = 512;
    h->max_waves_per_simd = 8;
    h->lds_bytes_per_cu = 163840;
    h->clock_mhz = 2400;
    h->mfma_flops_per_clk_per_cu = 4096;
    h->bw_global_bytes_per_clk_per_cu = 64;
    h->bw_lds_bytes_per_clk_per_cu = 256;
    h->ktile_latency_clk = 400;
    h->solo_copy_exposed_pct = 50;
    h->hbm_gbytes_per_s = 8000;
    h->num_xcds = 8;
    h->part_exchange_clk = 2000;
    h->part_exchange_bytes_per_clk = 16;
    h->phase_latency_clk = 150;
}

void tuning_defaults(ft_tuning *t) {
    std::memset(t, 0, sizeof(*t));
    t->struct_size = sizeof(*t);
    t->eps_min_pm = 500; t->eps_max_pm = 950; t->eps_step_pm = 10;   // Sec. 4.2: 50%..95%, +1%
    t->lam_max_pm = 950; t->lam_min_pm = 900; t->lam_step_pm = 1;    // 95%..90%, -0.1%
    t->zeta = 2;                                                     // Sec. 4.2
    t->rest_regs = 72;
    t->psi_num = 1; t->psi_den = 64;
    t->c0 = t->c1 = t->c2 = 1;                                       // Sec. 5.2
    t->sia_form = FT_SIA_PRODUCT;
    t->k_parts_max = 8;
    t->k_part_min_tiles = 8;
    t->second_axis_strips = 0;
    t->two_team_bodies = 1;
}

struct Gemm {                // GEMM view of an operator: static extents (0 = dynamic)
    uint32_t m, n, k;
};

Gemm static_view(const ft_op_desc &d) {
    if (d.kind == FT_OP_CONV2D) return {0u, d.c_out, d.r * d.s * d.c_in};
    return {d.m, d.n, d.k};
}

// Eq. 6 / Eq. 7: compute_eff = (FLOPs / FLOPS) : K_mem as num/den.  K_mem is the time the k loop
// needs, so the ratio is the share of that time the MFMA pipes are busy.  With t_c = FLOPs/FLOPS,
// t_g = global bytes / bw_G, t_s = LDS bytes / bw_S; a wave walks through nk_w = ceil(nk / gk) of the
// nk = ceil(K/tk) k-tiles, so the MFMA phase lasts t_ce = t_c * gk * nk_w / nk (= t_c unless a split-k
// grid leaves waves idle) and the loop pays t_l = ktile_latency_clk * nk_w:
//   residents >= 2 (workgroups sharing a CU): phases of different waves overlap,
//       K_mem = max(t_ce, t_g, t_s) + t_l / residents
//   residents == 1: the single wave of a SIMD issues copies and MFMAs itself,
//       K_mem = t_ce + solo_copy_exposed_pct % of t_g + t_l
//   eight waves on the same k-tiles (gm * gn = 8), alone on the CU: the two waves of a SIMD pass the
//       workgroup's barriers together, so they read their fragments at the same time (t_s at half the
//       LDS rate) and half as much of the copy time stays exposed as for a single wave; the latency
//       of a k-tile is shared by the two but not hidden:
//       K_mem = max(t_c, 2 t_s) + solo_copy_exposed_pct / 2 % of t_g + 2/3 t_l
//   two teams (gk = 2, eight waves): a SIMD holds one wave of each team; while one runs the MFMAs of its
//       k-tile the other issues copies, one s_barrier per k-tile:
//       K_mem = max(t_c, t_g, t_s) + phase_latency_clk * nk / residents
// exchange_clk: a fixed time added to t_l: the round trips of a workgroup that hands its partial
// tile to the others of a reduce-axis split.
void compute_eff(uint32_t tm, uint32_t tn, uint32_t gm, uint32_t gn, uint32_t gk, uint32_t tk, uint64_t kref,
                 uint32_t residents, uint32_t out_bytes, const ft_hw_model &hw, u128 *num, u128 *den,
                 uint32_t exchange_clk = 0) {
    const u128 F = hw.mfma_flops_per_clk_per_cu, G = hw.bw_global_bytes_per_clk_per_cu, S = hw.bw_lds_bytes_per_clk_per_cu;
    const u128 flops = (u128)2 * tm * tn * kref;
    const u128 gbytes = (u128)(tm + tn) * kref * ELT + (u128)tm * tn * out_bytes;                // data_r + data_w
    const u128 sbytes = (u128)(tm + tn) * kref * ELT + (u128)kref * ELT * ((u128)tm * gn + (u128)tn * gm);
    const u128 nk = ceil_div(kref, tk);
    const u128 r = residents;
    const u128 ed = 100;
    if (gm * gn == 8 && gk == 1 && residents < 2) {
        // over the common denominator F * G * S * 600
        const u128 c8 = flops * G * S * 600;
        const u128 s8 = sbytes * F * G * 1200;
        const u128 g8 = gbytes * F * S * 3 * hw.solo_copy_exposed_pct;
        const u128 l8 = ((u128)hw.ktile_latency_clk * nk + exchange_clk) * F * G * S * 400;
        *num = c8;
        *den = std::max(c8, s8) + g8 + l8;
        return;
    }
    if (gk == 2) {
        // over the common denominator F * G * S * r
        const u128 c2 = flops * G * S * r;
        const u128 g2 = gbytes * F * S * r;
        const u128 s2 = sbytes * F * G * r;
        const u128 l2 = ((u128)hw.phase_latency_clk * nk + exchange_clk) * F * G * S;
        *num = c2;
        *den = std::max(c2, std::max(g2, s2)) + l2;
        return;
    }
    const u128 nk_w = ceil_div((uint64_t)nk, gk);
    // everything over the common denominator F * G * S * nk * r * ed
    const u128 c = flops * G * S * nk * r * ed;
    const u128 ce = flops * G * S * gk * nk_w * r * ed;
    const u128 lt = ((u128)hw.ktile_latency_clk * nk_w + exchange_clk) * F * G * S * nk * ed;
    *num = c;
    if (r >= 2) {
        const u128 g = gbytes * F * S * nk * r * ed;
        const u128 s = sbytes * F * G * nk * r * ed;
        *den = std::max(ce, std::max(g, s)) + lt;
    } else {
        *den = ce + gbytes * F * S * nk * hw.solo_copy_exposed_pct + lt;
    }
}

// Shapes of the workload along one dynamic axis: both ends of the registered range and the
// multiples of the granule between them, thinned to about cap points by a fixed stride.
void axis_samples(uint64_t lo, uint64_t hi, uint64_t cap, std::vector<uint64_t> &out) {
    out.clear();
    if (lo < 1) lo = 1;
    if (hi < lo) return;
    out.push_back(lo);
    uint64_t first = ceil_by(lo, GRANULE);
    if (first <= hi) {
        uint64_t n_mult = (hi - first) / GRANULE + 1;
        uint64_t stride = std::max<uint64_t>(1, ceil_div(n_mult, cap)) * GRANULE;
        for (uint64_t v = first; v <= hi; v += stride) out.push_back(v);
    }
    out.push_back(hi);
    std::sort(out.begin(), out.end());
    out.erase(std::unique(out.begin(), out.end()), out.end());
}

struct Part { uint32_t id, count; };
// second-axis strip of a part: id < 0 = none; n_full tiles of the part's own uKernel across the
// other axis, then n_strip tiles of uKernel id
struct Strip { int32_t id; uint32_t n_full, n_strip; };
struct Region { uint32_t id; uint64_t tiles, useful, area; };     // one uKernel-homogeneous region, per batch entry

struct Program {
    Part part[2];
    uint32_t nparts;
    int64_t k1, k2;           // pool identity (k2 = -1: single)
    uint64_t tiles, area;
    uint32_t block_bound;
    bool in_bound, cross, saturated;
    uint32_t pad_q, occ_q, cmr_q;
    uint64_t sia_q;
    uint32_t k_parts;         // workgroups per tile along the reduce axis (0 reads as 1)
    Strip strip[2];           // aligned with part[]
    bool has_strips;
};

inline uint32_t ext(const ft_ukernel_info &u, uint32_t axis) { return axis == 0 ? u.tm : u.tn; }
// workgroups of eight waves (two teams, or an eight-wave grid) run in kernels of their own: one launch,
// one workgroup size
inline bool eight_waves(const ft_ukernel_info &u) { return u.gk == 2 || u.gm * u.gn == 8; }

// What a uKernel offers against Alg. 1's block.bound (workgroups a CU should hold): its residency, and
// twice that for an eight-wave grid, whose workgroup already puts two waves on every SIMD.  (A two-team
// workgroup does too, but its teams take turns on the k-tiles: it counts as one.)
inline uint32_t waves_bound(const ft_ukernel_info &u) { return u.max_wg_per_cu * (u.gm * u.gn == 8 ? 2u : 1u); }

// Reduce-axis split (occupancy rescue): k-tiles per part when the nk = ceil(K / tk) k-tiles are
// dealt out in equal runs.
inline uint64_t part_tiles(uint64_t K, uint32_t tk, uint32_t k_parts) {
    return ceil_div(std::max<uint64_t>(ceil_div(K, tk), 1), k_parts);
}

const uint32_t kPartChoices[] = {1, 2, 3, 4, 6, 8};     // parts per tile the planner considers

struct Program;
bool split_allowed(const Program &p, const ft_ukset &set, uint64_t K, uint32_t k_parts);

bool cross_pick(u128 pn, u128 pd, u128 on, u128 od, const ft_tuning &t) {
    // lock-step staircase: eps up, lambda down, until either bound is passed (Alg. 1)
    uint32_t eps = t.eps_min_pm;
    int64_t lam = t.lam_max_pm;
    if (t.eps_step_pm == 0 && t.lam_step_pm == 0)
        return 1000 * pn >= (u128)eps * pd && 1000 * on >= (u128)lam * od;
    while (eps <= t.eps_max_pm && lam >= (int64_t)t.lam_min_pm) {
        if (1000 * pn >= (u128)eps * pd && 1000 * on >= (u128)lam * od) return true;
        eps += t.eps_step_pm;
        lam -= t.lam_step_pm;
    }
    return false;
}

// CrossPick and Eq. 5 for one uKernel over the workload: kept iff some shape, composed of this
// uKernel alone, passes the staircase with a tile count of at least Active Blocks = zeta x NumCores.
// (SetBound needs the shape's block.bound and is applied when a shape is planned.)
bool passes_workload(uint32_t tm, uint32_t tn, const std::vector<uint64_t> &ms,
                     const std::vector<uint64_t> &ns, uint64_t batch, const ft_hw_model &hw, const ft_tuning &t) {
    for (uint64_t M : ms)
        for (uint64_t N : ns) {
            uint64_t T = batch * ceil_div(M, tm) * ceil_div(N, tn);
            if (T < (uint64_t)t.zeta * hw.num_cus) continue;        // Eq. 5
            u128 pn = (u128)M * N, pd = (u128)T * tm * tn;
            u128 on = T, od = ceil_by(T, hw.num_cus);
            if (cross_pick(pn, pd, on, od, t)) return true;
        }
    return false;
}

// Cached-metric evaluation of one program on the actual shape (Sec. 5.2).  With k_parts > 1 every
// tile is worked on by k_parts workgroups: the workgroup count of Eq. 3, Eq. 5 and SetBound is
// k_parts times the tile count and compute_eff is taken on one part of the reduce axis (its share
// of the k-tiles, 8 more bytes of global traffic per output element for the fp32 partial written
// and read once, and the exchange's round trips).
// The uKernel-homogeneous regions of a program in placement order (parts ascending by id; a part's
// own tiles, then its strip): tiles, useful outputs and covered area per batch entry.
uint32_t regions_of(const Program &p, const ft_ukset &set, uint64_t M, uint64_t N, uint32_t tau, Region (&out)[4]) {
    const uint64_t H = tau == 0 ? M : N, W = tau == 0 ? N : M;
    const uint64_t Wp = ceil_by(W, GRANULE);
    uint64_t off = 0;
    uint32_t n = 0;
    for (uint32_t i = 0; i < p.nparts; ++i) {
        const ft_ukernel_info &u = set.uk[p.part[i].id];
        const uint64_t e = ext(u, tau), cnt = p.part[i].count, span = cnt * e;
        const uint64_t rows = H > off ? std::min<uint64_t>(H - off, span) : 0;
        off += span;
        if (!p.has_strips || p.strip[i].id < 0) {
            const uint64_t across = ceil_div(Wp, ext(u, 1 - tau));
            out[n++] = {u.id, cnt * across, rows * W, cnt * across * u.tm * u.tn};
        } else {
            const ft_ukernel_info &v = set.uk[(uint32_t)p.strip[i].id];
            const uint64_t w_main = std::min<uint64_t>(W, (uint64_t)p.strip[i].n_full * ext(u, 1 - tau));
            out[n++] = {u.id, cnt * p.strip[i].n_full, rows * w_main, cnt * p.strip[i].n_full * u.tm * u.tn};
            out[n++] = {v.id, cnt * p.strip[i].n_strip, rows * (W - w_main), cnt * p.strip[i].n_strip * v.tm * v.tn};
        }
    }
    return n;
}

void evaluate(Program &p, const ft_ukset &set, uint64_t batch, uint64_t M, uint64_t N, uint32_t tau,
              uint32_t k_parts = 1, uint64_t K = 0) {
    const ft_hw_model &hw = set.hw;
    const ft_tuning &t = set.t;
    if (p.nparts == 2 && p.part[0].id > p.part[1].id) {       // placement order: ascending id
        std::swap(p.part[0], p.part[1]);
        std::swap(p.strip[0], p.strip[1]);
    }
    Region reg[4];
    const uint32_t nreg = regions_of(p, set, M, N, tau, reg);
    uint64_t per_batch = 0, area = 0;
    for (uint32_t i = 0; i < nreg; ++i) { per_batch += reg[i].tiles; area += reg[i].area; }
    p.tiles = batch * per_batch;
    p.area = area;
    p.k_parts = k_parts;
    const uint64_t wgs = p.tiles * k_parts;                                         // workgroups
    const uint32_t out_bytes = set.op.out_dtype == FT_OUT_SAME ? ELT : 4;
    uint64_t need = std::max<uint64_t>(1, ceil_div(wgs, hw.num_cus));              // K.wkl.block
    p.block_bound = (uint32_t)std::min<uint64_t>(need, t.zeta);                     // SetBound
    p.in_bound = true;
    for (uint32_t i = 0; i < nreg; ++i)
        if (waves_bound(set.uk[reg[i].id]) < p.block_bound) p.in_bound = false;
    u128 on = wgs, od = ceil_by(wgs, hw.num_cus);                                   // Eq. 3
    u128 pn = (u128)M * N, pd = area;                                               // Eq. 2
    p.occ_q = (uint32_t)((on << QBITS) / od);
    p.pad_q = (uint32_t)((pn << QBITS) / pd);
    p.cross = cross_pick(pn, pd, on, od, t);
    p.saturated = wgs >= (uint64_t)t.zeta * hw.num_cus;                             // Eq. 5
    // each constituent contributes the compute_eff cached for the number of workgroups that share
    // a CU on this shape: min(its capacity, block.bound)
    auto cmr_at = [&](const ft_ukernel_info &u) -> uint64_t {
        const bool shared = std::min<uint32_t>(u.max_wg_per_cu, p.block_bound) >= 2;
        if (k_parts == 1) return shared ? u.cmr_shared_q20 : u.cmr_q20;
        u128 cn, cd;
        // the exchange: round trips, plus the last workgroup reading k_parts fp32 partial tiles
        const uint64_t slabs = (uint64_t)k_parts * u.tm * u.tn * 4;
        const uint64_t exchange = hw.part_exchange_clk +
                                  (hw.part_exchange_bytes_per_clk ? slabs / hw.part_exchange_bytes_per_clk : 0);
        compute_eff(u.tm, u.tn, u.gm, u.gn, u.gk, u.tk, part_tiles(K, u.tk, k_parts) * u.tk, shared ? 2 : 1,
                    out_bytes + 8, hw, &cn, &cd, (uint32_t)exchange);
        return (uint64_t)((cn << QBITS) / cd);
    };
    uint64_t acc = 0;
    for (uint32_t i = 0; i < nreg; ++i) {
        uint64_t c = std::min<uint64_t>(cmr_at(set.uk[reg[i].id]), set.cap_q);
        acc += (uint64_t)(((u128)c << QBITS) / set.cap_q);
    }
    p.cmr_q = (uint32_t)(acc / nreg);
    if (t.sia_form == FT_SIA_LINEAR) {
        p.sia_q = (uint64_t)t.c0 * p.cmr_q + (uint64_t)t.c1 * p.pad_q + (uint64_t)t.c2 * p.occ_q;   // Eq. 1 as printed
    } else {
        // multiplicative form, per uKernel on its own sub-workload; the constituents are combined
        // by the harmonic mean weighted with the useful output elements of each (Sec. 5.2):
        // total work over the time all need at their own rates; a constituent with no useful
        // output carries no weight
        u128 us[4], xs[4];
        uint32_t n = 0;
        for (uint32_t i = 0; i < nreg; ++i) {
            const ft_ukernel_info &u = set.uk[reg[i].id];
            const uint64_t T = batch * reg[i].tiles * k_parts;      // workgroups of this constituent
            const uint64_t cq = (uint64_t)(((u128)std::min<uint64_t>(cmr_at(u), set.cap_q) << QBITS) / set.cap_q);
            const uint64_t pq = (uint64_t)(((u128)reg[i].useful << QBITS) / reg[i].area);
            const uint64_t oq = (uint64_t)(((u128)T << QBITS) / ceil_by(T, hw.num_cus));
            u128 x = (u128)1 << QBITS;
            const uint64_t qs[3] = {cq, pq, oq};
            const uint32_t cs[3] = {t.c0, t.c1, t.c2};
            for (int k = 0; k < 3; ++k)
                for (uint32_t r = 0; r < cs[k]; ++r) x = (x * qs[k]) >> QBITS;
            if (nreg > 1 && reg[i].useful == 0) continue;
            us[n] = reg[i].useful;
            xs[n] = x;
            ++n;
        }
        if (n == 0) {                     // every region lies in the padding: keep the first
            n = 1;
            us[0] = 0;
            u128 x = (u128)1 << QBITS;
            const ft_ukernel_info &u = set.uk[reg[0].id];
            const uint64_t T = batch * reg[0].tiles * k_parts;
            const uint64_t qs[3] = {(uint64_t)(((u128)std::min<uint64_t>(cmr_at(u), set.cap_q) << QBITS) / set.cap_q), 0,
                                    (uint64_t)(((u128)T << QBITS) / ceil_by(T, hw.num_cus))};
            const uint32_t cs[3] = {t.c0, t.c1, t.c2};
            for (int k = 0; k < 3; ++k)
                for (uint32_t r = 0; r < cs[k]; ++r) x = (x * qs[k]) >> QBITS;
            xs[0] = x;
        }
        bool zero = false;
        for (uint32_t i = 0; i < n; ++i) zero = zero || xs[i] == 0;
        if (zero) p.sia_q = 0;
        else if (n == 1) p.sia_q = (uint64_t)xs[0];
        else {
            u128 usum = 0, prod = 1, den = 0;
            for (uint32_t i = 0; i < n; ++i) { usum += us[i]; prod *= xs[i]; }
            for (uint32_t i = 0; i < n; ++i) {
                u128 others = 1;
                for (uint32_t j = 0; j < n; ++j) if (j != i) others *= xs[j];
                den += us[i] * others;
            }
            p.sia_q = (uint64_t)((usum * prod) / den);
        }
    }
}

// May every tile of program p (evaluated: p.tiles is set) be split over k_parts workgroups along
// the reduce axis?  Needs room in the registers of every constituent for the exchange, at least
// k_part_min_tiles k-tiles per part, no empty part, and all tiles * k_parts workgroups resident at
// once (the split fills a device the tiles alone leave partly idle; it does not queue more rounds).
bool split_allowed(const Program &p, const ft_ukset &set, uint64_t K, uint32_t k_parts) {
    if (k_parts == 1) return true;
    if (k_parts > set.t.k_parts_max) return false;
    uint32_t per_cu = set.t.zeta;
    for (uint32_t i = 0; i < p.nparts; ++i) {
        const ft_ukernel_info &u = set.uk[p.part[i].id];
        if (u.acc_regs > FT_KPART_ACC_MAX || eight_waves(u)) return false;   // (four-wave bodies only)
        per_cu = std::min(per_cu, u.max_wg_per_cu);
    }
    if (p.tiles * k_parts > (uint64_t)set.hw.num_cus * per_cu) return false;
    const uint64_t nk = std::max<uint64_t>(ceil_div(K, set.uk[p.part[0].id].tk), 1);
    const uint64_t per = ceil_div(nk, k_parts);
    return nk / k_parts >= std::max<uint32_t>(set.t.k_part_min_tiles, 1) && ceil_div(nk, per) == k_parts;
}

// Second-axis combination for one part (both space axes dynamic): along the other axis a part of
// uKernel K1 places Num1 = floor(W' / K1.ext) whole tiles and covers the rest with Num2 tiles of a
// narrower uKernel K2 that has K1's extent along tau.  Candidates for K2: every narrower uKernel
// with that tau extent whose tiles pad less than one more K1 tile would, widest first (ties: lower
// index), at most kStripChoices.  None if K1 divides W' or is wider than W'.
const uint32_t kStripChoices = 3;
uint32_t strip_choices(const ft_ukernel_info &u, const ft_ukset &set, uint64_t Wp, uint32_t tau, Strip (&out)[kStripChoices]) {
    const uint64_t e = ext(u, 1 - tau);
    const uint64_t n_full = Wp / e, rem = Wp % e;
    if (n_full < 1 || rem == 0) return 0;
    std::vector<const ft_ukernel_info *> c;
    for (const ft_ukernel_info &v : set.uk)
        if (ext(v, tau) == ext(u, tau) && ext(v, 1 - tau) < e && ceil_by(rem, ext(v, 1 - tau)) < e &&
            eight_waves(v) == eight_waves(u)) c.push_back(&v);
    std::stable_sort(c.begin(), c.end(), [&](const ft_ukernel_info *a, const ft_ukernel_info *b) {
        if (ext(*a, 1 - tau) != ext(*b, 1 - tau)) return ext(*a, 1 - tau) > ext(*b, 1 - tau);
        return a->id < b->id;
    });
    uint32_t n = 0;
    for (size_t i = 0; i < c.size() && n < kStripChoices; ++i)
        out[n++] = {(int32_t)c[i]->id, (uint32_t)n_full, (uint32_t)ceil_div(rem, ext(*c[i], 1 - tau))};
    return n;
}

// Every way to give the parts of program p a strip or none (at least one strip), in a fixed order:
// the choices of the first part vary slowest, "no strip" comes first.
void strip_variants(const Program &p, const ft_ukset &set, uint64_t Wp, uint32_t tau, std::vector<Program> &out) {
    Strip ch[2][kStripChoices + 1];
    uint32_t nch[2] = {1, 1};
    for (uint32_t i = 0; i < p.nparts; ++i) {
        const ft_ukernel_info &u = set.uk[p.part[i].id];
        ch[i][0] = {-1, (uint32_t)ceil_div(Wp, ext(u, 1 - tau)), 0};
        Strip tmp[kStripChoices];
        uint32_t n = strip_choices(u, set, Wp, tau, tmp);
        for (uint32_t j = 0; j < n; ++j) ch[i][1 + j] = tmp[j];
        nch[i] = 1 + n;
    }
    for (uint32_t a = 0; a < nch[0]; ++a)
        for (uint32_t b = 0; b < (p.nparts == 2 ? nch[1] : 1); ++b) {
            if (ch[0][a].id < 0 && (p.nparts == 1 || ch[1][b].id < 0)) continue;
            Program q = p;
            q.has_strips = true;
            q.strip[0] = ch[0][a];
            q.strip[1] = p.nparts == 2 ? ch[1][b] : Strip{-1, 0, 0};
            out.push_back(q);
        }
}

// Alg. 2 over the set's main-axis extents on the granule-rounded size Hp (last-success form).
void build_pool(const ft_ukset &set, uint64_t Hp, uint32_t tau, std::vector<Program> &pool) {
    const size_t n = set.uk.size();
    for (size_t i1 = 0; i1 < n; ++i1) {
        uint64_t e1 = ext(set.uk[i1], tau);
        if (Hp % e1 == 0) {
            Program p{};
            p.nparts = 1;
            p.part[0] = {(uint32_t)i1, (uint32_t)(Hp / e1)};
            p.k1 = (int64_t)i1; p.k2 = -1;
            pool.push_back(p);
            continue;
        }
        for (uint64_t n1 = Hp / e1; n1 >= 1; --n1) {
            uint64_t rem = Hp - n1 * e1;
            bool found = false;
            for (size_t i2 = 0; i2 < n; ++i2) {
                uint64_t e2 = ext(set.uk[i2], tau);
                // (one launch has one workgroup size: two-team uKernels pair with two-team uKernels)
                if (e2 != e1 && rem % e2 == 0 && eight_waves(set.uk[i1]) == eight_waves(set.uk[i2])) {
                    Program p{};
                    p.nparts = 2;
                    p.part[0] = {(uint32_t)i1, (uint32_t)n1};
                    p.part[1] = {(uint32_t)i2, (uint32_t)(rem / e2)};
                    p.k1 = (int64_t)i1; p.k2 = (int64_t)i2;
                    pool.push_back(p);
                    found = true;
                }
            }
            if (found) break;
        }
    }
}

uint32_t main_axis(const ft_op_desc &d, uint64_t M, uint64_t N) {
    Gemm s = static_view(d);
    bool dyn_m = s.m == 0, dyn_n = s.n == 0;
    if (dyn_m && dyn_n) return M >= N ? 0u : 1u;
    if (dyn_n && !dyn_m) return 1u;
    return 0u;
}

struct Resolved { uint64_t batch, M, N, K; uint32_t P, Q; };

ft_status resolve_axis(uint32_t stat, uint32_t lo, uint32_t hi, uint32_t given, uint64_t *out) {
    if (stat > 0) {
        if (given != 0 && given != stat) return FT_ERR_INVALID_ARG;
        *out = stat;
        return FT_OK;
    }
    if (given < lo || given > hi) return FT_ERR_OUT_OF_RANGE;
    *out = given;
    return FT_OK;
}

ft_status resolve(const ft_op_desc &d, const ft_shape &s, Resolved *r) {
    r->P = r->Q = 0;
    if (d.kind == FT_OP_CONV2D) {
        if (s.img_h + 2 * d.pad < d.r || s.img_w + 2 * d.pad < d.s) {
            if (s.img_n == 0 || s.img_h == 0 || s.img_w == 0) { r->batch = 1; r->M = 0; r->N = d.c_out; r->K = d.r * d.s * d.c_in; return FT_OK; }
            return FT_ERR_INVALID_ARG;
        }
        r->P = (s.img_h + 2 * d.pad - d.r) / d.stride + 1;
        r->Q = (s.img_w + 2 * d.pad - d.s) / d.stride + 1;
        r->batch = 1;
        r->M = (uint64_t)s.img_n * r->P * r->Q;
        r->N = d.c_out;
        r->K = (uint64_t)d.r * d.s * d.c_in;
        if (r->M < d.m_lo || r->M > d.m_hi) return FT_ERR_OUT_OF_RANGE;
        return FT_OK;
    }
    r->batch = d.kind == FT_OP_BMM ? s.batch : 1;
    ft_status st;
    if ((st = resolve_axis(d.m, d.m_lo, d.m_hi, s.m, &r->M)) != FT_OK) return st;
    if ((st = resolve_axis(d.n, d.n_lo, d.n_hi, s.n, &r->N)) != FT_OK) return st;
    if ((st = resolve_axis(d.k, d.k_lo, d.k_hi, s.k, &r->K)) != FT_OK) return st;
    return FT_OK;
}

struct SlotGrid { uint32_t first, rows, cols, m_base, n_base, tm, tn; };

void emit(const Program &p, const ft_ukset &set, const Resolved &r, uint32_t tau, std::vector<ft_tile_desc> &out,
          SlotGrid (&grid)[2]) {
    out.clear();
    out.reserve(p.tiles);
    uint64_t Wp = ceil_by(tau == 0 ? r.N : r.M, GRANULE);
    uint64_t off = 0;
    for (uint32_t i = 0; i < p.nparts; ++i) {           // parts are in ascending id order
        const ft_ukernel_info &u = set.uk[p.part[i].id];
        const uint64_t cnt = p.part[i].count;
        // runs across the other axis: the part's own tiles, then (if any) its strip's
        struct Run { const ft_ukernel_info *v; uint64_t start, count; } runs[2];
        uint32_t nruns = 1;
        if (!p.has_strips || p.strip[i].id < 0) {
            runs[0] = {&u, 0, ceil_div(Wp, ext(u, 1 - tau))};
        } else {
            runs[0] = {&u, 0, p.strip[i].n_full};
            runs[1] = {&set.uk[(uint32_t)p.strip[i].id], (uint64_t)p.strip[i].n_full * ext(u, 1 - tau), p.strip[i].n_strip};
            nruns = 2;
        }
        if (!p.has_strips) grid[i] = {(uint32_t)out.size(), (uint32_t)(tau == 0 ? cnt : runs[0].count),
                                      (uint32_t)(tau == 0 ? runs[0].count : cnt),
                                      (uint32_t)(tau == 0 ? off : 0), (uint32_t)(tau == 0 ? 0 : off), u.tm, u.tn};
        for (uint32_t q = 0; q < nruns; ++q) {
            const ft_ukernel_info &v = *runs[q].v;
            for (uint64_t b = 0; b < r.batch; ++b)
                for (uint64_t ia = 0; ia < (tau == 0 ? cnt : runs[q].count); ++ia)
                    for (uint64_t ib = 0; ib < (tau == 0 ? runs[q].count : cnt); ++ib) {
                        // tau == 0: ia walks the part's rows, ib the run's columns; tau == 1: the reverse
                        const uint64_t m0 = tau == 0 ? off + ia * v.tm : runs[q].start + ia * v.tm;
                        const uint64_t n0 = tau == 0 ? runs[q].start + ib * v.tn : off + ib * v.tn;
                        ft_tile_desc d;
                        d.ukernel_id = v.id;
                        d.batch = (uint32_t)b;
                        d.m0 = (uint32_t)m0;
                        d.n0 = (uint32_t)n0;
                        d.m_valid = (uint16_t)std::min<uint64_t>(v.tm, r.M - m0);
                        d.n_valid = (uint16_t)std::min<uint64_t>(v.tn, r.N - n0);
                        d.flags = (d.m_valid < v.tm || d.n_valid < v.tn) ? 1u : 0u;
                        out.push_back(d);
                    }
        }
        off += cnt * ext(u, tau);
    }
    if (p.has_strips)       // canonical order of the table: uKernel id, batch, m0, n0
        std::sort(out.begin(), out.end(), [](const ft_tile_desc &a, const ft_tile_desc &b) {
            if (a.ukernel_id != b.ukernel_id) return a.ukernel_id < b.ukernel_id;
            if (a.batch != b.batch) return a.batch < b.batch;
            if (a.m0 != b.m0) return a.m0 < b.m0;
            return a.n0 < b.n0;
        });
}

bool better(const Program &a, const Program &b) {      // Top-1 order: SIA, then fewer parts, fewer tiles, K1, K2
    if (a.sia_q != b.sia_q) return a.sia_q > b.sia_q;
    if (a.k_parts != b.k_parts) return a.k_parts < b.k_parts;
    if (a.tiles != b.tiles) return a.tiles < b.tiles;
    if (a.has_strips != b.has_strips) return !a.has_strips;
    if (a.k1 != b.k1) return a.k1 < b.k1;
    return a.k2 < b.k2;          // (strip variants of one program that tie: the first listed stays)
}

int level_of(const Program &p) { return p.in_bound ? 0 : 1; }

ftk::LaunchOrder launch_order_of(const ft_plan &plan) {
    ftk::LaunchOrder o;
    o.n[0] = plan.slot_first[1] - plan.slot_first[0];
    o.n[1] = (uint32_t)plan.descs.size() - plan.slot_first[1];
    for (int i = 0; i < 2; ++i) {
        o.first[i] = plan.slot_first[i];
        o.rows[i] = plan.slot_rows[i];
        o.cols[i] = plan.slot_cols[i];
        o.group[i] = plan.slot_group[i];
        o.m_base[i] = plan.slot_m0[i]; o.n_base[i] = plan.slot_n0[i];
        o.tm[i] = plan.slot_tm[i]; o.tn[i] = plan.slot_tn[i];
    }
    o.nx = plan.num_xcds;
    return o;
}

thread_local int g_last_hip_error = 0;

// owns a handle under construction: released to the caller on success, destroyed on every other path
// (error returns and exceptions alike)
struct PlanGuard {
    ft_plan *p;
    ~PlanGuard() { if (p) ft_plan_destroy(p); }
    ft_plan *release() { ft_plan *q = p; p = nullptr; return q; }
};
struct SetGuard {
    ft_ukset *p;
    ~SetGuard() { if (p) ft_ukset_destroy(p); }
    ft_ukset *release() { ft_ukset *q = p; p = nullptr; return q; }
};

// No exception may cross the C boundary: every entry point that allocates runs its body in here.
template <typename F> ft_status guarded(F &&body) {
    try {
        return body();
    } catch (const std::bad_alloc &) {
        return FT_ERR_OOM;
    } catch (...) {
        return FT_ERR_INVALID_ARG;
    }
}

constexpr size_t kPlanCacheMax = 65536;      // plans a uKernel set keeps for ft_plan_cached / grouped plans

}  // namespace

void ftd_set_hip_error(int e) { g_last_hip_error = e; }

extern "C" {

const char *ft_status_string(ft_status s) {
    switch (s) {
    case FT_OK: return "FT_OK";
    case FT_ERR_INVALID_ARG: return "FT_ERR_INVALID_ARG";
    case FT_ERR_UNSUPPORTED: return "FT_ERR_UNSUPPORTED";
    case FT_ERR_OUT_OF_RANGE: return "FT_ERR_OUT_OF_RANGE";
    case FT_ERR_NO_COVER: return "FT_ERR_NO_COVER";
    case FT_ERR_HIP: return "FT_ERR_HIP";
    case FT_ERR_OOM: return "FT_ERR_OOM";
    default: return "FT_ERR_UNKNOWN";
    }
}

int32_t ft_last_hip_error(void) { return g_last_hip_error; }

ft_status ft_hw_default_gfx950(ft_hw_model *out) {
    if (!out) return FT_ERR_INVALID_ARG;
    hw_defaults(out);
    return FT_OK;
}

ft_status ft_tuning_default(ft_tuning *out) {
    if (!out) return FT_ERR_INVALID_ARG;
    tuning_defaults(out);
    return FT_OK;
}

ft_status ft_op_register(const ft_op_desc *desc, ft_op **out) {
    if (!desc || !out || desc->struct_size != sizeof(ft_op_desc)) return FT_ERR_INVALID_ARG;
    const ft_op_desc &d = *desc;
    if (d.kind > FT_OP_CONV2D || d.dtype > FT_BF16) return FT_ERR_INVALID_ARG;
    if (d.out_dtype > FT_OUT_SAME || d.epilogue > FT_EPI_BIAS) return FT_ERR_INVALID_ARG;
    if (d.b_layout > FT_B_NK || (d.b_layout == FT_B_NK && d.kind == FT_OP_CONV2D)) return FT_ERR_INVALID_ARG;
    if (d.kind == FT_OP_CONV2D) {
        if (!d.c_in || !d.c_out || !d.r || !d.s || !d.stride) return FT_ERR_INVALID_ARG;
        if (d.m_lo > d.m_hi) return FT_ERR_INVALID_ARG;
        if ((uint64_t)d.r * d.s * d.c_in >= (1ull << 31)) return FT_ERR_UNSUPPORTED;
    } else {
        if (d.m == 0 && d.m_lo > d.m_hi) return FT_ERR_INVALID_ARG;
        if (d.n == 0 && d.n_lo > d.n_hi) return FT_ERR_INVALID_ARG;
        if (d.k == 0 && d.k_lo > d.k_hi) return FT_ERR_INVALID_ARG;
    }
    ft_op *op = new (std::nothrow) ft_op;
    if (!op) return FT_ERR_OOM;
    op->d = d;
    *out = op;
    return FT_OK;
}

void ft_op_destroy(ft_op *op) { delete op; }

static ft_status ukernels_derive_impl(const ft_op *op, const ft_hw_model *hw, const ft_tuning *tuning, ft_ukset **out);
ft_status ft_ukernels_derive(const ft_op *op, const ft_hw_model *hw, const ft_tuning *tuning, ft_ukset **out) {
    return guarded([&] { return ukernels_derive_impl(op, hw, tuning, out); });
}
static ft_status ukernels_derive_impl(const ft_op *op, const ft_hw_model *hw, const ft_tuning *tuning, ft_ukset **out) {
    if (!op || !out) return FT_ERR_INVALID_ARG;
    if (hw && hw->struct_size != sizeof(ft_hw_model)) return FT_ERR_INVALID_ARG;
    if (tuning && tuning->struct_size != sizeof(ft_tuning)) return FT_ERR_INVALID_ARG;
    ft_ukset *set = new (std::nothrow) ft_ukset;
    if (!set) return FT_ERR_OOM;
    SetGuard set_guard{set};
    set->op = op->d;
    if (hw) set->hw = *hw; else hw_defaults(&set->hw);
    if (tuning) set->t = *tuning; else tuning_defaults(&set->t);
    const ft_hw_model &h = set->hw;
    const ft_tuning &t = set->t;
    if (!h.num_cus || !h.wave_size || h.regs_per_lane < 4 || !h.mfma_flops_per_clk_per_cu || !h.bw_global_bytes_per_clk_per_cu ||
        !h.bw_lds_bytes_per_clk_per_cu || !t.zeta || !t.psi_den || t.sia_form > FT_SIA_PRODUCT ||
        (t.sia_form == FT_SIA_PRODUCT && (t.c0 > 4 || t.c1 > 4 || t.c2 > 4))) {
        return FT_ERR_INVALID_ARG;
    }
    Gemm sv = static_view(op->d);
    uint64_t kref = sv.k ? sv.k : op->d.k_hi;
    if (kref == 0) kref = 1;

    // HardwareAlign: RegTileRule (per-wave accumulator tiles built from MFMA shapes) x
    // SmemTileRule (wave grids; tk = one 128-byte line of 16-bit elements)
    std::vector<uint64_t> ms, ns;
    {
        const bool both = sv.m == 0 && sv.n == 0;
        const uint64_t cap = both ? 48 : 256;
        if (sv.m) ms.assign(1, sv.m); else axis_samples(op->d.m_lo, op->d.m_hi, cap, ms);
        if (sv.n) ns.assign(1, sv.n); else axis_samples(op->d.n_lo, op->d.n_hi, cap, ns);
    }
    std::vector<char> kept, psi_ok;
    static const uint32_t sizes[4] = {16, 32, 64, 128};
    // wave grids over (rows, columns, reduce axis); the split-k grid lets each wave own the whole
    // tile and a quarter of k (accumulator tiles of 1024..4096 elements only)
    // (gk = 2: the standard grids again as two teams of four waves that take alternate k-tiles, Matmul
    // and Conv2d only: grouped batched launches run workgroups of four waves)
    // (gm * gn = 8: eight waves, two per SIMD, on the same k-tiles -- the large tiles at half the accumulator
    // registers per wave)
    static const uint32_t grids[9][3] = {{1, 4, 1}, {2, 2, 1}, {4, 1, 1}, {1, 1, 4}, {1, 4, 2}, {2, 2, 2}, {4, 1, 2}, {2, 4, 1}, {4, 2, 1}};
    for (uint32_t wm : sizes)
        for (uint32_t wn : sizes) {
            uint32_t mfma;
            if (wm == 16 && wn <= 64) mfma = 1;
            else if (wm >= 32 && wn >= 32 && wm <= 2 * wn && wn <= 2 * wm) mfma = 0;
            else continue;
            for (auto &g : grids) {
                uint32_t gm = g[0], gn = g[1], gk = g[2], tk = FT_TK;
                uint32_t tm = gm * wm, tn = gn * wn;
                // (B as [N][K]: bodies of the four-wave standard grids only)
                if (op->d.b_layout == FT_B_NK && (gk != 1 || gm * gn != 4)) continue;
                if (gk == 4 && (wm * wn < 256 || wm * wn > 4096)) continue;
                if (gk == 2 && (!t.two_team_bodies || op->d.kind == FT_OP_BMM || ceil_div(kref, FT_TK) < 4)) continue;   // (each team wants at least two k-tiles)
                // (eight-wave grids: plain GEMMs only; the gather of the convolution and the batched walk
                // have no body of that shape)
                if (gm * gn == 8 && (!t.two_team_bodies || op->d.kind != FT_OP_MATMUL)) continue;
                if (ft_body_code(wm, wn, gm, gn, gk) < 0) continue;      // no compiled body
                // static space axes are divided evenly (after rounding to the MFMA granule)
                if (sv.m && ceil_by(sv.m, GRANULE) % tm) continue;
                if (sv.n && ceil_by(sv.n, GRANULE) % tn) continue;
                uint32_t acc = wm * wn / h.wave_size;
                uint32_t regs = acc + t.rest_regs;
                const uint32_t waves_per_simd = (gk == 2 || gm * gn == 8) ? 2 : 1;
                if (regs * waves_per_simd > h.regs_per_lane) continue;   // Eq. 4 at block.bound = 1
                // registers are granted in power-of-two fractions of the file (128, 256, 512)
                uint32_t budget = h.regs_per_lane / 4;
                while (budget < regs) budget *= 2;
                // LDS ring depth: as many k-tiles as fit in one workgroup's share of the LDS when
                // zeta workgroups are resident (2..8); every stage beyond the one being consumed
                // is global-memory traffic in flight (measured: a third stage for tiles that are
                // alone on the CU anyway gains nothing, the loop is bound by fetch bandwidth)
                // (a split-k workgroup keeps one ring per wave and is meant to own the CU's LDS)
                uint32_t stage_bytes = (tm + tn) * tk * ELT;
                // (two teams: one ring per team; the workgroup owns the CU's LDS as well)
                uint32_t stages = gk == 1 ? (h.lds_bytes_per_cu / t.zeta) / stage_bytes
                                          : h.lds_bytes_per_cu / (gk * stage_bytes);
                stages = std::max(MIN_STAGES, std::min(MAX_STAGES, stages));
                uint32_t lds = gk * stages * stage_bytes;
                if (lds > h.lds_bytes_per_cu) continue;                  // mem.IsOverflow
                u128 cn, cd;
                const uint32_t out_bytes = op->d.out_dtype == FT_OUT_SAME ? ELT : 4;
                compute_eff(tm, tn, gm, gn, gk, tk, kref, 1, out_bytes, h, &cn, &cd);
                psi_ok.push_back(cn * t.psi_den >= (u128)t.psi_num * cd ? 1 : 0);   // Eq. 6
                ft_ukernel_info u;
                std::memset(&u, 0, sizeof(u));
                u.struct_size = sizeof(u);
                u.tm = tm; u.tn = tn; u.tk = tk; u.wm = wm; u.wn = wn; u.gm = gm; u.gn = gn; u.gk = gk;
                u.mfma = mfma; u.stages = stages; u.lds_bytes = lds; u.acc_regs = acc; u.regs = regs;
                u.reg_budget = budget;
                u.max_wg_per_cu = std::min(std::min(h.lds_bytes_per_cu / lds, h.regs_per_lane / budget / waves_per_simd),
                                           h.max_waves_per_simd / waves_per_simd);
                u.cmr_q20 = (uint64_t)((cn << QBITS) / cd);
                compute_eff(tm, tn, gm, gn, gk, tk, kref, 2, out_bytes, h, &cn, &cd);
                u.cmr_shared_q20 = (uint64_t)((cn << QBITS) / cd);
                set->uk.push_back(u);
                // the tile count of a batched workload scales with a batch only known at run time:
                // with no upper bound given the workload filters cannot be evaluated and keep everything
                if (op->d.kind == FT_OP_BMM)
                    kept.push_back(op->d.batch_hi == 0 || passes_workload(tm, tn, ms, ns, op->d.batch_hi, h, t) ? 1 : 0);
                else
                    kept.push_back(passes_workload(tm, tn, ms, ns, 1, h, t) ? 1 : 0);
            }
        }
    // Eq. 6's threshold, unless no uKernel reaches it (a reduce axis of a few elements)
    if (std::find(psi_ok.begin(), psi_ok.end(), 1) != psi_ok.end()) {
        std::vector<ft_ukernel_info> f;
        std::vector<char> fk;
        for (size_t i = 0; i < set->uk.size(); ++i)
            if (psi_ok[i]) { f.push_back(set->uk[i]); fk.push_back(kept[i]); }
        set->uk.swap(f);
        kept.swap(fk);
    }
    // K.Filter: the uKernels that pass the workload filters; all of them if none does
    if (std::find(kept.begin(), kept.end(), 1) != kept.end()) {
        std::vector<ft_ukernel_info> f;
        for (size_t i = 0; i < set->uk.size(); ++i)
            if (kept[i]) f.push_back(set->uk[i]);
        set->uk.swap(f);
    }
    std::sort(set->uk.begin(), set->uk.end(), [](const ft_ukernel_info &a, const ft_ukernel_info &b) {
        uint64_t aa = (uint64_t)a.tm * a.tn, ab = (uint64_t)b.tm * b.tn;
        if (aa != ab) return aa > ab;
        if (a.tm != b.tm) return a.tm > b.tm;
        if (a.tn != b.tn) return a.tn > b.tn;
        if (a.tk != b.tk) return a.tk > b.tk;
        if (a.wm != b.wm) return a.wm > b.wm;
        if (a.wn != b.wn) return a.wn > b.wn;
        if (a.gk != b.gk) return a.gk < b.gk;
        return a.gm > b.gm;
    });
    set->cap_q = 0;
    for (size_t i = 0; i < set->uk.size(); ++i) {
        set->uk[i].id = (uint32_t)i;
        set->cap_q = std::max(set->cap_q, std::max(set->uk[i].cmr_q20, set->uk[i].cmr_shared_q20));
    }
    if (set->uk.empty()) return FT_ERR_NO_COVER;
    *out = set_guard.release();
    return FT_OK;
}

ft_status ft_ukset_size(const ft_ukset *set, uint32_t *n) {
    if (!set || !n) return FT_ERR_INVALID_ARG;
    *n = (uint32_t)set->uk.size();
    return FT_OK;
}

ft_status ft_ukset_get(const ft_ukset *set, uint32_t i, ft_ukernel_info *out) {
    if (!set || !out || i >= set->uk.size()) return FT_ERR_INVALID_ARG;
    *out = set->uk[i];
    return FT_OK;
}

void ft_ukset_destroy(ft_ukset *set) {
    if (!set) return;
    for (auto &kv : set->cache) ft_plan_destroy(kv.second);
    delete set;
}

static ft_status check_common(const ft_op *op, const ft_ukset *set, const ft_shape *shape, Resolved *r) {
    if (!op || !set || !shape || shape->struct_size != sizeof(ft_shape)) return FT_ERR_INVALID_ARG;
    if (std::memcmp(&op->d, &set->op, sizeof(ft_op_desc)) != 0) return FT_ERR_INVALID_ARG;
    ft_status st = resolve(op->d, *shape, r);
    if (st != FT_OK) return st;
    const uint64_t lim = 1ull << 31;      // 32-bit element offsets inside one batch entry
    if (op->d.kind == FT_OP_CONV2D) {
        if ((uint64_t)shape->img_n * shape->img_h * shape->img_w * op->d.c_in >= lim) return FT_ERR_UNSUPPORTED;
        if (shape->img_h >= 32768 || shape->img_w >= 32768) return FT_ERR_UNSUPPORTED;
    } else if (r->M * r->K >= lim) return FT_ERR_UNSUPPORTED;
    if (r->K * r->N >= lim || r->M * r->N >= lim || r->batch >= lim) return FT_ERR_UNSUPPORTED;
    if (r->N >= (1ull << 20)) return FT_ERR_UNSUPPORTED;   // byte offsets inside one wave tile of C stay below 2^31
    return FT_OK;
}

static ft_status plan_pool_impl(const ft_op *op, const ft_ukset *set, const ft_shape *shape, ft_pool_entry *out,
                                uint32_t cap, uint32_t *n);
ft_status ft_plan_pool(const ft_op *op, const ft_ukset *set, const ft_shape *shape, ft_pool_entry *out,
                       uint32_t cap, uint32_t *n) {
    return guarded([&] { return plan_pool_impl(op, set, shape, out, cap, n); });
}
static ft_status plan_pool_impl(const ft_op *op, const ft_ukset *set, const ft_shape *shape, ft_pool_entry *out,
                                uint32_t cap, uint32_t *n) {
    Resolved r;
    ft_status st = check_common(op, set, shape, &r);
    if (st != FT_OK) return st;
    if (!n || (cap && !out)) return FT_ERR_INVALID_ARG;
    *n = 0;
    if (r.batch == 0 || r.M == 0 || r.N == 0) return FT_OK;
    uint32_t tau = main_axis(op->d, r.M, r.N);
    std::vector<Program> pool;
    build_pool(*set, ceil_by(tau == 0 ? r.M : r.N, GRANULE), tau, pool);
    *n = (uint32_t)pool.size();
    for (size_t i = 0; i < pool.size() && i < cap; ++i) {
        Program p = pool[i];
        uint32_t c1 = p.part[0].count, c2 = p.nparts == 2 ? p.part[1].count : 0;
        evaluate(p, *set, r.batch, r.M, r.N, tau);
        ft_pool_entry &e = out[i];
        e.k1 = (uint32_t)p.k1; e.count1 = c1;
        e.k2 = p.k2 < 0 ? UINT32_MAX : (uint32_t)p.k2; e.count2 = c2;
        e.pad_q20 = p.pad_q; e.occ_q20 = p.occ_q; e.cmr_q20 = p.cmr_q;
        e.flags = (p.in_bound ? 1u : 0u) | (p.cross ? 2u : 0u) | (p.saturated ? 4u : 0u);
        e.sia_q20 = p.sia_q; e.n_tiles = p.tiles;
    }
    return FT_OK;
}

// set by ft_plan_create_grouped around its calls of ft_plan_create: the batch of the whole launch
static thread_local uint64_t tl_launch_batch = 0;

static ft_status plan_create_impl(const ft_op *op, const ft_ukset *set, const ft_shape *shape, uint32_t flags,
                                  const ft_forced_program *forced, ft_plan **out);
ft_status ft_plan_create(const ft_op *op, const ft_ukset *set, const ft_shape *shape, uint32_t flags,
                         const ft_forced_program *forced, ft_plan **out) {
    return guarded([&] { return plan_create_impl(op, set, shape, flags, forced, out); });
}
static ft_status plan_create_impl(const ft_op *op, const ft_ukset *set, const ft_shape *shape, uint32_t flags,
                                  const ft_forced_program *forced, ft_plan **out) {
    Resolved r;
    ft_status st = check_common(op, set, shape, &r);
    if (st != FT_OK) return st;
    if (!out) return FT_ERR_INVALID_ARG;
    const uint32_t mode = flags & FT_PLAN_MODE_MASK;
    if (mode > FT_PLAN_FORCED) return FT_ERR_INVALID_ARG;
    if (mode == FT_PLAN_FORCED && (!forced || forced->struct_size != sizeof(ft_forced_program)))
        return FT_ERR_INVALID_ARG;

    ft_plan *pl = new (std::nothrow) ft_plan;
    if (!pl) return FT_ERR_OOM;
    PlanGuard plan_guard{pl};
    pl->d_descs = nullptr; pl->d_ws = nullptr; pl->d_arrive = nullptr; pl->d_groups = nullptr;
    pl->op = op->d;
    pl->d_descs = nullptr;
    pl->d_ws = nullptr;
    pl->d_arrive = nullptr;
    pl->d_groups = nullptr;
    pl->grp_stage_bytes = 0; pl->grp_acc = 0; pl->grp_k_min = 0; pl->grp_rows_on_blocks = false;
    pl->grp_aligned = false; pl->grp_fast_lds = 0; pl->grp_fast_acc = 0;
    pl->ws_tile_stride = 0;
    pl->device = -1;
    pl->num_xcds = set->hw.num_xcds ? set->hw.num_xcds : 1;
    pl->img_h = shape->img_h; pl->img_w = shape->img_w; pl->out_p = r.P; pl->out_q = r.Q;
    for (int i = 0; i < 4; ++i) { pl->slot_id[i] = 0; pl->slot_code[i] = 0; pl->slot_stages[i] = MIN_STAGES; }
    pl->n_slots = 0;
    pl->table_order = false;
    pl->two_teams = false;
    for (int i = 0; i < 2; ++i) {
        pl->slot_first[i] = 0; pl->slot_rows[i] = pl->slot_cols[i] = pl->slot_group[i] = 1;
        pl->slot_m0[i] = pl->slot_n0[i] = pl->slot_tm[i] = pl->slot_tn[i] = 0;
    }
    ft_plan_stats &s = pl->st;
    std::memset(&s, 0, sizeof(s));
    s.struct_size = sizeof(s);
    uint32_t tau = main_axis(op->d, r.M, r.N);
    s.tau = tau;
    s.batch = (uint32_t)r.batch; s.m = (uint32_t)r.M; s.n = (uint32_t)r.N; s.k = (uint32_t)r.K;
    s.useful_elems = r.batch * r.M * r.N;
    s.k_parts = 1;
    if (r.batch == 0 || r.M == 0 || r.N == 0) {           // empty input: empty plan
        *out = plan_guard.release();
        return FT_OK;
    }

    // programs are scored for the batch the launch as a whole has (a group of a grouped launch shares
    // the device with the other groups); the table is emitted for the shape's own batch
    const uint64_t eval_batch = tl_launch_batch ? std::max<uint64_t>(r.batch, tl_launch_batch) : r.batch;
    Program best{};
    if (mode == FT_PLAN_PAD_BASELINE) {
        // pad every dynamic axis up to the largest uKernel of the set (Fig. 2)
        const ft_ukernel_info &u = set->uk[0];
        uint64_t Hp = ceil_by(tau == 0 ? r.M : r.N, ext(u, tau));
        best.nparts = 1;
        best.part[0] = {0u, (uint32_t)(Hp / ext(u, tau))};
        best.k1 = 0; best.k2 = -1;
        evaluate(best, *set, eval_batch, r.M, r.N, tau);
        s.pool_size = 1;
        s.level = (uint32_t)level_of(best);
    } else if (mode == FT_PLAN_FORCED) {
        uint64_t Hp = ceil_by(tau == 0 ? r.M : r.N, GRANULE);
        if (forced->k1 >= set->uk.size() || forced->count1 == 0) return FT_ERR_INVALID_ARG;
        uint64_t total = (uint64_t)forced->count1 * ext(set->uk[forced->k1], tau);
        best.nparts = 1;
        best.part[0] = {forced->k1, forced->count1};
        best.k1 = forced->k1; best.k2 = -1;
        if (forced->count2) {
            if (forced->k2 >= set->uk.size() || forced->k2 == forced->k1) return FT_ERR_INVALID_ARG;
            total += (uint64_t)forced->count2 * ext(set->uk[forced->k2], tau);
            if (eight_waves(set->uk[forced->k1]) != eight_waves(set->uk[forced->k2])) return FT_ERR_INVALID_ARG;
            best.nparts = 2;
            best.part[1] = {forced->k2, forced->count2};
            best.k2 = forced->k2;
        }
        if (total != Hp) return FT_ERR_NO_COVER;
        // parts per tile: as asked, cut down to the k-tiles there are (no empty part); 1 if a
        // constituent has no registers left for the exchange
        uint32_t parts = 1;
        if (forced->k_parts > 1) {
            if (forced->k_parts > 64) return FT_ERR_INVALID_ARG;
            bool room = op->d.kind != FT_OP_CONV2D && r.K % 8 == 0 && r.N % 8 == 0;    // the split runs in the LDS-DMA Matmul bodies only
            for (uint32_t i = 0; i < best.nparts; ++i)
                room = room && set->uk[best.part[i].id].acc_regs <= FT_KPART_ACC_MAX && !eight_waves(set->uk[best.part[i].id]);
            if (room) {
                const uint64_t nk = std::max<uint64_t>(ceil_div(r.K, FT_TK), 1);
                const uint64_t per = ceil_div(nk, std::min<uint64_t>(forced->k_parts, nk));
                parts = (uint32_t)ceil_div(nk, per);
            }
        }
        evaluate(best, *set, eval_batch, r.M, r.N, tau, parts, r.K);
        s.pool_size = 1;
        s.level = (uint32_t)level_of(best);
    } else {
        std::vector<Program> pool;
        build_pool(*set, ceil_by(tau == 0 ? r.M : r.N, GRANULE), tau, pool);
        if (pool.empty()) {
            // Alg. 2 found nothing (main axis shorter than every extent the static axes admit):
            // pad it up to the uKernel with the smallest main-axis extent (first in set order)
            uint64_t Hp = ceil_by(tau == 0 ? r.M : r.N, GRANULE);
            size_t pick = 0;
            for (size_t i = 1; i < set->uk.size(); ++i)
                if (ext(set->uk[i], tau) < ext(set->uk[pick], tau)) pick = i;
            Program p{};
            p.nparts = 1;
            p.part[0] = {(uint32_t)pick, (uint32_t)ceil_div(Hp, ext(set->uk[pick], tau))};
            p.k1 = (int64_t)pick; p.k2 = -1;
            pool.push_back(p);
        }
        // Occupancy rescue (Matmul): every program is also scored with its tiles split over
        // 2, 3, ... workgroups along the reduce axis, where that is allowed
        s.pool_size = (uint32_t)pool.size();
        {
            std::vector<Program> scored;
            scored.reserve(pool.size());
            // Two dynamic space axes: every program is also scored with second-axis strips
            const Gemm sv = static_view(op->d);
            const bool two_axes = sv.m == 0 && sv.n == 0 && set->t.second_axis_strips != 0;
            const uint64_t Wp = ceil_by(tau == 0 ? r.N : r.M, GRANULE);
            std::vector<Program> variants;
            for (Program &p : pool) {
                if (two_axes) {                       // (before evaluate: it may reorder the parts)
                    variants.clear();
                    strip_variants(p, *set, Wp, tau, variants);
                }
                evaluate(p, *set, eval_batch, r.M, r.N, tau);
                scored.push_back(p);
                // (the split runs in the LDS-DMA bodies only: rows of 16-byte chunks, K and N multiples of 8)
                if (op->d.kind == FT_OP_MATMUL && r.K % 8 == 0 && r.N % 8 == 0)
                    for (uint32_t kp : kPartChoices) {
                        if (kp == 1 || !split_allowed(p, *set, r.K, kp)) continue;
                        Program q = p;
                        evaluate(q, *set, eval_batch, r.M, r.N, tau, kp, r.K);
                        scored.push_back(q);
                    }
                if (two_axes)
                    for (Program &q : variants) {
                        evaluate(q, *set, eval_batch, r.M, r.N, tau);
                        scored.push_back(q);
                    }
            }
            pool.swap(scored);
        }
        int lvl = 2;
        for (const Program &p : pool) lvl = std::min(lvl, level_of(p));
        bool have = false;
        for (const Program &p : pool) {
            // a program belongs to every level at or above its own
            if (level_of(p) > lvl) continue;
            if (!have || better(p, best)) { best = p; have = true; }
        }
        s.level = (uint32_t)lvl;
    }

    SlotGrid grid[2] = {{0, 1, 1, 0, 0, 0, 0}, {0, 1, 1, 0, 0, 0, 0}};
    emit(best, *set, r, tau, pl->descs, grid);
    if (best.nparts == 1) grid[1] = {(uint32_t)pl->descs.size(), 1, 1, 0, 0, 0, 0};
    for (int i = 0; i < 2; ++i) {
        pl->slot_first[i] = grid[i].first;
        pl->slot_rows[i] = grid[i].rows;
        pl->slot_cols[i] = grid[i].cols;
        pl->slot_m0[i] = grid[i].m_base; pl->slot_n0[i] = grid[i].n_base;
        pl->slot_tm[i] = grid[i].tm; pl->slot_tn[i] = grid[i].tn;
    }
    s.n_ukernels = best.nparts;
    uint32_t lds = 0, klass = 0;
    pl->table_order = best.has_strips;
    for (uint32_t i = 0; i < 2; ++i) { s.strip_ukernel_id[i] = UINT32_MAX; s.strip_tiles[i] = 0; s.main_tiles[i] = 0; }
    // slots 0, 1: the parts (the launch order is computed on their tile grids); 2, 3: strips
    auto set_slot = [&](uint32_t slot, const ft_ukernel_info &u) {
        if (eight_waves(u)) pl->two_teams = true;
        pl->slot_id[slot] = u.id;
        pl->slot_code[slot] = (uint32_t)ft_body_code(u.wm, u.wn, u.gm, u.gn, u.gk);
        pl->slot_stages[slot] = u.stages;
        lds = std::max(lds, u.lds_bytes);
        uint32_t by_model = 0;
        for (uint32_t b = set->hw.regs_per_lane / 4; b < u.reg_budget && by_model < FT_NUM_CLASSES - 1; b *= 2) ++by_model;
        klass = std::max<uint32_t>(klass, std::max<uint32_t>(by_model, (uint32_t)ft_class_of_acc((int)u.acc_regs)));
    };
    const uint64_t Wp_plan = ceil_by(tau == 0 ? r.N : r.M, GRANULE);
    for (uint32_t i = 0; i < best.nparts; ++i) {
        const ft_ukernel_info &u = set->uk[best.part[i].id];
        s.ukernel_id[i] = u.id;
        s.count_tau[i] = best.part[i].count;
        s.main_tiles[i] = (uint32_t)ceil_div(Wp_plan, ext(u, 1 - tau));
        set_slot(i, u);
        // Launch order: an XCD works on a window of consecutive tiles (its share of the table, at
        // most what its CUs hold at once).  Walk the grid in groups of g tile rows so that window is
        // a g x (window/g) block, with g chosen to minimise the A + B panel bytes the block touches.
        {
            const uint64_t nx = pl->num_xcds;
            const uint64_t share = ceil_div((uint64_t)grid[i].rows * grid[i].cols * r.batch, nx);
            const uint64_t held = (uint64_t)std::max<uint32_t>(1, set->hw.num_cus / (uint32_t)nx) * std::max<uint32_t>(1, u.max_wg_per_cu);
            const uint64_t window = std::max<uint64_t>(1, std::min(share, held));
            uint32_t best_g = 1;
            uint64_t best_cost = ~0ull;
            for (uint32_t g = 1; g <= 16; g *= 2) {
                const uint64_t rows_in = std::min<uint64_t>(g, grid[i].rows);
                const uint64_t cost = rows_in * u.tm + std::min<uint64_t>(ceil_div(window, rows_in), grid[i].cols) * u.tn;
                if (cost <= best_cost) { best_cost = cost; best_g = g; }
            }
            pl->slot_group[i] = best_g;
        }
    }
    if (best.nparts == 1) { pl->slot_id[1] = pl->slot_id[0]; pl->slot_code[1] = pl->slot_code[0]; pl->slot_stages[1] = pl->slot_stages[0]; }
    pl->n_slots = 2;
    for (uint32_t i = 0; i < 2; ++i) {                    // unused strip slots repeat slot 0
        pl->slot_id[2 + i] = pl->slot_id[0]; pl->slot_code[2 + i] = pl->slot_code[0]; pl->slot_stages[2 + i] = pl->slot_stages[0];
    }
    if (best.has_strips) {
        pl->n_slots = 4;
        for (uint32_t i = 0; i < best.nparts; ++i) {
            if (best.strip[i].id < 0) continue;
            const ft_ukernel_info &v = set->uk[(uint32_t)best.strip[i].id];
            s.strip_ukernel_id[i] = v.id;
            s.main_tiles[i] = best.strip[i].n_full;
            s.strip_tiles[i] = best.strip[i].n_strip;
            set_slot(2 + i, v);
        }
    }
    s.block_bound = best.block_bound;
    s.pad_q20 = best.pad_q; s.occ_q20 = best.occ_q; s.cmr_q20 = best.cmr_q; s.sia_q20 = best.sia_q;
    s.lds_bytes = lds;
    s.kernel_class = klass;
    s.n_tiles = pl->descs.size();
    s.covered_elems = r.batch * best.area;

    // Reduce-axis split: the planner's choice travels with the program; a forced program names its own
    {
        const uint64_t nk = std::max<uint64_t>(ceil_div(r.K, FT_TK), 1);
        uint32_t parts = best.k_parts ? best.k_parts : 1;
        const uint64_t per = ceil_div(nk, parts);
        uint32_t stride = 0;
        for (uint32_t i = 0; i < best.nparts; ++i) {
            const ft_ukernel_info &u = set->uk[best.part[i].id];
            stride = std::max(stride, u.tm * u.tn);
        }
        s.k_parts = parts;
        s.k_part_tiles = (uint32_t)per;
        s.workspace_bytes = parts > 1 ? s.n_tiles * parts * stride * 4ull : 0;
        pl->ws_tile_stride = stride;
    }

    // Launch order, second pass: for launches of modest size (up to 1024 tiles), count what the group heights chosen
    // above really make the XCDs fetch -- every XCD reads once the A row panels and the B column
    // panels of the tiles it runs together (windows of what its CUs hold at once) -- and take the
    // height, any integer up to 16, that fetches least.  The closed form above stays the starting
    // point and wins ties.
    if (!best.has_strips && pl->descs.size() <= 1024) {
        const uint32_t nx = pl->num_xcds;
        const size_t total = pl->descs.size();
        std::vector<uint32_t> seen_r, seen_c;              // window that last touched a row / column panel
        // which tiles of a constituent an XCD takes, as positions in the walk of its grid, does not
        // depend on the group heights: take them from the launch order once (a height of 1 walks the
        // grid in table order, so a position is a descriptor index less the constituent's first)
        std::vector<uint32_t> walk[2];                     // per constituent: positions, XCD by XCD
        std::vector<uint32_t> walk_end[2];                 // ... and where each XCD's run ends
        {
            ftk::LaunchOrder o = launch_order_of(*pl);
            o.group[0] = o.group[1] = 1;
            for (uint32_t x = 0; x < nx; ++x) {
                for (size_t b = x; b < total; b += nx) {
                    const ftk::TileOfWorkgroup w = ftk::tile_of_workgroup(o, (uint32_t)b);
                    walk[w.slot].push_back(w.index - o.first[w.slot]);
                }
                for (int i = 0; i < 2; ++i) walk_end[i].push_back((uint32_t)walk[i].size());
            }
        }
        auto fetched = [&](uint32_t slot, uint32_t g) -> uint64_t {
            const ft_ukernel_info &u = set->uk[best.part[slot].id];
            const size_t held = (size_t)std::max<uint32_t>(1, set->hw.num_cus / nx) * std::max<uint32_t>(1, u.max_wg_per_cu);
            const uint32_t rows = pl->slot_rows[slot], cols = pl->slot_cols[slot];
            // (batch entries as the walk numbers them: sized from the walk, not from the shape)
            const size_t entries = ((size_t)walk[slot].size() + (size_t)rows * cols - 1) / ((size_t)rows * cols);
            seen_r.assign(entries * rows, 0);
            seen_c.assign(entries * cols, 0);
            uint64_t cost = 0;
            uint32_t window = 0;
            size_t at = 0;
            for (uint32_t x = 0; x < nx; ++x) {
                size_t in_window = 0;
                ++window;
                for (; at < walk_end[slot][x]; ++at) {
                    uint32_t bi, row, col;
                    ftk::grouped_coords(walk[slot][at], rows, cols, g, &bi, &row, &col);
                    const size_t ri = (size_t)bi * rows + row, ci = (size_t)bi * cols + col;
                    if (seen_r[ri] != window) { seen_r[ri] = window; cost += u.tm; }
                    if (seen_c[ci] != window) { seen_c[ci] = window; cost += u.tn; }
                    if (++in_window == held) { ++window; in_window = 0; }
                }
            }
            return cost;
        };
        for (uint32_t i = 0; i < best.nparts; ++i) {
            if (pl->slot_rows[i] < 2 || pl->slot_cols[i] < 2) continue;
            uint32_t best_g = pl->slot_group[i];
            uint64_t best_cost = fetched(i, best_g);
            for (uint32_t g = 1; g <= std::min<uint32_t>(16, pl->slot_rows[i]); ++g) {
                if (g == pl->slot_group[i]) continue;
                const uint64_t c = fetched(i, g);
                if (c < best_cost) { best_cost = c; best_g = g; }
            }
            pl->slot_group[i] = best_g;
        }
    }

    // The kernels derive a workgroup's tile in closed form from the grids above instead of reading
    // the table: check that form against every descriptor; a plan that fails is walked in table
    // order (its workgroups then read their descriptors).
    if (!pl->table_order) {
        const ftk::LaunchOrder o = launch_order_of(*pl);
        const size_t total = pl->descs.size();
        std::vector<char> seen(total, 0);
        bool ok = true;
        for (size_t b = 0; b < total && ok; ++b) {
            const ftk::TileOfWorkgroup w = ftk::tile_of_workgroup(o, (uint32_t)b);
            if (w.index >= total || seen[w.index]) { ok = false; break; }
            seen[w.index] = 1;
            const ft_tile_desc &d = pl->descs[w.index];
            const uint32_t want_id = w.slot ? pl->slot_id[1] : pl->slot_id[0];
            ok = d.batch == w.batch && d.m0 == w.m0 && d.n0 == w.n0 && d.ukernel_id == want_id;
        }
        if (!ok) pl->table_order = true;
    }
    if (flags & FT_PLAN_TABLE_ORDER) pl->table_order = true;
    s.table_order = pl->table_order ? 1u : 0u;

    if (!(flags & FT_PLAN_HOST_ONLY)) {
        st = ftd_upload(pl);
        if (st != FT_OK) return st;
    }
    *out = plan_guard.release();
    return FT_OK;
}

static ft_status plan_create_grouped_impl(const ft_op *op, ft_ukset *set, const ft_shape *groups, uint32_t n_groups,
                                          uint32_t flags, ft_plan **out);
ft_status ft_plan_create_grouped(const ft_op *op, ft_ukset *set, const ft_shape *groups, uint32_t n_groups,
                                 uint32_t flags, ft_plan **out) {
    return guarded([&] { return plan_create_grouped_impl(op, set, groups, n_groups, flags, out); });
}
static ft_status plan_create_grouped_impl(const ft_op *op, ft_ukset *set, const ft_shape *groups, uint32_t n_groups,
                                          uint32_t flags, ft_plan **out) {
    if (!op || !set || !out || (n_groups && !groups) || n_groups >= (1u << 20)) return FT_ERR_INVALID_ARG;
    if (op->d.kind != FT_OP_BMM) return FT_ERR_UNSUPPORTED;
    const uint32_t mode = flags & FT_PLAN_MODE_MASK;
    if (mode != FT_PLAN_PATCHWORK && mode != FT_PLAN_PAD_BASELINE) return FT_ERR_INVALID_ARG;
    // an empty plan of the operator as the shell: the first group's shape with no batch entries
    ft_plan *pl = nullptr;
    {
        ft_shape none;
        std::memset(&none, 0, sizeof(none));
        none.struct_size = sizeof(none);
        if (n_groups) { none = groups[0]; none.batch = 0; }
        else { none.m = op->d.m ? 0 : op->d.m_lo; none.n = op->d.n ? 0 : op->d.n_lo; none.k = op->d.k ? 0 : op->d.k_lo; }
        ft_status st = ft_plan_create(op, set, &none, mode | FT_PLAN_HOST_ONLY, nullptr, &pl);
        if (st != FT_OK) return st;
    }
    PlanGuard plan_guard{pl};
    ft_plan_stats &s = pl->st;
    const uint32_t es_c = op->d.out_dtype == FT_OUT_SAME ? 2 : 4;
    uint64_t off_a = 0, off_b = 0, off_c = 0;
    pl->grp_rows_on_blocks = true;
    pl->grp_aligned = true;
    pl->grp_k_min = UINT32_MAX;
    s.batch = 0; s.m = 0; s.n = 0; s.k = 0; s.useful_elems = 0; s.covered_elems = 0;
    // The groups share the device: a group's program is the one the planner picks for its shape at
    // the batch of the whole launch (planned alone, a short group would be cut into small tiles to
    // fill a device that the other groups fill anyway); its descriptors are those of its own entries.
    // The batch is rounded up to a power of two so that launches of similar size share their programs:
    // a group's program is cached in the uKernel set under (mode, m, n, k, that batch) as the plan of
    // ONE batch entry, and every later launch replicates its tiles.
    uint64_t launch_batch = 0;
    for (uint32_t gi = 0; gi < n_groups; ++gi) launch_batch += groups[gi].batch;
    { uint64_t p2 = 1; while (p2 < launch_batch) p2 <<= 1; launch_batch = p2; }
    if (op->d.batch_hi && launch_batch > op->d.batch_hi) launch_batch = op->d.batch_hi;
    if (launch_batch > (1u << 30)) launch_batch = 1u << 30;
    // Operands are laid out in group order; the table lists the groups with the longest reduce axis
    // first (then the largest outputs), so that the workgroups with the most work start first and the
    // short ones fill the end of the launch (PV of 64 sequences: 68 -> 62 us, 89 -> 69 us).
    std::vector<uint32_t> by_work(n_groups);
    for (uint32_t gi = 0; gi < n_groups; ++gi) by_work[gi] = gi;
    std::vector<ft_group_rec> recs(n_groups);
    for (uint32_t gi = 0; gi < n_groups; ++gi) {
        Resolved rr;
        ft_status st = check_common(op, set, &groups[gi], &rr);
        if (st != FT_OK) return st;
        ft_group_rec &rec = recs[gi];
        rec.m = (uint32_t)rr.M; rec.n = (uint32_t)rr.N; rec.k = (uint32_t)rr.K; rec.batch = (uint32_t)rr.batch;
        rec.off_a = off_a; rec.off_b = off_b; rec.off_c = off_c;
        if (off_c * es_c % 64 || (uint64_t)rec.n * es_c % 64) pl->grp_rows_on_blocks = false;
        off_a += rr.batch * rr.M * rr.K;
        off_b += rr.batch * rr.K * rr.N;
        off_c += rr.batch * rr.M * rr.N;
    }
    pl->groups = recs;
    std::stable_sort(by_work.begin(), by_work.end(), [&](uint32_t a, uint32_t b) {
        if (recs[a].k != recs[b].k) return recs[a].k > recs[b].k;
        return (uint64_t)recs[a].m * recs[a].n > (uint64_t)recs[b].m * recs[b].n;
    });
    for (uint32_t oi = 0; oi < n_groups; ++oi) {
        const uint32_t gi = by_work[oi];
        const uint32_t own_batch = groups[gi].batch;
        const ft_plan *sub = nullptr;
        {
            ft_shape unit = groups[gi];
            unit.batch = own_batch ? 1 : 0;
            // validate the group's own shape first (its batch against batch_hi)
            Resolved rr;
            ft_status st = check_common(op, set, &groups[gi], &rr);
            if (st != FT_OK) return st;
            const std::vector<uint32_t> key = {mode | FT_PLAN_HOST_ONLY, 0xFFFFFFFFu, (uint32_t)launch_batch,
                                               unit.batch, unit.m, unit.n, unit.k};
            std::lock_guard<std::mutex> lock(set->cache_mu);
            auto it = set->cache.find(key);
            if (it == set->cache.end()) {
                ft_plan *made = nullptr;
                tl_launch_batch = launch_batch;
                st = ft_plan_create(op, set, &unit, mode | FT_PLAN_HOST_ONLY, nullptr, &made);   // (catches its own exceptions)
                tl_launch_batch = 0;
                if (st != FT_OK) return st;
                PlanGuard made_guard{made};
                if (set->cache.size() >= kPlanCacheMax) return FT_ERR_OOM;
                it = set->cache.emplace(key, made).first;
                made_guard.release();
            }
            sub = it->second;
        }
        ft_plan_stats g = sub->st;             // figures of one batch entry
        g.useful_elems *= own_batch;
        g.covered_elems *= own_batch;
        g.batch = own_batch;
        const ft_group_rec &rec = recs[gi];
        bool any = false;
        // the table of `own_batch` entries in canonical order: per uKernel, per batch entry, its tiles
        std::vector<ft_tile_desc> own;
        for (size_t i = 0; i < sub->descs.size();) {
            size_t j = i;
            while (j < sub->descs.size() && sub->descs[j].ukernel_id == sub->descs[i].ukernel_id) ++j;
            for (uint32_t b = 0; b < own_batch; ++b)
                for (size_t t = i; t < j; ++t) { own.push_back(sub->descs[t]); own.back().batch = b; }
            i = j;
        }
        for (ft_tile_desc d : own) {
            any = true;
            const ft_ukernel_info &u = set->uk[d.ukernel_id];
            int code = ft_body_code((int)u.wm, (int)u.wn, (int)u.gm, (int)u.gn, (int)u.gk);
            if (code < 0 || code > 0x7f || u.stages > 0xf) return FT_ERR_UNSUPPORTED;
            // a group whose rows end inside a 16-byte chunk runs the body that fixes such chunks up
            if (rec.k % 8 || (op->d.b_layout != FT_B_NK && rec.n % 8)) code = ft_ragged_code(code);

            d.flags = (d.flags & 1u) | ((uint32_t)code << 1) | (u.stages << 8) | (gi << 12);
            pl->descs.push_back(d);
            const int twin = ft_general_code(code);          // what the general bodies run for it
            pl->grp_stage_bytes = std::max(pl->grp_stage_bytes, ft_stage_bytes_of_code(twin));
            pl->grp_acc = std::max(pl->grp_acc, (uint32_t)ft_acc_of_code(twin));
            pl->grp_fast_lds = std::max(pl->grp_fast_lds, u.lds_bytes);
            pl->grp_fast_acc = std::max(pl->grp_fast_acc, u.acc_regs);
        }
        // LDS-DMA bodies, B stored [K][N]: rows of at least one 16-byte chunk (the reduce axis: see below)
        if (any && g.n < 8 && op->d.b_layout != FT_B_NK) pl->grp_aligned = false;
        if (any) pl->grp_k_min = std::min(pl->grp_k_min, g.k);
        s.batch += g.batch;
        s.m = std::max(s.m, g.m); s.n = std::max(s.n, g.n); s.k = std::max(s.k, g.k);
        s.useful_elems += g.useful_elems;
        s.covered_elems += g.covered_elems;
    }
    ft_group_rec total;                        // one past the last group: the buffers' sizes
    total.m = total.n = total.k = total.batch = 0;
    total.off_a = off_a; total.off_b = off_b; total.off_c = off_c;
    // LDS-DMA bodies fetch rows of fewer than 8 elements (a reduce axis shorter than one 16-byte chunk) as
    // they lie, together with what follows them, and clear the rest in LDS: fine inside the packed buffers,
    // where other rows and groups follow, except for a last row less than 8 elements from a buffer's end.
    for (const ft_group_rec &r : recs) {
        if (!r.batch || !r.m || !r.n || !r.k || r.k >= 8) continue;
        const uint64_t last_a = r.off_a + (uint64_t)r.batch * r.m * r.k - r.k;
        const uint64_t last_b = r.off_b + (uint64_t)r.batch * r.n * r.k - r.k;
        if (last_a + 8 > off_a || (op->d.b_layout == FT_B_NK && last_b + 8 > off_b)) pl->grp_aligned = false;
    }
    pl->groups.push_back(total);
    if (pl->descs.size() > UINT32_MAX / 2) return FT_ERR_UNSUPPORTED;
    s.n_tiles = pl->descs.size();
    s.n_ukernels = 0;                          // a program per group: no single pair of uKernels describes the plan
    s.k_parts = 1; s.k_part_tiles = 0; s.workspace_bytes = 0;
    s.lds_bytes = 2 * pl->grp_stage_bytes;
    s.kernel_class = pl->grp_acc <= 64 ? 1 : 2;
    s.table_order = 1;
    pl->table_order = true;
    if (!(flags & FT_PLAN_HOST_ONLY) && !pl->descs.empty()) {
        ft_status st = ftd_upload(pl);
        if (st != FT_OK) return st;
    }
    *out = plan_guard.release();
    return FT_OK;
}

ft_status ft_plan_group_layout(const ft_plan *plan, uint32_t group, uint64_t *off_a, uint64_t *off_b, uint64_t *off_c) {
    if (!plan || !off_a || !off_b || !off_c || group >= plan->groups.size()) return FT_ERR_INVALID_ARG;
    const ft_group_rec &r = plan->groups[group];
    *off_a = r.off_a; *off_b = r.off_b; *off_c = r.off_c;
    return FT_OK;
}

static ft_status plan_cached_impl(const ft_op *op, ft_ukset *set, const ft_shape *shape, uint32_t flags, const ft_plan **out);
ft_status ft_plan_cached(const ft_op *op, ft_ukset *set, const ft_shape *shape, uint32_t flags, const ft_plan **out) {
    return guarded([&] { return plan_cached_impl(op, set, shape, flags, out); });
}
static ft_status plan_cached_impl(const ft_op *op, ft_ukset *set, const ft_shape *shape, uint32_t flags, const ft_plan **out) {
    if (!op || !set || !shape || !out || shape->struct_size != sizeof(ft_shape)) return FT_ERR_INVALID_ARG;
    if ((flags & FT_PLAN_MODE_MASK) == FT_PLAN_FORCED) return FT_ERR_INVALID_ARG;
    const std::vector<uint32_t> key = {flags, shape->batch, shape->m, shape->n, shape->k,
                                       shape->img_n, shape->img_h, shape->img_w};
    std::lock_guard<std::mutex> lock(set->cache_mu);
    auto it = set->cache.find(key);
    if (it != set->cache.end()) {
        *out = it->second;
        return FT_OK;
    }
    if (set->cache.size() >= kPlanCacheMax) return FT_ERR_OOM;     // the cache is bounded: see ftuner.h
    ft_plan *pl = nullptr;
    ft_status st = ft_plan_create(op, set, shape, flags, nullptr, &pl);
    if (st != FT_OK) return st;
    PlanGuard plan_guard{pl};
    set->cache.emplace(key, pl);
    *out = plan_guard.release();
    return FT_OK;
}

ft_status ft_plan_descriptors(const ft_plan *plan, const ft_tile_desc **descs, uint64_t *n) {
    if (!plan || !descs || !n) return FT_ERR_INVALID_ARG;
    *descs = plan->descs.empty() ? nullptr : plan->descs.data();
    *n = plan->descs.size();
    return FT_OK;
}

ft_status ft_plan_launch_order(const ft_plan *plan, uint32_t *order, uint64_t cap, uint64_t *n) {
    if (!plan || !n || (cap && !order)) return FT_ERR_INVALID_ARG;
    // workgroups of the launch: the tiles, or for a plan walked in table order whole rounds of chunks
    const uint64_t total = plan->table_order ? ftk::table_grid((uint32_t)plan->descs.size(), plan->num_xcds) : plan->descs.size();
    *n = total;
    const ftk::LaunchOrder o = launch_order_of(*plan);
    for (uint64_t b = 0; b < total && b < cap; ++b) {
        if (plan->table_order) {
            const uint32_t t = ftk::table_index_of_workgroup((uint32_t)b, plan->num_xcds);
            order[b] = t < plan->descs.size() ? t : UINT32_MAX;          // idle workgroup
        } else {
            order[b] = ftk::tile_of_workgroup(o, (uint32_t)b).index;
        }
    }
    return FT_OK;
}

ft_status ft_plan_stats_get(const ft_plan *plan, ft_plan_stats *out) {
    if (!plan || !out) return FT_ERR_INVALID_ARG;
    *out = plan->st;
    return FT_OK;
}

void ft_plan_destroy(ft_plan *plan) {
    if (!plan) return;
    ftd_release(plan);
    delete plan;
}

}  // extern "C"
