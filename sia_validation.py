#!/usr/bin/env python3
"""How good is the planner's Top-1?  (The analogue of the paper's check of its performance model,
Sec. 6.3 / Fig. 15: every program of the pool is run and compared with the model's choice.)

For each shape every program Alg. 2 puts in the pool is forced (FT_PLAN_FORCED) and timed on
operands that rotate through a ring larger than the caches; Matmul programs are also timed with
their tiles split over 2, 3, 4, 6, 8 workgroups along the reduce axis where the planner would
consider that split.  Reported per shape: the best time in the pool, the time of the plan the
planner picks by itself, their ratio; at the end the geomean of the ratios and the worst one.

    python sia_validation.py                 # 21 BERT-shaped GEMMs + 18 LLM-shaped ones
    python sia_validation.py --heldout       # 28 shapes the model constants were not fitted on
    python sia_validation.py --four-wave     # without the eight-wave two-team uKernels in the set
    ... --json sia.json                      # every timed program with its scores, for fitting

Prints a markdown table (kept under profiles/sia_validation.md).
"""
import argparse
import json
import math
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

KP_CHOICES = (2, 3, 4, 6, 8)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--heldout", action="store_true")
    ap.add_argument("--four-wave", action="store_true")
    ap.add_argument("--iters", type=int, default=30)
    ap.add_argument("--ring-mb", type=float, default=600.0)
    ap.add_argument("--json", default="")
    a = ap.parse_args()

    import torch
    import paper_2407_21418_amd as ft
    import synth_inputs as si

    stream = torch.cuda.current_stream().cuda_stream
    hw = ft.ft_hw_query(0)
    tuning = ft.ft_tuning_default()
    if a.four_wave:
        tuning.two_team_bodies = 0
    if a.heldout:
        shapes = [(M, N, K, ft.FT_F16) for (N, K) in ((1024, 1024), (2304, 768), (5120, 2048), (1536, 4096))
                  for M in (96, 200, 400, 777, 1500, 3000, 6000)]
    else:
        shapes = [(M, N, K, ft.FT_F16) for (M, N, K) in si.config1_shapes()] + \
                 [(M, N, 4096, ft.FT_BF16) for N in (4096, 11008) for M in (16, 45, 128, 300, 512, 1024, 2048, 4096, 8192)]
    ops, out, ratios = {}, [], []
    print("| M | N | K | programs timed | best in pool | us | planner's pick | us | best / pick |")
    print("|---|---|---|---|---|---|---|---|---|")
    for (M, N, K, dt) in shapes:
        if (N, K, dt) not in ops:
            op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dt, n=N, k=K, m_lo=1, m_hi=8192))
            ops[(N, K, dt)] = (op, ft.ft_ukernels_derive(op, hw, tuning))
        op, uks = ops[(N, K, dt)]
        infos = [ft.ft_ukset_get(uks, i) for i in range(ft.ft_ukset_size(uks))]
        bytes_alg = 2 * (M * K + K * N) + 4 * M * N
        nsets = max(2, int(math.ceil(a.ring_mb * 1e6 / bytes_alg)))
        A = [si.device_normal_bits((M, K), si.F16 if dt == ft.FT_F16 else si.BF16) for _ in range(nsets)]
        B = [si.device_normal_bits((K, N), si.F16 if dt == ft.FT_F16 else si.BF16) for _ in range(nsets)]
        C = [torch.empty((M, N), dtype=torch.float32, device="cuda") for _ in range(nsets)]
        pa, pb, pc = [t.data_ptr() for t in A], [t.data_ptr() for t in B], [t.data_ptr() for t in C]

        def timed(plan):
            ft.ft_launch_timed(plan, pa, pb, pc, stream, 3)
            return ft.ft_launch_timed(plan, pa, pb, pc, stream, a.iters) * 1e3

        pick_plan = ft.ft_plan_create(op, uks, ft.ft_shape(m=M), ft.FT_PLAN_PATCHWORK)
        ps = ft.ft_plan_stats_get(pick_plan)
        pick_key = (tuple(sorted((ps.ukernel_id[i], ps.count_tau[i]) for i in range(ps.n_ukernels))), ps.k_parts)
        nk = max(1, -(-K // 64))
        res = []
        for e in ft.ft_plan_pool(op, uks, ft.ft_shape(m=M)):
            us_ = [infos[e.k1]] + ([infos[e.k2]] if e.count2 else [])
            per_cu = min([tuning.zeta] + [u.max_wg_per_cu for u in us_])
            kps = [1] + [kp for kp in KP_CHOICES
                         if all(u.acc_regs <= 128 and u.gk != 2 and u.gm * u.gn != 8 for u in us_) and e.n_tiles * kp <= hw.num_cus * per_cu
                         and nk // kp >= tuning.k_part_min_tiles and -(-nk // -(-nk // kp)) == kp and kp <= tuning.k_parts_max]
            for kp in kps:
                fp = ft.ft_forced_program(k1=e.k1, count1=e.count1, k2=(e.k2 if e.count2 else 0), count2=e.count2, k_parts=kp)
                pl = ft.ft_plan_create(op, uks, ft.ft_shape(m=M), ft.FT_PLAN_FORCED, fp)
                st = ft.ft_plan_stats_get(pl)
                if st.k_parts != kp:
                    continue
                key = (tuple(sorted([(e.k1, e.count1)] + ([(e.k2, e.count2)] if e.count2 else []))), kp)
                us_sorted = [infos[uid] for uid, _ in key[0]]
                res.append(dict(parts=[list(p) for p in key[0]], kp=kp, us=timed(pl), sia=st.sia_q20, tiles=int(st.n_tiles),
                                pick=key == pick_key,
                                uk=[dict(tm=u.tm, tn=u.tn, wm=u.wm, wn=u.wn, gm=u.gm, gn=u.gn, gk=u.gk, stages=u.stages) for u in us_sorted]))
        best = min(res, key=lambda r: r["us"])

        def name(r):
            s = " + ".join("%dx(%dx%d w%dx%d g%dx%dx%d)" % (c, u["tm"], u["tn"], u["wm"], u["wn"], u["gm"], u["gn"], u["gk"]) for (_, c), u in zip(r["parts"], r["uk"]))
            return s + (" / %d parts" % r["kp"] if r["kp"] > 1 else "")
        pk = [r for r in res if r["pick"]]
        us_pick = pk[0]["us"] if pk else timed(pick_plan)          # the same program, timed in its turn
        pick_name = name(pk[0]) if pk else "(not in the timed pool)"
        ratio = min(1.0, best["us"] / us_pick)
        ratios.append(ratio)
        print("| %d | %d | %d | %d | %s | %.2f | %s | %.2f | %.3f |" % (M, N, K, len(res), name(best), best["us"], pick_name, us_pick, ratio), flush=True)
        out.append(dict(M=M, N=N, K=K, dtype=dt, us_pick=us_pick, programs=res))
        del A, B, C
        torch.cuda.empty_cache()
    gm = math.exp(sum(math.log(r) for r in ratios) / len(ratios))
    print("\ngeomean of best-in-pool / pick over %d shapes: %.3f, worst %.3f" % (len(ratios), gm, min(ratios)))
    if a.json:
        os.makedirs(os.path.dirname(os.path.abspath(a.json)), exist_ok=True)
        json.dump(out, open(a.json, "w"))


if __name__ == "__main__":
    main()
