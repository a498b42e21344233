#!/usr/bin/env python3
"""Benchmark of the dynamic-shape contraction path on one MI355X.

Workload (N=1): the BERT-base-shaped dynamic sweep -- for seq_len L in {5,17,33,64,77,100,128},
batch 16: [16L,768]x[768,768], [16L,768]x[768,3072], [16L,3072]x[3072,768]; fp16 inputs,
fp32 accumulate/output.  One "step" = one pass over the 21 GEMMs through plan (cached per
shape) + launch.  Steps are executed shape-major: each GEMM is launched `steps` times back to
back between two HIP events on the launch stream, so every GEMM gets its own time; the sum
over GEMMs is the time of one step.  With --graph the `steps` launches of a GEMM are captured
into a HIP graph and the timed region is one replay of it (measured: no gain over direct
launches on this machine).

Headline `value`: geomean over the 21 GEMMs of useful TFLOP/s with operands resident in HBM
but NOT in cache (each launch uses the next of a ring of buffer sets totalling > 600 MB).
The same measurement with a single, cache-warm buffer set is reported beside it as
`warm_cache`, the pad-to-library baseline plan as `pad_baseline`, the bucketed padding of serving
stacks (M rounded up to the next power of two) as `bucketed_baseline`, the latency of a single
launch followed by a wait as `single_launch_us_geomean`, and, as a second workload of the same library,
one ragged attention batch run as a single grouped launch (`ragged_attention`).

Prints ONE JSON line on stdout; per-GEMM details go to the JSON file named by --detail.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2516.6      # dense fp16/bf16 MFMA, 256 CU x 4096 flop/clk x 2.4 GHz
HBM_PEAK_GBS = 8000.0
RING_BYTES = 600e6             # > 256 MB Infinity Cache + 8 x 4 MB L2
REPEATS = 5                    # timed regions per GEMM and variant; the median is reported
# Bytes crossing the L2 <-> fabric boundary per launch of each dispatcher kernel (average over the cold
# launches of this sweep): counters cannot be read from inside this process, so the figures are those
# of the committed counter runs of this same file, kept with their commands and calibration in
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "ft_dispatch_traffic.json")


def measured_traffic(kernel):
    """L2-miss read + write-back bytes per launch of `kernel` from the committed counter profile, or None."""
    try:
        with open(TRAFFIC_TABLE) as f:
            k = json.load(f)["kernels"].get(kernel)
        return None if k is None else float(k["fetch_bytes"]) + float(k["write_bytes"])
    except (OSError, ValueError, KeyError):
        return None


def geomean(xs):
    return math.exp(sum(math.log(x) for x in xs) / len(xs))


def private_l2_floor_bytes(ft, np, plan, K, num_xcds):
    """Bytes one launch of this plan must move across the L2 <-> fabric boundary when every XCD has
    its own L2 and nothing is fetched twice by the same XCD: each XCD reads once the rows of A and the
    columns of B that its tiles touch (workgroup b runs on XCD b % num_xcds), and C is written once.
    Partial tiles of a reduce-axis split are not counted (the parts of a tile share an XCD)."""
    desc = np.frombuffer(ft.ft_plan_descriptors(plan), dtype=np.dtype(
        [("uk", "<u4"), ("batch", "<u4"), ("m0", "<u4"), ("n0", "<u4"), ("mv", "<u2"), ("nv", "<u2"), ("flags", "<u4")]))
    rows = [set() for _ in range(num_xcds)]
    cols = [set() for _ in range(num_xcds)]
    c_elems = 0
    for e, t in enumerate(ft.ft_plan_launch_order(plan)):
        if t == 0xFFFFFFFF:
            continue
        d = desc[t]
        x = e % num_xcds
        rows[x].add((int(d["m0"]), int(d["mv"])))
        cols[x].add((int(d["n0"]), int(d["nv"])))
        c_elems += int(d["mv"]) * int(d["nv"])

    def covered(spans):                               # length of the union of [start, start + len)
        n, end = 0, 0
        for a, l in sorted(spans):
            lo, hi = max(a, end), a + l
            if hi > lo:
                n += hi - lo
                end = hi
        return n
    read = sum(covered(rows[x]) + covered(cols[x]) for x in range(num_xcds)) * K * 2
    return read + 4 * c_elems


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true", help="time one HIP-graph replay of the launches instead of direct launches")
    ap.add_argument("--variants", default="cold,warm,base,out16,bucket,single,ragged",
                    help="comma list of the timed variants: cold (headline), warm (one buffer set), base "
                         "(pad-to-library plan), out16 (same sweep with C stored as fp16, reported beside the "
                         "headline), bucket (M padded to the next power of two, the planner's plan for that "
                         "shape), single (one launch between two events, median of 5), ragged (a ragged attention "
                         "batch as one grouped launch, informational); 'cold' alone is what the committed profiles run")
    ap.add_argument("--detail", default=os.path.join(ROOT, "gpurun_out", "bench_detail.json"))
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path shards by rows with no exchange step)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2407_21418_amd as ft
    import synth_inputs as si

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    side = torch.cuda.Stream()                      # graph capture needs a non-NULL stream
    stream = side.cuda_stream
    use_graph = args.graph
    variants = set(args.variants.split(","))
    assert "cold" in variants and variants <= {"cold", "warm", "base", "out16", "bucket", "single", "ragged"}, \
        "--variants: cold[,warm][,base][,out16][,bucket][,single][,ragged]"
    hw = ft.ft_hw_query(0)

    def timed_once(plan, pa, pb, pc, iters, graph=None):
        return ft.ft_launch_timed(plan, pa, pb, pc, stream, iters, graph=use_graph if graph is None else graph)

    def timed(plan, pa, pb, pc, iters, graph=None):
        """Median over REPEATS regions of `iters` back-to-back launches each (ms per launch)."""
        if graph is False:                                # warm-up calls
            return timed_once(plan, pa, pb, pc, iters, graph)
        return sorted(timed_once(plan, pa, pb, pc, iters, graph) for _ in range(REPEATS))[REPEATS // 2]

    shapes = si.config1_shapes()
    ops = {}
    rows = []
    t_plan_cold = 0.0
    for (M, N, K) in shapes:
        if (N, K) not in ops:
            t0 = time.perf_counter()
            op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=N, k=K, m_lo=1, m_hi=8192))
            uks = ft.ft_ukernels_derive(op, hw, None)
            ops[(N, K)] = (op, uks, time.perf_counter() - t0)
        op, uks, _ = ops[(N, K)]
        t0 = time.perf_counter()
        plan = ft.ft_plan_create(op, uks, ft.ft_shape(m=M), ft.FT_PLAN_PATCHWORK)
        t_plan_cold += time.perf_counter() - t0
        base = ft.ft_plan_create(op, uks, ft.ft_shape(m=M), ft.FT_PLAN_PAD_BASELINE)
        rows.append(dict(M=M, N=N, K=K, plan=plan, base=base))
        if "out16" in variants:                      # the same operator with a 16-bit C
            if (N, K, 16) not in ops:
                op16 = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_F16, n=N, k=K, m_lo=1, m_hi=8192,
                                                       out_dtype=ft.FT_OUT_SAME))
                ops[(N, K, 16)] = (op16, ft.ft_ukernels_derive(op16, hw, None), 0.0)
            op16, uks16, _ = ops[(N, K, 16)]
            rows[-1]["plan16"] = ft.ft_plan_create(op16, uks16, ft.ft_shape(m=M), ft.FT_PLAN_PATCHWORK)
        if "bucket" in variants:                     # what a serving stack does: pad M to the next power of two
            Mb = max(16, 1 << (M - 1).bit_length())
            rows[-1]["Mb"] = Mb
            rows[-1]["planb"] = ft.ft_plan_create(op, uks, ft.ft_shape(m=Mb), ft.FT_PLAN_PATCHWORK)

    # the same plans through the per-shape cache: what a serving loop pays per call once a shape was seen
    for r in rows:
        op, uks, _ = ops[(r["N"], r["K"])]
        ft.ft_plan_cached(op, uks, ft.ft_shape(m=r["M"]))
    t0 = time.perf_counter()
    for _ in range(50):
        for r in rows:
            op, uks, _ = ops[(r["N"], r["K"])]
            ft.ft_plan_cached(op, uks, ft.ft_shape(m=r["M"]))
    t_plan_cached_us = (time.perf_counter() - t0) * 1e6 / (50 * len(rows))

    per_class_time = {}
    per_class_flops = {}
    per_class_launches = {}
    per_class_bytes = {}
    per_class_floor = {}
    for r in rows:
        M, N, K = r["M"], r["N"], r["K"]
        p = si.config1_problem(M, N, K)
        A0 = torch.from_numpy(p["A"].view(np.int16)).cuda()
        B0 = torch.from_numpy(p["B"].view(np.int16)).cuda()
        bytes_alg = 2 * (M * K + K * N) + 4 * M * N
        flops = 2.0 * M * N * K
        n_sets = max(2, int(math.ceil(RING_BYTES / bytes_alg)))
        As = [A0] + [A0.clone() for _ in range(n_sets - 1)]
        Bs = [B0] + [B0.clone() for _ in range(n_sets - 1)]
        Cs = [torch.empty((M, N), dtype=torch.float32, device="cuda") for _ in range(n_sets)]
        pa, pb, pc = [t.data_ptr() for t in As], [t.data_ptr() for t in Bs], [t.data_ptr() for t in Cs]
        torch.cuda.synchronize()
        st = ft.ft_plan_stats_get(r["plan"])
        sb = ft.ft_plan_stats_get(r["base"])
        # warm-up (untimed), then exactly `steps` timed launches per variant
        timed(r["plan"], pa, pb, pc, max(1, args.warmup), graph=False)
        ms_cold = timed(r["plan"], pa, pb, pc, args.steps)
        ms_warm = ms_base = float("inf")
        if "warm" in variants:
            timed(r["plan"], pa[:1], pb[:1], pc[:1], max(1, args.warmup), graph=False)
            ms_warm = timed(r["plan"], pa[:1], pb[:1], pc[:1], args.steps)
        if "base" in variants:
            timed(r["base"], pa, pb, pc, max(1, args.warmup), graph=False)
            ms_base = timed(r["base"], pa, pb, pc, args.steps)
        ms_out16 = float("inf")
        if "out16" in variants:                      # C buffers are large enough for either type
            timed(r["plan16"], pa, pb, pc, max(1, args.warmup), graph=False)
            ms_out16 = timed(r["plan16"], pa, pb, pc, args.steps)
        ms_bucket = float("inf")
        if "bucket" in variants:                     # same GEMM with M padded to its bucket, the planner's own plan for it
            Mb = r["Mb"]
            nb = max(2, int(math.ceil(RING_BYTES / (2 * (Mb * K + K * N) + 4 * Mb * N))))
            Ab = [torch.zeros((Mb, K), dtype=torch.int16, device="cuda") for _ in range(nb)]
            for t in Ab:
                t[:M].copy_(A0)
            Cb = [torch.empty((Mb, N), dtype=torch.float32, device="cuda") for _ in range(nb)]
            qa, qb, qc = [t.data_ptr() for t in Ab], [Bs[i % n_sets].data_ptr() for i in range(nb)], [t.data_ptr() for t in Cb]
            timed(r["planb"], qa, qb, qc, max(1, args.warmup), graph=False)
            ms_bucket = timed(r["planb"], qa, qb, qc, args.steps)
            del Ab, Cb
        us_single = float("inf")
        if "single" in variants:                     # one launch between two events, then a wait: median of 5
            one = sorted(timed_once(r["plan"], pa[i + 1:i + 2], pb[i + 1:i + 2], pc[i + 1:i + 2], 1, graph=False) for i in range(5))
            us_single = one[2] * 1e3
        t_roof = max(flops / (MFMA_PEAK_TFLOPS * 1e12), bytes_alg / (HBM_PEAK_GBS * 1e9))
        r.update(ms_bucket=ms_bucket, tflops_bucket=flops / ms_bucket / 1e9, us_single=us_single)
        r.update(ms_cold=ms_cold, ms_warm=ms_warm, ms_base=ms_base, ms_out16=ms_out16, tflops_out16=flops / ms_out16 / 1e9,
                 flops=flops, bytes_alg=bytes_alg,
                 tflops_cold=flops / ms_cold / 1e9, tflops_warm=flops / ms_warm / 1e9,
                 tflops_base=flops / ms_base / 1e9, gbs_cold=bytes_alg / ms_cold / 1e6,
                 roof_frac_cold=t_roof * 1e3 / ms_cold, n_tiles=st.n_tiles, n_ukernels=st.n_ukernels,
                 kernel_class=st.kernel_class, useful=st.useful_elems, covered=st.covered_elems,
                 base_covered=sb.covered_elems, base_tiles=sb.n_tiles)
        two_team = st.n_ukernels > 0 and ft.ft_ukset_get(ops[(N, K)][1], st.ukernel_id[0]).gk == 2
        k = ("ft_dispatch_dt0_pp_c%d" if two_team else "ft_dispatch_dt0_c%d") % st.kernel_class
        r["kernel"] = k
        r["bytes_private_l2_floor"] = private_l2_floor_bytes(ft, np, r["plan"], K, hw.num_xcds)
        per_class_floor[k] = per_class_floor.get(k, 0.0) + r["bytes_private_l2_floor"] * args.steps
        per_class_time[k] = per_class_time.get(k, 0.0) + ms_cold * args.steps
        per_class_flops[k] = per_class_flops.get(k, 0.0) + flops * args.steps
        per_class_launches[k] = per_class_launches.get(k, 0) + args.steps
        per_class_bytes[k] = per_class_bytes.get(k, 0.0) + bytes_alg * args.steps
        if not args.no_cpu_baseline:                    # set 0 holds the seeded problem: checked against the oracle below
            timed_once(r["plan"], pa[:1], pb[:1], pc[:1], 1, graph=False)
            r["C0"] = Cs[0].cpu().numpy()
        del As, Bs, Cs
        torch.cuda.empty_cache()

    # attainable memory rates of this device beside the 8 TB/s of the roofline: plain streaming kernels over 1 GiB
    sbuf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    sbuf.fill_(1)
    torch.cuda.synchronize()
    stream_read, stream_write, stream_copy = ft.ft_stream_rate(sbuf.data_ptr(), sbuf.data_ptr() + (1 << 30), 1 << 30, 5, stream)
    del sbuf
    torch.cuda.empty_cache()

    # informational, beside the headline: a second workload of the same library, one ragged batch of
    # attention (64 sequences x 12 heads, one length each) as ONE grouped launch against padding every
    # sequence to the longest and against one launch per sequence
    ragged = None
    if "ragged" in variants:
        import run_ragged
        rr = run_ragged.measure(draws=1, iters=10)
        ragged = {r["op"]: {"grouped_us": r["us_grouped"], "padded_to_longest_us": r["us_padded"],
                            "one_launch_per_sequence_us": r["us_looped"], "useful_tflops": r["tflops_grouped"]} for r in rr}
        ragged["note"] = "64 sequences x 12 heads, lengths uniform on 1..512, fp16 in, fp32 out, cold ring; not the headline"

    ms_per_step = sum(r["ms_cold"] for r in rows)
    value = geomean([r["tflops_cold"] for r in rows])
    warm = geomean([r["tflops_warm"] for r in rows]) if "warm" in variants else 0.0
    basev = geomean([r["tflops_base"] for r in rows]) if "base" in variants else 0.0
    useful = sum(r["useful"] for r in rows)
    waste_patch = 100.0 * (1.0 - useful / sum(r["covered"] for r in rows))
    waste_base = 100.0 * (1.0 - useful / sum(r["base_covered"] for r in rows))
    dom = max(per_class_time, key=per_class_time.get)
    achieved = per_class_flops[dom] / per_class_time[dom] / 1e9          # TFLOP/s
    achieved_gbs = per_class_bytes[dom] / per_class_time[dom] / 1e6      # GB/s, algorithmic bytes
    # which roofline binds the dominant kernel's launches: the one that alone would take longer
    hbm_bound = per_class_bytes[dom] / HBM_PEAK_GBS / 1e9 > per_class_flops[dom] / MFMA_PEAK_TFLOPS / 1e12
    total_flops = sum(r["flops"] for r in rows)
    total_bytes = sum(r["bytes_alg"] for r in rows)

    out = {
        "metric": "geomean TFLOP/s & % MFMA peak over dynamic-shape sweep; padding waste %",
        "value": round(value, 3),
        "unit": "TFLOP/s (geomean over 21 GEMMs, useful flops, operands from HBM)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "repeats": REPEATS,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "configs[1]: BERT-base-shaped dynamic sweep, 21 GEMMs, M=16*L, L in "
                               "{5,17,33,64,77,100,128}, (K,N) in {(768,768),(768,3072),(3072,768)}",
                   "order": "shape-major: each GEMM launched `steps` times back to back, %d such regions, the median one reported" % REPEATS,
                   "launch": "one HIP-graph replay of the `steps` launches" if use_graph else "direct launches",
                   "buffers": "ring of buffer sets > 600 MB per GEMM (cold caches)"},
        "pct_mfma_peak_geomean": round(100.0 * value / MFMA_PEAK_TFLOPS, 3),
        "aggregate_tflops": round(total_flops / ms_per_step / 1e9, 3),
        "aggregate_hbm_gbs": round(total_bytes / ms_per_step / 1e6, 1),
        "roofline_frac_geomean": round(geomean([r["roof_frac_cold"] for r in rows]), 4),
        "padding_waste_pct": {"patchwork": round(waste_patch, 3), "pad_baseline": round(waste_base, 3)},
        "warm_cache": {"value": round(warm, 3), "pct_mfma_peak_geomean": round(100.0 * warm / MFMA_PEAK_TFLOPS, 3),
                       "ms_per_step": round(sum(r["ms_warm"] for r in rows), 5)} if "warm" in variants else None,
        "pad_baseline": {"value": round(basev, 3),
                         "ms_per_step": round(sum(r["ms_base"] for r in rows), 5)} if "base" in variants else None,
        "fp16_output": {"value": round(geomean([r["tflops_out16"] for r in rows]), 3),
                        "ms_per_step": round(sum(r["ms_out16"] for r in rows), 5),
                        "note": "same sweep, cold, C rounded to fp16 in the epilogue (not the headline: the "
                                "north star fixes fp32 output)"} if "out16" in variants else None,
        "bucketed_baseline": {"value": round(geomean([r["tflops_bucket"] for r in rows]), 3),
                              "ms_per_step": round(sum(r["ms_bucket"] for r in rows), 5),
                              "padding_waste_pct": round(100.0 * (1.0 - sum(r["M"] * r["N"] for r in rows) /
                                                                  sum(r["Mb"] * r["N"] for r in rows)), 3),
                              "note": "M padded to the next power of two (>= 16), the planner's own plan for the padded "
                                      "shape, useful flops of the true M; cold"} if "bucket" in variants else None,
        "single_launch_us_geomean": round(geomean([r["us_single"] for r in rows]), 3) if "single" in variants else None,
        "ragged_attention": ragged,
        "plan_ms_cold_total": round(t_plan_cold * 1e3, 3),
        "plan_us_cached_lookup": round(t_plan_cached_us, 2),
        "roofline": {"bound": "hbm" if hbm_bound else "mfma", "kernel": dom,
                     "achieved": round(achieved_gbs if hbm_bound else achieved, 3),
                     "peak": HBM_PEAK_GBS if hbm_bound else MFMA_PEAK_TFLOPS,
                     "unit": "GB/s" if hbm_bound else "TFLOP/s",
                     "frac": round(achieved_gbs / HBM_PEAK_GBS if hbm_bound else achieved / MFMA_PEAK_TFLOPS, 5),
                     "other_roof": {"bound": "mfma" if hbm_bound else "hbm",
                                    "achieved": round(achieved if hbm_bound else achieved_gbs, 3),
                                    "unit": "TFLOP/s" if hbm_bound else "GB/s",
                                    "frac": round(achieved / MFMA_PEAK_TFLOPS if hbm_bound else achieved_gbs / HBM_PEAK_GBS, 5)},
                     "traffic": measured_traffic(dom),
                     "traffic_note": "L2-miss read + write-back bytes per launch (rocprofv3 --pmc, copy-calibrated; "
                                     "Infinity Cache hits included) from profiles/ft_dispatch_traffic.json, "
                                     "algorithmic bytes per launch: %d" % round(per_class_bytes[dom] / per_class_launches[dom]),
                     "hbm_attainable_gbs": {"read": round(stream_read, 1), "write": round(stream_write, 1), "copy": round(stream_copy, 1),
                                            "note": "plain streaming kernels over 1 GiB (ft_stream_rate), this run"},
                     "frac_of_attainable": round(achieved_gbs / stream_copy, 5) if hbm_bound else None,
                     "traffic_floor_private_l2": round(per_class_floor[dom] / per_class_launches[dom]),
                     "traffic_floor_note": "bytes per launch if each of the 8 XCDs (private L2s) fetches the A rows and "
                                           "B columns of its own tiles exactly once and C is written once, from the "
                                           "plans' launch order; traffic above it is what the L2s re-fetch or the "
                                           "reduce-axis split exchanges",
                     "avg_launch_us": round(1e3 * per_class_time[dom] / per_class_launches[dom], 3),
                     "launches": per_class_launches[dom],
                     "note": "achieved = algorithmic bytes (hbm) or useful flops (mfma) of the launches that ran "
                             "this kernel / their event-timed duration (back-to-back launches on one stream, "
                             "gaps between kernels included); bound = the roofline that alone takes longer "
                             "for those launches"},
    }

    if not args.no_cpu_baseline:
        # the oracle as it stands, on the host cores: whole passes over the same 21 GEMMs until about
        # 10 s of oracle time have been spent (bounded at 30 s); per GEMM the mean over the passes
        from oracle import contraction as oc
        probs = [si.config1_problem(r["M"], r["N"], r["K"]) for r in rows]
        secs, passes = [0.0] * len(rows), 0
        while sum(secs) < 10.0 and passes < 64:
            for i, p in enumerate(probs):
                t1 = time.perf_counter()
                oc.matmul(p["A"], p["B"], si.F16)
                secs[i] += time.perf_counter() - t1
            passes += 1
            if sum(secs) > 30.0:
                break
        # every benched GEMM's output (buffer set 0, the seeded problem) against the oracle: max relative
        # error 2e-3 of fp32-accumulated fp16 products, per element against sum |a||b|
        worst = 0.0
        for r, p in zip(rows, probs):
            ref, refabs = oc.matmul(p["A"], p["B"], si.F16, want_abs=True)
            d = np.abs(r.pop("C0").astype(np.float64) - ref)
            worst = max(worst, float((d / (refabs + 1e-30)).max()))
            assert d.max() <= 2e-3 * np.abs(ref).max() and (d <= 2e-3 * refabs + 1e-30).all(), \
                "benched GEMM %dx%dx%d differs from the oracle" % (r["M"], r["N"], r["K"])
        out["verified"] = {"gemms": len(rows), "worst_error_over_sum_abs_products": worst, "tolerance": 2e-3}
        for r, s_ in zip(rows, secs):
            r["oracle_s"] = s_ / passes
        total = sum(secs)
        out["cpu_baseline"] = {
            "value": round(geomean([r["flops"] / r["oracle_s"] / 1e12 for r in rows]), 6),
            "unit": "TFLOP/s (geomean, fp64 oracle)", "cores": oc.num_threads(), "kind": "oracle",
            "sample": "%d passes over the 21 GEMMs of the same sweep, %.1f s of oracle time" % (passes, total),
            "aggregate_gflops": round(passes * sum(r["flops"] for r in rows) / total / 1e9, 2)}

    os.makedirs(os.path.dirname(args.detail), exist_ok=True)
    with open(args.detail, "w") as f:
        json.dump([{k: v for k, v in r.items() if k not in ("plan", "base", "plan16", "planb", "C0")} for r in rows], f, indent=1)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
