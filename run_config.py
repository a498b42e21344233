"""Time one of the workload configurations through the C ABI: patchwork plan vs pad-to-library plan.

    python run_config.py --config 2     # attention BMM, B x 32 drawn lengths, QK^T and PV
    python run_config.py --config 3     # LLM token-count GEMMs (K = 4096, N in {4096, 11008})
    python run_config.py --config 4     # dynamic-resolution Conv2d

Shapes come from synth_inputs (the seeded draws of the configuration); operand values are random bit
patterns made on the device (timing only).  Operands rotate over buffer sets totalling about
--ring-mb so that launches do not find them in the caches.  Prints one line per group and a JSON
summary line: geomean TFLOP/s and GB/s (algorithmic bytes), padding waste, speed-up over the baseline.
"""
import argparse
import json
import math
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def geomean(xs):
    return math.exp(sum(math.log(x) for x in xs) / len(xs)) if xs else float("nan")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True, choices=[2, 3, 4])
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--ring-mb", type=float, default=600.0)
    ap.add_argument("--max-sets", type=int, default=48)
    ap.add_argument("--b-nk", action="store_true", help="config 2: hand the K matrices of Q K^T over as [L, 64] (FT_B_NK)")
    a = ap.parse_args()

    import torch
    import paper_2407_21418_amd as ft
    import synth_inputs as si

    stream = torch.cuda.current_stream().cuda_stream
    hw = ft.ft_hw_query(0)
    ops = {}

    def get_op(key, desc):
        if key not in ops:
            op = ft.ft_op_register(desc)
            ops[key] = (op, ft.ft_ukernels_derive(op, hw, None))
        return ops[key]

    def rand16(shape):
        return si.device_normal_bits(shape, si.BF16 if a.config == 3 else si.F16)

    def measure(op, uks, shape, a_shape, b_shape, c_elems, flops, bytes_alg):
        nsets = max(2, min(a.max_sets, int(math.ceil(a.ring_mb * 1e6 / bytes_alg))))
        A = [rand16(a_shape) for _ in range(nsets)]
        B = [rand16(b_shape) for _ in range(nsets)]
        Cs = [torch.empty(c_elems, dtype=torch.float32, device="cuda") for _ in range(nsets)]
        pa, pb, pc = [t.data_ptr() for t in A], [t.data_ptr() for t in B], [t.data_ptr() for t in Cs]
        out = {}
        for name, mode in (("patch", ft.FT_PLAN_PATCHWORK), ("base", ft.FT_PLAN_PAD_BASELINE)):
            plan = ft.ft_plan_create(op, uks, shape, mode)
            st = ft.ft_plan_stats_get(plan)
            ft.ft_launch_timed(plan, pa, pb, pc, stream, 2)
            ms = ft.ft_launch_timed(plan, pa, pb, pc, stream, a.iters)
            out[name] = dict(ms=ms, covered=st.covered_elems, useful=st.useful_elems, tiles=st.n_tiles)
        del A, B, Cs
        torch.cuda.empty_cache()
        return dict(flops=flops, bytes=bytes_alg, **{k + "_" + kk: vv for k, v in out.items() for kk, vv in v.items()})

    groups = {}
    if a.config == 2:
        lengths = si.config2_lengths()
        for Bsz in si.ATT_BATCH:
            nb = Bsz * si.ATT_HEADS
            for which in ("qk", "pv"):
                rows = []
                for L in lengths[Bsz]:
                    if which == "qk":
                        op, uks = get_op("qk", ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, k=64, m_lo=1, m_hi=512, n_lo=1, n_hi=512,
                                                            batch_hi=max(si.ATT_BATCH) * si.ATT_HEADS,
                                                            b_layout=ft.FT_B_NK if a.b_nk else ft.FT_B_KN))
                        M, N, K, shape = L, L, 64, ft.ft_shape(batch=nb, m=L, n=L)
                    else:
                        op, uks = get_op("pv", ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, n=64, m_lo=1, m_hi=512, k_lo=1, k_hi=512,
                                                            batch_hi=max(si.ATT_BATCH) * si.ATT_HEADS))
                        M, N, K, shape = L, 64, L, ft.ft_shape(batch=nb, m=L, k=L)
                    rows.append(measure(op, uks, shape, (nb, M, K), (nb, K, N), nb * M * N, 2.0 * nb * M * N * K,
                                        nb * (2 * (M * K + K * N) + 4 * M * N)))
                groups["B=%d %s" % (Bsz, which)] = rows
    elif a.config == 3:
        for N in si.LLM_N:
            op, uks = get_op(N, ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=ft.FT_BF16, n=N, k=si.LLM_K, m_lo=1, m_hi=8192))
            rows = []
            for M in si.config3_token_counts():
                rows.append(measure(op, uks, ft.ft_shape(m=M), (M, si.LLM_K), (si.LLM_K, N), M * N, 2.0 * M * N * si.LLM_K,
                                    2 * (M * si.LLM_K + si.LLM_K * N) + 4 * M * N))
            groups["N=%d" % N] = rows
    else:
        op, uks = get_op("conv", ft.ft_op_desc(kind=ft.FT_OP_CONV2D, dtype=ft.FT_F16, c_in=si.CONV_CIN, c_out=si.CONV_COUT,
                                                r=si.CONV_R, s=si.CONV_S, stride=1, pad=1, m_lo=1, m_hi=1 << 22))
        rows = []
        for res in si.CONV_RES:
            n, ci, co = si.CONV_BATCH, si.CONV_CIN, si.CONV_COUT
            M = n * res * res
            rows.append(measure(op, uks, ft.ft_shape(img_n=n, img_h=res, img_w=res), (n, res, res, ci), (3, 3, ci, co), M * co,
                                2.0 * M * co * 9 * ci, 2 * (M * ci + 9 * ci * co) + 4 * M * co))
        groups["conv 64->128 3x3"] = rows

    summary = {}
    for name, rows in groups.items():
        tf = geomean([r["flops"] / r["patch_ms"] / 1e9 for r in rows])
        tfb = geomean([r["flops"] / r["base_ms"] / 1e9 for r in rows])
        gbs = geomean([r["bytes"] / r["patch_ms"] / 1e6 for r in rows])
        waste = 100.0 * (1.0 - sum(r["patch_useful"] for r in rows) / sum(r["patch_covered"] for r in rows))
        wasteb = 100.0 * (1.0 - sum(r["base_useful"] for r in rows) / sum(r["base_covered"] for r in rows))
        tot, totb = sum(r["patch_ms"] for r in rows), sum(r["base_ms"] for r in rows)
        summary[name] = dict(n=len(rows), geomean_tflops=round(tf, 2), geomean_gbs=round(gbs, 1), baseline_geomean_tflops=round(tfb, 2),
                             padding_waste_pct=round(waste, 2), baseline_padding_waste_pct=round(wasteb, 2),
                             total_ms=round(tot, 4), baseline_total_ms=round(totb, 4), speedup_total=round(totb / tot, 3))
        print("%-18s n=%3d  %8.1f TFLOP/s geomean  %7.0f GB/s  waste %5.2f%% (baseline %5.2f%%)  total %.3f ms vs %.3f ms" % (
            name, len(rows), tf, gbs, waste, wasteb, tot, totb), flush=True)
    print(json.dumps({"config": a.config, "iters": a.iters, "groups": summary}), flush=True)


if __name__ == "__main__":
    main()
