"""Ragged attention batches through the C ABI: one grouped launch against the alternatives.

    python run_ragged.py [--seqs 64] [--heads 12] [--iters 20] [--draws 4] [--align 8]

A batch holds --seqs sequences whose lengths are drawn like the attention configuration's (the
paper's motivation, Sec. 1 / Fig. 1(b): sequence lengths in a batch differ widely and padding them to
the longest wastes most of the work).  For QK^T (K = 64, fp32 scores) and PV (N = 64) the batch is run
  grouped : ONE launch over per-sequence groups (ft_plan_create_grouped), every sequence at its own length
  padded  : one plain batched launch with every sequence padded to the longest of the batch
            (the planner's plan for that shape; useful flops are those of the true lengths)
  looped  : one plain launch per sequence, back to back on one stream
Operands are random bit patterns made on the device (timing only; tests/ checks grouped launches against
the oracle).  Buffers rotate over a ring so that launches do not find them in the caches.  Prints one
line per draw and operator and a JSON summary line.
"""
import argparse
import json
import math
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seqs", type=int, default=64)
    ap.add_argument("--heads", type=int, default=12)
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--draws", type=int, default=4)
    ap.add_argument("--ring-mb", type=float, default=600.0)
    ap.add_argument("--align", type=int, default=1, help="round every length up to a multiple of this (8: the "
                    "grouped launch then runs the LDS-DMA bodies)")
    ap.add_argument("--b-nk", action="store_true", help="Q K^T with the K matrices stored [L, 64] (FT_B_NK): the LDS-DMA "
                    "bodies at every length")
    a = ap.parse_args()
    rows = measure(a.seqs, a.heads, a.iters, a.draws, a.align, a.ring_mb, verbose=True, b_nk=a.b_nk)
    gm = lambda xs: math.exp(sum(math.log(x) for x in xs) / len(xs))
    print(json.dumps({"workload": "ragged attention batches, %d sequences x %d heads, lengths rounded up to multiples of %d, fp16 in, fp32 out" % (a.seqs, a.heads, a.align),
                      "speedup_vs_padded_geomean": round(gm([r["us_padded"] / r["us_grouped"] for r in rows]), 3),
                      "speedup_vs_looped_geomean": round(gm([r["us_looped"] / r["us_grouped"] for r in rows]), 3),
                      "rows": rows}))


def measure(seqs=64, heads=12, iters=20, draws=4, align=1, ring_mb=600.0, verbose=False, b_nk=False):
    """The measurement itself; returns one row per draw and operator."""
    import argparse as _ap
    a = _ap.Namespace(seqs=seqs, heads=heads, iters=iters, draws=draws, align=align, ring_mb=ring_mb)

    import torch
    import paper_2407_21418_amd as ft
    import synth_inputs as si

    assert torch.cuda.is_available(), "run_ragged needs a GPU"
    stream = torch.cuda.current_stream().cuda_stream
    hw = ft.ft_hw_query(0)
    H = a.heads
    ops = {
        "qk": ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, k=64, m_lo=0, m_hi=512, n_lo=0, n_hi=512,
                                              batch_hi=a.seqs * H, b_layout=ft.FT_B_NK if b_nk else ft.FT_B_KN)),
        "pv": ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_BMM, dtype=ft.FT_F16, n=64, m_lo=0, m_hi=512, k_lo=0, k_hi=512,
                                              batch_hi=a.seqs * H)),
    }
    sets = {k: ft.ft_ukernels_derive(op, hw, None) for k, op in ops.items()}

    def dims(which, L):
        return (L, L, 64) if which == "qk" else (L, 64, L)

    def rand16(n):
        return si.device_normal_bits((max(n, 8),), si.F16)

    def timed(plan, na, nb, nc):
        nsets = max(2, min(16, int(math.ceil(a.ring_mb * 1e6 / (2 * (na + nb) + 4 * nc)))))
        A = [rand16(na) for _ in range(nsets)]
        B = [rand16(nb) for _ in range(nsets)]
        Cs = [torch.empty(max(nc, 8), dtype=torch.float32, device="cuda") for _ in range(nsets)]
        pa, pb, pc = [t.data_ptr() for t in A], [t.data_ptr() for t in B], [t.data_ptr() for t in Cs]
        ft.ft_launch_timed(plan, pa, pb, pc, stream, 2)
        return ft.ft_launch_timed(plan, pa, pb, pc, stream, a.iters) * 1e3

    rows = []
    for draw in range(a.draws):
        lengths = [min(512, -(-L // a.align) * a.align) for L in si.ragged_lengths(draw, a.seqs)]
        Lmax = max(lengths)
        for which in ("qk", "pv"):
            op, uks = ops[which], sets[which]
            shape = (lambda L, b: ft.ft_shape(batch=b, m=L, n=L) if which == "qk" else ft.ft_shape(batch=b, m=L, k=L))
            flops = sum(2.0 * H * m * n * k for m, n, k in (dims(which, L) for L in lengths))
            grouped = ft.ft_plan_create_grouped(op, uks, [shape(L, H) for L in lengths])
            na, nb, nc = ft.ft_plan_group_layout(grouped, len(lengths))
            us_grouped = timed(grouped, na, nb, nc)
            m, n, k = dims(which, Lmax)
            padded = ft.ft_plan_create(op, uks, shape(Lmax, a.seqs * H))
            us_padded = timed(padded, a.seqs * H * m * k, a.seqs * H * k * n, a.seqs * H * m * n)
            # one launch per sequence on slices of one packed set (no ring: the operands of 64 launches
            # already exceed the L2s), timed as a whole with events
            plans = [ft.ft_plan_create(op, uks, shape(L, H)) for L in lengths]
            A, B, Cb = rand16(na), rand16(nb), torch.empty(max(nc, 8), dtype=torch.float32, device="cuda")
            offs = [ft.ft_plan_group_layout(grouped, i) for i in range(len(lengths))]

            def loop_once():
                for p, (oa, ob, oc) in zip(plans, offs):
                    ft.ft_launch(p, A.data_ptr() + 2 * oa, B.data_ptr() + 2 * ob, Cb.data_ptr() + 4 * oc, stream)
            loop_once()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(a.iters):
                loop_once()
            e1.record()
            e1.synchronize()
            us_looped = e0.elapsed_time(e1) * 1e3 / a.iters
            st = ft.ft_plan_stats_get(grouped)
            rows.append(dict(draw=draw, op=which, max_len=Lmax, mean_len=round(sum(lengths) / len(lengths), 1),
                             us_grouped=round(us_grouped, 1), us_padded=round(us_padded, 1), us_looped=round(us_looped, 1),
                             tflops_grouped=round(flops / us_grouped / 1e6, 1), tiles=int(st.n_tiles),
                             padded_work_ratio=round(a.seqs * Lmax * Lmax / max(1, sum(L * L for L in lengths)), 2)))
            r = rows[-1]
            if verbose:
                print("draw %d %s: %d seqs x %d heads, L mean %.0f max %d | grouped %7.1f us (%5.1f TFLOP/s useful, %d tiles) | "
                      "padded to max %7.1f us (x%.2f, %.2fx the work) | one launch per sequence %7.1f us (x%.2f)"
                      % (draw, which, a.seqs, H, r["mean_len"], Lmax, us_grouped, r["tflops_grouped"], r["tiles"], us_padded,
                         us_padded / us_grouped, r["padded_work_ratio"], us_looped, us_looped / us_grouped), flush=True)
    return rows


if __name__ == "__main__":
    main()
