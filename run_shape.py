"""Time one Matmul shape through the C ABI (plan + repeated launch); used for profiling.

    python run_shape.py --m 8192 --n 4096 --k 4096 --dtype bf16 --iters 20
    ... --force 256,256,128,128     # force the single-uKernel program (tm,tn,wm,wn), M % tm == 0
    ... --baseline                  # the pad-to-library plan

Prints one line: shape, program, tiles, microseconds per launch, TFLOP/s, GB/s (algorithmic bytes).
"""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--m", type=int, required=True)
    ap.add_argument("--n", type=int, required=True)
    ap.add_argument("--k", type=int, required=True)
    ap.add_argument("--dtype", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--iters", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--force", default="")
    ap.add_argument("--k-parts", type=int, default=0, help="with --force: workgroups per tile along the reduce axis")
    ap.add_argument("--waves", type=int, default=4, choices=[4, 8], help="with --force: 8 picks the eight-wave grid of that tile")
    ap.add_argument("--teams", type=int, default=1, choices=[1, 2], help="with --force: 2 picks the eight-wave two-team uKernel of that tile")
    ap.add_argument("--baseline", action="store_true")
    ap.add_argument("--zeta", type=int, default=0, help="override the tuning's zeta (workgroups per CU)")
    ap.add_argument("--ring-mb", type=float, default=0.0, help="rotate over buffer sets totalling this many MB")
    ap.add_argument("--copy-mb", type=float, default=0.0,
                    help="also run a plain device copy of this many MB (calibrates FETCH_SIZE / WRITE_SIZE)")
    a = ap.parse_args()

    import torch
    import paper_2407_21418_amd as ft
    import synth_inputs as si

    dt = ft.FT_F16 if a.dtype == "f16" else ft.FT_BF16
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dt, n=a.n, k=a.k, m_lo=1, m_hi=max(8192, a.m)))
    tuning = None
    if a.zeta:
        tuning = ft.ft_tuning_default()
        tuning.zeta = a.zeta
    uks = ft.ft_ukernels_derive(op, ft.ft_hw_query(0), tuning)
    mode, forced = (ft.FT_PLAN_PAD_BASELINE if a.baseline else ft.FT_PLAN_PATCHWORK), None
    if a.force:
        want = tuple(int(x) for x in a.force.split(","))
        ids = [i for i in range(ft.ft_ukset_size(uks))
               if (lambda u: (u.tm, u.tn, u.wm, u.wn) == want and (u.gk == 2) == (a.teams == 2) and u.gm * u.gn == (8 if a.waves == 8 else 4))(ft.ft_ukset_get(uks, i))]
        if not ids:
            raise SystemExit("uKernel %s is not in the derived set" % (want,))
        mode, forced = ft.FT_PLAN_FORCED, ft.ft_forced_program(k1=ids[0], count1=-(-a.m // want[0] * want[0] // want[0]))
        forced.count1 = ((a.m + 15) // 16 * 16) // want[0]
        forced.k_parts = a.k_parts
    plan = ft.ft_plan_create(op, uks, ft.ft_shape(m=a.m), mode, forced)
    st = ft.ft_plan_stats_get(plan)
    bytes_alg = 2 * (a.m * a.k + a.k * a.n) + 4 * a.m * a.n
    nsets = max(1, int(a.ring_mb * 1e6 // bytes_alg))
    A = [si.device_normal_bits((a.m, a.k), si.F16 if a.dtype == "f16" else si.BF16) for _ in range(nsets)]
    B = [si.device_normal_bits((a.k, a.n), si.F16 if a.dtype == "f16" else si.BF16) for _ in range(nsets)]
    Cs = [torch.empty((a.m, a.n), dtype=torch.float32, device="cuda") for _ in range(nsets)]
    pa, pb, pc = [t.data_ptr() for t in A], [t.data_ptr() for t in B], [t.data_ptr() for t in Cs]
    s = torch.cuda.current_stream().cuda_stream
    if a.copy_mb > 0:
        n = int(a.copy_mb * 1e6) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print("copy of %d bytes done (reads %d B, writes %d B per copy kernel)" % (4 * n, 4 * n, 4 * n), flush=True)
    ft.ft_launch_timed(plan, pa, pb, pc, s, max(1, a.warmup))
    ms = ft.ft_launch_timed(plan, pa, pb, pc, s, a.iters)
    prog = [(ft.ft_ukset_get(uks, st.ukernel_id[i]), st.count_tau[i]) for i in range(st.n_ukernels)]
    desc = " + ".join("%dx(%dx%d w%dx%d gk%d s%d)" % (c, u.tm, u.tn, u.wm, u.wn, u.gk, u.stages) for u, c in prog)
    print("%dx%dx%d %s: %s, %d tiles x %d parts, class %d, lds %d: %.2f us, %.1f TFLOP/s, %.0f GB/s" % (
        a.m, a.n, a.k, a.dtype, desc, st.n_tiles, st.k_parts, st.kernel_class, st.lds_bytes, ms * 1e3,
        2.0 * a.m * a.n * a.k / ms / 1e9, bytes_alg / ms / 1e6), flush=True)


if __name__ == "__main__":
    main()
