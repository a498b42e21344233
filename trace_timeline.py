#!/usr/bin/env python3
"""Where the time of one launch goes: per-workgroup timestamps from the development build of the
library (python -m paper_2407_21418_amd.build --trace -> libftuner_trace.so, kernels compiled with
-DFT_TRACE: every workgroup of the LDS-DMA bodies leaves the device-wide 100 MHz counter at kernel
entry, body start, first copies issued, first k-tile landed, middle of the loop, end of the loop,
after the exchange of a split, after its last store).

    python trace_timeline.py --m 2048 --n 768 --k 3072 [--force 128,64,64,32 [--teams 2] [--k-parts 2]]

The traced launch is the last of three back-to-back launches on operands that were rotated out of the
caches.  Prints, per mark, min / median / 90th percentile / max over the workgroups in microseconds
from the first workgroup's entry, and the medians of the three phases of a workgroup.
"""
import argparse
import ctypes as C
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
os.environ.setdefault("FTUNER_LIB", os.path.join(ROOT, "paper_2407_21418_amd", "libftuner_trace.so"))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--m", type=int, required=True)
    ap.add_argument("--n", type=int, required=True)
    ap.add_argument("--k", type=int, required=True)
    ap.add_argument("--dtype", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--force", default="")
    ap.add_argument("--waves", type=int, default=4, choices=[4, 8], help="with --force: 8 picks the eight-wave grid of that tile")
    ap.add_argument("--teams", type=int, default=1, choices=[1, 2])
    ap.add_argument("--k-parts", type=int, default=0)
    ap.add_argument("--ring-mb", type=float, default=700.0)
    a = ap.parse_args()

    import numpy as np
    import torch
    import paper_2407_21418_amd as ft
    import synth_inputs as si

    lib = ft.lib()
    if not hasattr(lib, "ft_debug_set_trace"):
        raise SystemExit("needs the development build: python -m paper_2407_21418_amd.build --trace")
    lib.ft_debug_set_trace.restype, lib.ft_debug_set_trace.argtypes = None, [C.c_void_p]
    s = torch.cuda.current_stream().cuda_stream
    dt = ft.FT_F16 if a.dtype == "f16" else ft.FT_BF16
    op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dt, n=a.n, k=a.k, m_lo=1, m_hi=max(8192, a.m)))
    uks = ft.ft_ukernels_derive(op, ft.ft_hw_query(0), None)
    mode, forced = ft.FT_PLAN_PATCHWORK, None
    if a.force:
        want = tuple(int(x) for x in a.force.split(","))
        ids = [i for i in range(ft.ft_ukset_size(uks))
               if (lambda u: (u.tm, u.tn, u.wm, u.wn) == want and (u.gk == 2) == (a.teams == 2) and u.gm * u.gn == (8 if a.waves == 8 else 4))(ft.ft_ukset_get(uks, i))]
        if not ids:
            raise SystemExit("uKernel %s is not in the derived set" % (want,))
        mode = ft.FT_PLAN_FORCED
        forced = ft.ft_forced_program(k1=ids[0], count1=((a.m + 15) // 16 * 16) // want[0], k_parts=a.k_parts)
    plan = ft.ft_plan_create(op, uks, ft.ft_shape(m=a.m), mode, forced)
    st = ft.ft_plan_stats_get(plan)
    bytes_alg = 2 * (a.m * a.k + a.k * a.n) + 4 * a.m * a.n
    nsets = max(3, int(a.ring_mb * 1e6 // bytes_alg))
    A = [si.device_normal_bits((a.m, a.k), si.F16 if a.dtype == "f16" else si.BF16) for _ in range(nsets)]
    B = [si.device_normal_bits((a.k, a.n), si.F16 if a.dtype == "f16" else si.BF16) for _ in range(nsets)]
    Cs = [torch.empty((a.m, a.n), dtype=torch.float32, device="cuda") for _ in range(nsets)]
    tr = torch.zeros((int(st.n_tiles) * max(1, st.k_parts) + 64) * 16, dtype=torch.int64, device="cuda")
    lib.ft_debug_set_trace(None)
    for i in range(nsets):
        ft.ft_launch(plan, A[i].data_ptr(), B[i].data_ptr(), Cs[i].data_ptr(), s)
    torch.cuda.synchronize()
    lib.ft_debug_set_trace(tr.data_ptr())
    for i in range(3):
        ft.ft_launch(plan, A[i].data_ptr(), B[i].data_ptr(), Cs[i].data_ptr(), s)
    torch.cuda.synchronize()
    lib.ft_debug_set_trace(None)
    t = tr.cpu().numpy().reshape(-1, 16).astype(np.float64)
    t = t[t[:, 0] > 0]
    us = (t - t[:, 0].min()) / 100.0
    prog = [(ft.ft_ukset_get(uks, st.ukernel_id[i]), st.count_tau[i]) for i in range(st.n_ukernels)]
    print("%dx%dx%d: %s, %d parts, %d workgroups traced" % (a.m, a.n, a.k, " + ".join(
        "%dx(%dx%d w%dx%d gk%d s%d)" % (c, u.tm, u.tn, u.wm, u.wn, u.gk, u.stages) for u, c in prog), st.k_parts, len(us)))
    for i, nm in enumerate(["entry", "body", "issued", "tile 0", "half", "loop end", "exchange", "stored"]):
        col = us[:, i][t[:, i] > 0]
        if len(col):
            print("   %-9s min %6.2f  median %6.2f  p90 %6.2f  max %6.2f" % (nm, col.min(), np.median(col), np.percentile(col, 90), col.max()))
    ok = (t[:, 7] > 0) & (t[:, 3] > 0)
    if ok.any():
        d = us[ok]
        print("   medians per workgroup: entry -> tile 0 %.2f us | tile 0 -> loop end %.2f us | loop end -> stored %.2f us" % (
            np.median(d[:, 3] - d[:, 0]), np.median(d[:, 5] - d[:, 3]), np.median(d[:, 7] - d[:, 5])))


if __name__ == "__main__":
    main()
