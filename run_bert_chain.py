"""A second workload through the C ABI: the dense layers of a BERT-base encoder, chained on one stream.

    python run_bert_chain.py [--layers 12] [--iters 20] [--dtype f16|bf16]

The paper's end-to-end BERT run is made of Dense + bias-add operators whose token count changes from
request to request (Sec. 6.2; Table 6 lists the (T, 2304, 768) projection).  For every token count
M = 16 T, T in Table 6's lengths, each encoder layer launches four GEMMs with the bias fused and C
stored in the inputs' 16-bit type:

    qkv = x   Wqkv + b     [M, 768] x [768, 2304]
    o   = ctx Wo   + b     [M, 768] x [768, 768]      ctx: a resident buffer standing for the attention
                                                      block's output (not part of this path)
    h   = o   W1   + b     [M, 768] x [768, 3072]     reads the C of the launch before it
    x'  = h   W2   + b     [M, 3072] x [3072, 768]    reads h; x' is the next layer's x

Every layer has its own weights (170 MB for 12 layers: they stream from memory, as in serving).  A
pass is layers x 4 launches issued back to back with no host synchronisation; each launch looks its
plan up with ft_plan_cached, as a serving loop would.  Timed with events over --iters passes after
two warm-up passes.  The same passes run with the pad-to-library plan and with M padded to the next
power of two (the bucketing of serving stacks; useful flops of the true M).  Operand values are
random bit patterns made on the device (timing only; tests/ checks a chained layer against the oracle).
Prints one line per token count and a JSON summary line.
"""
import argparse
import json
import math
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

TABLE6_T = (5, 24, 43, 62, 81, 100, 119, 128)
HIDDEN, FFN = 768, 3072
# (name, N, K) of the four GEMMs of a layer, in launch order
LAYER_GEMMS = (("qkv", 3 * HIDDEN, HIDDEN), ("o", HIDDEN, HIDDEN), ("ffn1", FFN, HIDDEN), ("ffn2", HIDDEN, FFN))


def layer_flops(M, only=None):
    return sum(2.0 * M * n * k for name, n, k in LAYER_GEMMS if only is None or name in only)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=12)
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--dtype", choices=["f16", "bf16"], default="f16")
    ap.add_argument("--batch", type=int, default=16)
    ap.add_argument("--lengths", default=",".join(str(t) for t in TABLE6_T), help="comma list of T (default: Table 6's)")
    ap.add_argument("--variants", default="patch,base,bucket",
                    help="comma list: patch (the planner's plan, always run), base (pad-to-library plan), "
                         "bucket (M padded to the next power of two); 'patch' alone is what the committed profile runs")
    ap.add_argument("--only", default="", help="comma list of qkv,o,ffn1,ffn2: launch only these GEMMs of each layer")
    ap.add_argument("--four-wave", action="store_true", help="uKernel sets without the eight-wave uKernels")
    a = ap.parse_args()
    variants = set(a.variants.split(","))
    only = set(a.only.split(",")) if a.only else {name for name, _, _ in LAYER_GEMMS}
    assert only <= {name for name, _, _ in LAYER_GEMMS}, "--only: qkv,o,ffn1,ffn2"
    assert variants <= {"patch", "base", "bucket"}, "--variants: patch[,base][,bucket]"

    import torch
    import paper_2407_21418_amd as ft
    import synth_inputs as si

    assert torch.cuda.is_available(), "run_bert_chain needs a GPU"
    dt = ft.FT_F16 if a.dtype == "f16" else ft.FT_BF16
    stream_t = torch.cuda.Stream()
    stream = stream_t.cuda_stream
    hw = ft.ft_hw_query(0)
    tuning = ft.ft_tuning_default()
    if a.four_wave:
        tuning.two_team_bodies = 0

    def rand16(shape, std=1.0):
        return si.device_normal_bits(shape, si.F16 if a.dtype == "f16" else si.BF16, std)

    ops = {}
    for name, n, k in LAYER_GEMMS:
        op = ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dt, n=n, k=k, m_lo=1, m_hi=8192,
                                             out_dtype=ft.FT_OUT_SAME, epilogue=ft.FT_EPI_BIAS))
        ops[name] = (op, ft.ft_ukernels_derive(op, hw, tuning))
    W = [{name: rand16((k, n), k ** -0.5) for name, n, k in LAYER_GEMMS} for _ in range(a.layers)]
    bias = [{name: torch.zeros(n, dtype=torch.float32, device="cuda") for name, n, k in LAYER_GEMMS} for _ in range(a.layers)]
    lengths = [int(t) for t in a.lengths.split(",")]
    m_max = a.batch * max(lengths)
    m_cap = 1 << (m_max - 1).bit_length()
    x = rand16((m_cap, HIDDEN))
    ctx = rand16((m_cap, HIDDEN))
    qkv = torch.empty((m_cap, 3 * HIDDEN), dtype=torch.int16, device="cuda")
    o = torch.empty((m_cap, HIDDEN), dtype=torch.int16, device="cuda")
    h = torch.empty((m_cap, FFN), dtype=torch.int16, device="cuda")
    x2 = torch.empty((m_cap, HIDDEN), dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()

    def one_pass(M, flags):
        """layers x 4 launches; returns the host time spent in plan look-ups."""
        t_lookup = 0.0
        src, dst = x, x2
        for l in range(a.layers):
            for name, A, Cbuf in (("qkv", src, qkv), ("o", ctx, o), ("ffn1", o, h), ("ffn2", h, dst)):
                if name not in only:
                    continue
                op, uks = ops[name]
                t0 = time.perf_counter()
                plan = ft.ft_plan_cached(op, uks, ft.ft_shape(m=M), flags)
                t_lookup += time.perf_counter() - t0
                ft.ft_launch_epilogue(plan, A.data_ptr(), W[l][name].data_ptr(), Cbuf.data_ptr(),
                                      bias[l][name].data_ptr(), stream)
            src, dst = dst, src
        return t_lookup

    def timed(M, flags):
        for _ in range(2):
            one_pass(M, flags)
        stream_t.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t_lookup = 0.0
        t0 = time.perf_counter()
        with torch.cuda.stream(stream_t):
            e0.record()
            for _ in range(a.iters):
                t_lookup += one_pass(M, flags)
            e1.record()
        t_issue = time.perf_counter() - t0
        e1.synchronize()
        n_launch = a.iters * a.layers * len(only)
        return e0.elapsed_time(e1) * 1e3 / (a.iters * a.layers), t_lookup * 1e6 / n_launch, t_issue * 1e6 / n_launch

    rows = []
    for T in lengths:
        M = a.batch * T
        Mb = max(16, 1 << (M - 1).bit_length())
        us_patch, us_lookup, us_issue = timed(M, ft.FT_PLAN_PATCHWORK)
        us_base = timed(M, ft.FT_PLAN_PAD_BASELINE)[0] if "base" in variants else float("nan")
        us_bucket = timed(Mb, ft.FT_PLAN_PATCHWORK)[0] if "bucket" in variants else float("nan")
        fl = layer_flops(M, only)
        rows.append(dict(T=T, M=M, us_per_layer=round(us_patch, 2), tflops=round(fl / us_patch / 1e6, 1),
                         us_per_layer_pad_baseline=round(us_base, 2), us_per_layer_bucketed=round(us_bucket, 2),
                         bucket_M=Mb, host_us_per_launch=round(us_issue, 2), lookup_us_per_launch=round(us_lookup, 2)))
        print("T=%3d M=%4d  %7.1f us/layer %6.1f TFLOP/s | pad baseline %7.1f us (x%.2f) | bucketed to M=%4d %7.1f us (x%.2f) | host %.1f us/launch (lookup %.1f)"
              % (T, M, us_patch, fl / us_patch / 1e6, us_base, us_base / us_patch, Mb, us_bucket, us_bucket / us_patch,
                 us_issue, us_lookup), flush=True)
    def gm(xs):
        xs = [v for v in xs if v == v]
        return math.exp(sum(math.log(v) for v in xs) / len(xs)) if xs else float("nan")

    print(json.dumps({"workload": "BERT-base dense layers chained, %d layers, batch %d, T in Table 6's lengths, %s in/out, bias fused"
                                  % (a.layers, a.batch, a.dtype),
                      "geomean_tflops": round(gm([r["tflops"] for r in rows]), 1),
                      "speedup_vs_pad_baseline_geomean": round(gm([r["us_per_layer_pad_baseline"] / r["us_per_layer"] for r in rows]), 3),
                      "speedup_vs_bucketed_geomean": round(gm([r["us_per_layer_bucketed"] / r["us_per_layer"] for r in rows]), 3),
                      "rows": rows}))


if __name__ == "__main__":
    main()
