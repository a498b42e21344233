"""Context measurement, not part of the library or of bench.py: torch.matmul (the vendor GEMM
library behind PyTorch-ROCm) on the bench sweep or on a list of LLM-sized shapes, with the same
cold operand ring, 16-bit inputs and a 16-bit output (torch offers no fp32 output for 16-bit
inputs).  Prints per shape the eager and the graph-replayed time per call and the geomean of the
better of the two.

    python -m paper_2407_21418_amd.run_vendor_context            # 21 GEMMs of the bench sweep, fp16
    python -m paper_2407_21418_amd.run_vendor_context --llm      # ten bf16 shapes with K = 4096
"""
import argparse
import math
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import synth_inputs as si  # noqa: E402

LLM_SHAPES = [(16, 4096, 4096), (128, 4096, 4096), (512, 4096, 4096), (1024, 4096, 4096), (2048, 4096, 4096),
              (8192, 4096, 4096), (16, 11008, 4096), (128, 11008, 4096), (1024, 11008, 4096), (8192, 11008, 4096)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--llm", action="store_true")
    args = ap.parse_args()
    shapes = LLM_SHAPES if args.llm else si.config1_shapes()
    dt = torch.bfloat16 if args.llm else torch.float16
    rates = []
    for (M, N, K) in shapes:
        ring = max(2, int(math.ceil(600e6 / (2 * (M * K + K * N) + 2 * M * N))))
        A = [torch.randn(M, K, device="cuda", dtype=dt) for _ in range(ring)]
        B = [torch.randn(K, N, device="cuda", dtype=dt) * 0.02 for _ in range(ring)]
        C = [torch.empty(M, N, device="cuda", dtype=dt) for _ in range(ring)]
        iters = 200 if M * N * K < 2e10 else 30
        for i in range(10):
            torch.matmul(A[i % ring], B[i % ring], out=C[i % ring])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            torch.matmul(A[i % ring], B[i % ring], out=C[i % ring])
        e1.record()
        torch.cuda.synchronize()
        eager_us = e0.elapsed_time(e1) * 1e3 / iters
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(iters):
                    torch.matmul(A[i % ring], B[i % ring], out=C[i % ring])
        graph.replay()
        torch.cuda.synchronize()
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        graph_us = e0.elapsed_time(e1) * 1e3 / iters
        rates.append(2.0 * M * N * K / min(eager_us, graph_us) / 1e6)
        print(f"{M:5d} {N:5d} {K:5d}  eager {eager_us:8.2f} us  graph {graph_us:8.2f} us  {rates[-1]:7.1f} TFLOP/s", flush=True)
        del A, B, C, graph
        torch.cuda.empty_cache()
    print("geomean TFLOP/s (better of eager / graph replay): %.1f" % math.exp(sum(map(math.log, rates)) / len(rates)))


if __name__ == "__main__":
    main()
