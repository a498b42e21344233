"""Seeded synthetic inputs shared by the oracle-side and GPU-side callers.

Holds no arithmetic of the method: only random draws, rounding of the drawn fp32 values
to fp16 / bf16 bit patterns, and the shape lists of the five workload configurations.
The same uint16 bit patterns are handed to the CPU oracle and to the GPU library.
"""
import numpy as np

F16, BF16 = 0, 1
BASE_SEED = 240721418


def rng(config_index, extra=0):
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config_index + extra))


def to_bits(x32, dtype):
    """Round fp32 values to nearest-even fp16 / bf16 and return the uint16 bit patterns."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == F16:
        return x32.astype(np.float16).view(np.uint16)
    u = x32.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def normal_bits(g, shape, std, dtype):
    return to_bits(g.standard_normal(shape, dtype=np.float32) * np.float32(std), dtype)


def uniform_bits(g, shape, lo, hi, dtype):
    return to_bits(g.uniform(lo, hi, size=shape).astype(np.float32), dtype)


def device_normal_bits(shape, dtype, std=1.0):
    """N(0, std^2) values as fp16 / bf16 bit patterns in a torch int16 tensor on the GPU: operands of the
    timing harnesses, whose outputs nobody checks (drawn on the device, from torch's generator).  The
    values matter for timings: the power an MFMA draws, and with it the clock, depends on its data."""
    import torch
    x = torch.randn(shape, device="cuda", dtype=torch.float32).mul_(std)
    return x.to(torch.float16 if dtype == F16 else torch.bfloat16).view(torch.int16)


# ---- configuration 0: one odd-M Matmul ------------------------------------------------
def config0():
    g = rng(0)
    M, K, N = 77, 768, 768
    return dict(M=M, N=N, K=K, dtype=F16,
                A=uniform_bits(g, (M, K), -1.0, 1.0, F16),
                B=uniform_bits(g, (K, N), -1.0, 1.0, F16))


# ---- configuration 1: BERT-base-shaped dense sweep --------------------------------------
BERT_SEQ = (5, 17, 33, 64, 77, 100, 128)
BERT_BATCH = 16
BERT_LAYERS = ((768, 768), (768, 3072), (3072, 768))      # (K, N)


def config1_shapes():
    return [(BERT_BATCH * L, N, K) for L in BERT_SEQ for (K, N) in BERT_LAYERS]


def config1_problem(M, N, K, which=0):
    g = rng(1, extra=(M * 131 + N * 17 + K) % 997 + 7919 * which)
    return dict(M=M, N=N, K=K, dtype=F16,
                A=normal_bits(g, (M, K), 1.0, F16),
                B=normal_bits(g, (K, N), 0.02, F16))


# ---- configuration 2: attention batched Matmul with dynamic length ----------------------
ATT_BATCH = (1, 8, 32, 64)
ATT_HEADS = 12
ATT_DHEAD = 64


def config2_lengths():
    g = rng(2)
    return {B: [int(v) for v in g.integers(1, 513, size=32)] for B in ATT_BATCH}


def ragged_lengths(draw, n_seqs):
    """Lengths of the sequences of one ragged batch: drawn like the attention configuration's
    (uniform on 1..512), one independent length per sequence."""
    g = rng(2, extra=7000003 + draw)
    return [int(v) for v in g.integers(1, 513, size=n_seqs)]


def config2_problem(B, L, which):
    """which = 'qk': (B*12,L,64)x(B*12,64,L); 'pv': (B*12,L,L)x(B*12,L,64)."""
    g = rng(2, extra=B * 1009 + L + (0 if which == "qk" else 500000))
    nb = B * ATT_HEADS
    if which == "qk":
        M, K, N = L, ATT_DHEAD, L
    else:
        M, K, N = L, L, ATT_DHEAD
    return dict(batch=nb, M=M, N=N, K=K, dtype=F16,
                A=normal_bits(g, (nb, M, K), 1.0, F16),
                B=normal_bits(g, (nb, K, N), 1.0, F16))


# ---- configuration 3: LLM-style token-count GEMM ----------------------------------------
LLM_K = 4096
LLM_N = (4096, 11008)


def config3_token_counts():
    g = rng(3)
    u = g.random(64)
    return [int(min(8192, max(1, round(2.0 ** (13.0 * x))))) for x in u]


def config3_problem(M, N, rows_only=None):
    g = rng(3, extra=M * 3 + N)
    return dict(M=M, N=N, K=LLM_K, dtype=BF16,
                A=normal_bits(g, (M, LLM_K), 1.0, BF16),
                B=normal_bits(g, (LLM_K, N), 0.02, BF16))


# ---- configuration 4: dynamic-resolution Conv2d -----------------------------------------
CONV_RES = (28, 37, 56, 91, 112, 150, 224)
CONV_BATCH, CONV_CIN, CONV_COUT, CONV_R, CONV_S = 8, 64, 128, 3, 3


def config4_problem(res, batch=CONV_BATCH):
    g = rng(4, extra=res)
    return dict(n=batch, H=res, W=res, Cin=CONV_CIN, Cout=CONV_COUT, R=CONV_R, S=CONV_S,
                stride=1, pad=1, dtype=F16,
                X=normal_bits(g, (batch, res, res, CONV_CIN), 1.0, F16),
                Wt=normal_bits(g, (CONV_R, CONV_S, CONV_CIN, CONV_COUT), 1.0, F16))
