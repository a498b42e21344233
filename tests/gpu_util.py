"""Helpers of the GPU parity tests: run an operator through the C ABI on torch-owned device
memory and compare with the CPU oracle to the stated tolerance."""
import numpy as np
import torch

import paper_2407_21418_amd as ft

REL_TOL = 2e-3          # max relative error for fp32-accumulated fp16/bf16 (the benchmark spec)
GUARD = 256             # canary floats on each side of C


def stream():
    return torch.cuda.current_stream().cuda_stream


def dev_bits(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def alloc_out(n_elems):
    buf = torch.full((n_elems + 2 * GUARD,), float("nan"), dtype=torch.float32, device="cuda")
    buf[:GUARD] = 12345.0
    buf[-GUARD:] = 12345.0
    return buf


def out_view(buf, n_elems):
    assert bool((buf[:GUARD] == 12345.0).all()) and bool((buf[-GUARD:] == 12345.0).all()), "write outside C"
    return buf[GUARD:GUARD + n_elems].cpu().numpy().astype(np.float64)


def run(plan, A_bits, B_bits, n_out):
    A, B = dev_bits(A_bits), dev_bits(B_bits)
    buf = alloc_out(n_out)
    ft.ft_launch(plan, A.data_ptr(), B.data_ptr(), buf.data_ptr() + 4 * GUARD, stream())
    torch.cuda.synchronize()
    return out_view(buf, n_out)


def check(got, ref, refabs, what=""):
    """(i) max|d| / max|ref| <= 2e-3; (ii) |d_ij| <= 2e-3 * sum_k |a_ik||b_kj| for every element."""
    got = got.reshape(ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite (uncovered?) outputs"
    d = np.abs(got - ref)
    scale = np.abs(ref).max()
    assert d.max() <= REL_TOL * max(scale, 1e-30), f"{what}: max err {d.max()} vs scale {scale}"
    assert (d <= REL_TOL * refabs + 1e-30).all(), f"{what}: element bound violated, worst {np.max(d - REL_TOL * refabs)}"


def matmul_op(N, K, dtype, m_hi=8192):
    return ft.ft_op_register(ft.ft_op_desc(kind=ft.FT_OP_MATMUL, dtype=dtype, n=N, k=K, m_lo=0, m_hi=m_hi))
