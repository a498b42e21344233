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


def run_epilogue(plan, A_bits, B_bits, n_out, bias=None, out16=None):
    """Launch through ft_launch_epilogue.  bias: fp32 numpy vector or None.  out16: None for an fp32
    C, else the 16-bit type (ft.FT_F16 / ft.FT_BF16) C is stored in; the result is decoded to fp64.
    C lies between two canary regions that must stay untouched."""
    A, B = dev_bits(A_bits), dev_bits(B_bits)
    bias_d = torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).cuda() if bias is not None else None
    if out16 is None:
        buf = alloc_out(n_out)
        cptr = buf.data_ptr() + 4 * GUARD
    else:
        buf = torch.full((n_out + 2 * GUARD,), 0x7e00 if out16 == ft.FT_F16 else 0x7fc0, dtype=torch.int16, device="cuda")
        buf[:GUARD] = 0x1234
        buf[-GUARD:] = 0x1234
        cptr = buf.data_ptr() + 2 * GUARD
    ft.ft_launch_epilogue(plan, A.data_ptr(), B.data_ptr(), cptr, bias_d.data_ptr() if bias_d is not None else 0, stream())
    torch.cuda.synchronize()
    if out16 is None:
        return out_view(buf, n_out)
    assert bool((buf[:GUARD] == 0x1234).all()) and bool((buf[-GUARD:] == 0x1234).all()), "write outside C"
    bits = buf[GUARD:GUARD + n_out].cpu().numpy().view(np.uint16)
    if out16 == ft.FT_F16:
        return bits.view(np.float16).astype(np.float64)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def check_epilogue(got, ref, refabs, bias, out16, what=""):
    """ref = exact sum + bias (fp64).  The kernel adds the bias in fp32 and, for a 16-bit C, rounds
    once to nearest: |d| <= 2e-3 * (sum |a||b| + |bias|) + half an output ulp of the reference
    (2^-11 relative for fp16, 2^-8 for bf16, plus the subnormal spacing)."""
    got = got.reshape(ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite (uncovered?) outputs"
    d = np.abs(got - ref)
    bound = REL_TOL * (refabs + (np.abs(bias) if bias is not None else 0.0)) + 1e-30
    if out16 is not None:
        rel, tiny = (2.0 ** -11, 2.0 ** -25) if out16 == ft.FT_F16 else (2.0 ** -8, 2.0 ** -134)
        bound = bound + rel * np.abs(ref) * (1 + 2 * REL_TOL) + tiny
    assert (d <= bound).all(), f"{what}: element bound violated, worst {np.max(d - bound)}"
    if out16 is not None:
        # against the oracle's own rounding: the same value or, where the fp32 sum fell on the other
        # side of a rounding boundary, its neighbour
        from oracle import epilogue as oe
        want = oe.round_to_16(ref, oe.F16 if out16 == ft.FT_F16 else oe.BF16)
        ulp = 2 * (rel * np.abs(ref) + tiny)
        assert (np.abs(got - want) <= ulp * (1 + 1e-9) + REL_TOL * refabs).all(), f"{what}: more than one output ulp from the rounded reference"
        assert (got == want).mean() > 0.9, f"{what}: only {(got == want).mean():.3f} of the outputs equal the rounded reference"


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
