"""Epilogue oracle (test infrastructure only): bias add and rounding of the output to a 16-bit
floating-point type, written out from the definitions in fp64.

The fused Dense + bias-add operator is the one the paper's BERT evaluation runs (Sec. 6.2,
end-to-end models); a 16-bit output is the same contraction with the result rounded once, to
nearest, ties to even.  Nothing here is shared with the GPU library.
"""
import numpy as np

F16, BF16 = 0, 1
# (fraction bits, minimum normal exponent, largest finite value)
_FORMAT = {F16: (10, -14, 65504.0), BF16: (7, -126, float(np.float32(3.3895313892515355e38)))}


def add_bias(C, bias):
    """C[..., j] + bias[j] in fp64 (bias: fp32 or fp64 values, one per output column)."""
    C = np.asarray(C, dtype=np.float64)
    bias = np.asarray(bias, dtype=np.float64)
    assert bias.shape == (C.shape[-1],)
    return C + bias


def round_to_16(x, dtype):
    """Round fp64 values to the nearest fp16 / bf16 value, ties to even; returns those values as
    fp64.  |x| = m * 2^e (0.5 <= m < 1): the spacing of representable numbers around x is
    2^(e - 1 - fraction_bits) for normal numbers and 2^(emin - fraction_bits) below the smallest
    normal; x is rounded to an integer multiple of that spacing (numpy.rint rounds half to even,
    and the division by a power of two is exact).  Values that round past the largest finite
    number become infinite."""
    frac, emin, fmax = _FORMAT[dtype]
    x = np.asarray(x, dtype=np.float64)
    out = np.array(x, dtype=np.float64, copy=True)
    fin = np.isfinite(x) & (x != 0)
    ax = np.abs(x[fin])
    _, e = np.frexp(ax)
    spacing_exp = np.maximum(e - 1, emin) - frac
    q = np.ldexp(1.0, spacing_exp)
    r = np.rint(ax / q) * q
    r = np.where(r > fmax, np.inf, r)
    out[fin] = np.copysign(r, x[fin])
    return out
