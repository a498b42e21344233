"""ctypes front end of the plain-C contraction oracle (test infrastructure only).

Matmul (Sec. 4.1), BatchMatmul (Fig. 12 caption) and NHWC Conv2d with space axes
(n,k,p,q) / reduce axes (c,r,s) (Fig. 7 caption), all as fp64 sums of exact products
of fp16/bf16 inputs.  Arrays are numpy uint16 bit patterns in, float64 out.
"""
import ctypes
import numpy as np

from . import build as _build

F16, BF16 = 0, 1
_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        i64, p, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.oracle_decode.argtypes = [p, p, i64, ci]
        lib.oracle_decode.restype = None
        lib.oracle_matmul_rows.argtypes = [p, p, p, p, i64, i64, i64, p, i64, ci]
        lib.oracle_matmul_rows.restype = ci
        lib.oracle_bmm.argtypes = [p, p, p, p, i64, i64, i64, i64, ci]
        lib.oracle_bmm.restype = ci
        lib.oracle_conv2d_nhwc_pixels.argtypes = [p, p, p, p] + [i64] * 9 + [p, i64, ci]
        lib.oracle_conv2d_nhwc_pixels.restype = ci
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def _bits(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("oracle inputs are uint16 bit patterns")
    return a


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def num_threads():
    return int(_load().oracle_num_threads())


def decode(bits, dtype):
    bits = _bits(bits)
    out = np.empty(bits.shape, dtype=np.float64)
    _load().oracle_decode(_ptr(bits), _ptr(out), bits.size, dtype)
    return out


def matmul(A, B, dtype, rows=None, want_abs=False):
    """C[i,j] = sum_k A[i,k] B[k,j].  rows: optional int64 row indices (sampled check)."""
    A, B = _bits(A), _bits(B)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        nrows = rows.size
    else:
        nrows = M
    C = np.empty((nrows, N), dtype=np.float64)
    Cabs = np.empty((nrows, N), dtype=np.float64) if want_abs else None
    rc = _load().oracle_matmul_rows(_ptr(A), _ptr(B), _ptr(C), _ptr(Cabs), M, N, K,
                                    _ptr(rows), nrows, dtype)
    if rc:
        raise RuntimeError(f"oracle_matmul_rows rc={rc}")
    return (C, Cabs) if want_abs else C


def bmm(A, B, dtype, want_abs=False):
    """C[b,i,j] = sum_k A[b,i,k] B[b,k,j]."""
    A, B = _bits(A), _bits(B)
    nb, M, K = A.shape
    nb2, K2, N = B.shape
    assert nb == nb2 and K == K2
    C = np.empty((nb, M, N), dtype=np.float64)
    Cabs = np.empty((nb, M, N), dtype=np.float64) if want_abs else None
    rc = _load().oracle_bmm(_ptr(A), _ptr(B), _ptr(C), _ptr(Cabs), nb, M, N, K, dtype)
    if rc:
        raise RuntimeError(f"oracle_bmm rc={rc}")
    return (C, Cabs) if want_abs else C


def matmul_nk(A, Bt, dtype, rows=None, want_abs=False):
    """C[i,j] = sum_k A[i,k] Bt[j,k]: the Matmul of Sec. 4.1 with B handed over transposed ([N, K], k
    contiguous).  The same definition on the re-laid-out operand."""
    return matmul(A, np.ascontiguousarray(_bits(Bt).T), dtype, rows=rows, want_abs=want_abs)


def bmm_nk(A, Bt, dtype, want_abs=False):
    """C[b,i,j] = sum_k A[b,i,k] Bt[b,j,k] (BatchMatmul, Fig. 12 caption, B handed over as [b, N, K])."""
    return bmm(A, np.ascontiguousarray(np.swapaxes(_bits(Bt), 1, 2)), dtype, want_abs=want_abs)


def conv2d_nhwc(X, W, dtype, stride=1, pad=1, pixels=None, want_abs=False):
    """Y[n,p,q,k] = sum_{r,s,c} X[n,p*stride-pad+r,q*stride-pad+s,c] W[r,s,c,k], zero halo.

    pixels: optional flattened output-pixel indices ((n*P+p)*Q+q) for a sampled check;
    then the result has shape [len(pixels), Cout], else [N,P,Q,Cout].
    """
    X, W = _bits(X), _bits(W)
    n, H, Wd, Cin = X.shape
    R, S, Cin2, Cout = W.shape
    assert Cin == Cin2
    P = (H + 2 * pad - R) // stride + 1
    Q = (Wd + 2 * pad - S) // stride + 1
    if pixels is not None:
        pixels = np.ascontiguousarray(pixels, dtype=np.int64)
        npix = pixels.size
    else:
        npix = n * P * Q
    Y = np.empty((npix, Cout), dtype=np.float64)
    Yabs = np.empty((npix, Cout), dtype=np.float64) if want_abs else None
    rc = _load().oracle_conv2d_nhwc_pixels(_ptr(X), _ptr(W), _ptr(Y), _ptr(Yabs), n, H, Wd, Cin,
                                           Cout, R, S, stride, pad, _ptr(pixels), npix, dtype)
    if rc:
        raise RuntimeError(f"oracle_conv2d rc={rc}")
    if pixels is None:
        Y = Y.reshape(n, P, Q, Cout)
        if want_abs:
            Yabs = Yabs.reshape(n, P, Q, Cout)
    return (Y, Yabs) if want_abs else Y
