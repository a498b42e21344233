"""Pins of the contraction oracle against things other than itself: exact rational brute
force, textbook special cases (identity, permutation, power-of-two scaling), numpy's fp64
matmul, and explicit im2col for the convolution.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import synth_inputs as si
from oracle import contraction as oc

F16, BF16 = 0, 1


def as_f64(bits, dtype):
    """Independent decode through numpy (not through the oracle's own decoder)."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def frac(x):
    return Fraction(float(x))


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_decoder_all_bit_patterns(dtype):
    bits = np.arange(65536, dtype=np.uint16)
    got = oc.decode(bits, dtype)
    ref = as_f64(bits, dtype)
    fin = np.isfinite(ref)
    assert np.array_equal(got[fin], ref[fin])
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref))
    assert np.array_equal(np.signbit(got[fin]), np.signbit(ref[fin]))


def test_rounding_of_generators():
    # bf16 round-to-nearest-even of the shared generator, against a slow scalar definition
    g = np.random.default_rng(1)
    x = g.standard_normal(2000).astype(np.float32)
    bits = si.to_bits(x, BF16)
    for xi, bi in zip(x[:300], bits[:300]):
        lo = np.uint32(np.float32(xi).view(np.uint32)) & np.uint32(0xFFFF0000)
        c0 = np.array([lo], dtype=np.uint32).view(np.float32)[0]
        c1 = np.array([lo + 0x10000], dtype=np.uint32).view(np.float32)[0]
        d0, d1 = abs(float(xi) - float(c0)), abs(float(c1) - float(xi))
        want = lo >> 16 if d0 < d1 or (d0 == d1 and ((lo >> 16) & 1) == 0) else (lo >> 16) + 1
        assert int(bi) == int(want)


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (8, 2, 4), (5, 8, 8), (2, 7, 1)])
def test_matmul_brute_force_exact(dtype, M, N, K):
    g = np.random.default_rng(M * 100 + N * 10 + K + dtype)
    A = si.to_bits(g.uniform(-2, 2, (M, K)).astype(np.float32), dtype)
    B = si.to_bits(g.uniform(-2, 2, (K, N)).astype(np.float32), dtype)
    C, Cabs = oc.matmul(A, B, dtype, want_abs=True)
    Ad, Bd = as_f64(A, dtype), as_f64(B, dtype)
    for i in range(M):
        for j in range(N):
            exact = sum(frac(Ad[i, k]) * frac(Bd[k, j]) for k in range(K))
            exabs = sum(abs(frac(Ad[i, k]) * frac(Bd[k, j])) for k in range(K))
            # fp64 accumulation of exact products: error <= K * 2^-53 * sum|a||b|
            assert abs(Fraction(C[i, j]) - exact) <= K * Fraction(1, 2 ** 53) * exabs
            assert abs(Fraction(Cabs[i, j]) - exabs) <= K * Fraction(1, 2 ** 53) * exabs


def test_matmul_small_integers_bit_exact():
    # small integers: every partial sum is exactly representable, so the result is exact
    g = np.random.default_rng(5)
    A32 = g.integers(-8, 9, (6, 9)).astype(np.float32)
    B32 = g.integers(-8, 9, (9, 4)).astype(np.float32)
    for dtype in (F16, BF16):
        C = oc.matmul(si.to_bits(A32, dtype), si.to_bits(B32, dtype), dtype)
        want = [[sum(int(A32[i, k]) * int(B32[k, j]) for k in range(9)) for j in range(4)]
                for i in range(6)]
        assert np.array_equal(C, np.array(want, dtype=np.float64))


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_identity_and_permutation(dtype):
    g = np.random.default_rng(11)
    n, N = 37, 29
    B = si.normal_bits(g, (n, N), 1.0, dtype)
    I = si.to_bits(np.eye(n, dtype=np.float32), dtype)
    assert np.array_equal(oc.matmul(I, B, dtype), as_f64(B, dtype))          # I*B = B
    A = si.normal_bits(g, (N, n), 1.0, dtype)
    assert np.array_equal(oc.matmul(A, I, dtype), as_f64(A, dtype))          # A*I = A
    perm = g.permutation(n)
    Pm = np.zeros((n, n), dtype=np.float32)
    Pm[np.arange(n), perm] = 1.0
    assert np.array_equal(oc.matmul(si.to_bits(Pm, dtype), B, dtype), as_f64(B, dtype)[perm])
    # permutation on the right permutes columns: (A*P)[i,j] = A[i, inv(j)] with P[k,j]=1 iff k=perm^-1..
    Pc = np.zeros((n, n), dtype=np.float32)
    Pc[perm, np.arange(n)] = 1.0
    assert np.array_equal(oc.matmul(A, si.to_bits(Pc, dtype), dtype), as_f64(A, dtype)[:, perm])


def test_power_of_two_scaling_exact():
    g = np.random.default_rng(3)
    A = g.standard_normal((9, 33)).astype(np.float32)
    B = g.standard_normal((33, 12)).astype(np.float32)
    Ab, Bb = si.to_bits(A, F16), si.to_bits(B, F16)
    A4 = (Ab.view(np.float16) * np.float16(4)).view(np.uint16)
    C, C4 = oc.matmul(Ab, Bb, F16), oc.matmul(A4, Bb, F16)
    assert np.array_equal(C4, 4.0 * C)


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("M,N,K", [(77, 768, 768), (130, 65, 257), (1, 300, 17)])
def test_matmul_vs_numpy_fp64(dtype, M, N, K):
    g = np.random.default_rng(M + N + K)
    A = si.normal_bits(g, (M, K), 1.0, dtype)
    B = si.normal_bits(g, (K, N), 0.5, dtype)
    C, Cabs = oc.matmul(A, B, dtype, want_abs=True)
    Ad, Bd = as_f64(A, dtype), as_f64(B, dtype)
    ref = Ad @ Bd
    refabs = np.abs(Ad) @ np.abs(Bd)
    assert np.all(np.abs(C - ref) <= 1e-12 * refabs)
    assert np.all(np.abs(Cabs - refabs) <= 1e-12 * refabs)


def test_sampled_rows_match_full():
    g = np.random.default_rng(8)
    A = si.normal_bits(g, (50, 40), 1.0, F16)
    B = si.normal_bits(g, (40, 30), 1.0, F16)
    full = oc.matmul(A, B, F16)
    rows = np.array([49, 0, 7, 7, 23], dtype=np.int64)
    assert np.array_equal(oc.matmul(A, B, F16, rows=rows), full[rows])


def test_bmm_is_per_batch_matmul():
    g = np.random.default_rng(9)
    A = si.normal_bits(g, (5, 13, 21), 1.0, F16)
    B = si.normal_bits(g, (5, 21, 8), 1.0, F16)
    C = oc.bmm(A, B, F16)
    ref = np.einsum("bik,bkj->bij", as_f64(A, F16), as_f64(B, F16))
    assert np.allclose(C, ref, rtol=0, atol=1e-12 * np.abs(ref).max())
    for b in range(5):
        assert np.array_equal(C[b], oc.matmul(A[b], B[b], F16))


def test_b_handed_over_as_nk():
    """B stored [N, K]: C[i,j] = sum_k A[i,k] Bt[j,k] against numpy's einsum on the decoded values and
    against a direct loop on a tiny case; a transposed operand with distinct rows and columns, so a
    missing (or doubled) transposition cannot pass."""
    g = np.random.default_rng(12)
    A = si.normal_bits(g, (9, 14), 1.0, BF16)
    Bt = si.normal_bits(g, (5, 14), 1.0, BF16)
    C = oc.matmul_nk(A, Bt, BF16)
    Ad, Bd = as_f64(A, BF16), as_f64(Bt, BF16)
    assert C.shape == (9, 5)
    assert np.allclose(C, np.einsum("ik,jk->ij", Ad, Bd), rtol=0, atol=1e-12 * np.abs(Ad).max() * np.abs(Bd).max() * 14)
    for i in (0, 8):
        for j in (0, 4):
            assert abs(C[i, j] - sum(Ad[i, k] * Bd[j, k] for k in range(14))) <= 1e-12
    Ab = si.normal_bits(g, (3, 7, 16), 1.0, F16)
    Bb = si.normal_bits(g, (3, 11, 16), 1.0, F16)
    Cb = oc.bmm_nk(Ab, Bb, F16)
    ref = np.einsum("bik,bjk->bij", as_f64(Ab, F16), as_f64(Bb, F16))
    assert Cb.shape == (3, 7, 11) and np.allclose(Cb, ref, rtol=0, atol=1e-12 * np.abs(ref).max())
    rows = np.array([6, 0], dtype=np.int64)
    assert np.array_equal(oc.matmul_nk(Ab[1], Bb[1], F16, rows=rows), Cb[1][rows])


def _im2col(Xd, R, S, stride, pad):
    n, H, W, Cin = Xd.shape
    P = (H + 2 * pad - R) // stride + 1
    Qo = (W + 2 * pad - S) // stride + 1
    Xp = np.zeros((n, H + 2 * pad, W + 2 * pad, Cin))
    Xp[:, pad:pad + H, pad:pad + W] = Xd
    cols = np.zeros((n, P, Qo, R, S, Cin))
    for r in range(R):
        for s in range(S):
            cols[:, :, :, r, s, :] = Xp[:, r:r + stride * P:stride, s:s + stride * Qo:stride, :]
    return cols.reshape(n * P * Qo, R * S * Cin), P, Qo


def test_conv_brute_force_tiny():
    g = np.random.default_rng(21)
    n, H, W, Cin, Cout, R, S = 1, 4, 4, 2, 3, 3, 3
    X = si.to_bits(g.integers(-4, 5, (n, H, W, Cin)).astype(np.float32), F16)
    Wt = si.to_bits(g.integers(-4, 5, (R, S, Cin, Cout)).astype(np.float32), F16)
    Y = oc.conv2d_nhwc(X, Wt, F16, stride=1, pad=1)
    Xd, Wd = as_f64(X, F16), as_f64(Wt, F16)
    for p in range(H):
        for q in range(W):
            for k in range(Cout):
                acc = 0
                for r in range(R):
                    for s in range(S):
                        h, w = p - 1 + r, q - 1 + s
                        if 0 <= h < H and 0 <= w < W:
                            for c in range(Cin):
                                acc += int(Xd[0, h, w, c]) * int(Wd[r, s, c, k])
                assert Y[0, p, q, k] == acc


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0)])
def test_conv_vs_im2col_matmul(stride, pad):
    g = np.random.default_rng(22)
    X = si.normal_bits(g, (2, 9, 7, 8), 1.0, F16)
    Wt = si.normal_bits(g, (3, 3, 8, 5), 1.0, F16)
    Y = oc.conv2d_nhwc(X, Wt, F16, stride=stride, pad=pad)
    cols, P, Qo = _im2col(as_f64(X, F16), 3, 3, stride, pad)
    ref = (cols @ as_f64(Wt, F16).reshape(72, 5)).reshape(2, P, Qo, 5)
    assert Y.shape == ref.shape
    assert np.allclose(Y, ref, rtol=0, atol=1e-12 * np.abs(ref).max())


def test_conv_single_tap_is_shift_and_centre_tap_is_matmul():
    g = np.random.default_rng(23)
    n, H, W, C = 2, 6, 5, 4
    X = si.normal_bits(g, (n, H, W, C), 1.0, F16)
    Xd = as_f64(X, F16)
    eye = np.eye(C, dtype=np.float32)
    for (r, s) in [(0, 0), (0, 2), (2, 1), (1, 1)]:
        Wt = np.zeros((3, 3, C, C), dtype=np.float32)
        Wt[r, s] = eye
        Y = oc.conv2d_nhwc(X, si.to_bits(Wt, F16), F16)
        want = np.zeros_like(Xd)
        for p in range(H):
            for q in range(W):
                h, w = p - 1 + r, q - 1 + s
                if 0 <= h < H and 0 <= w < W:
                    want[:, p, q] = Xd[:, h, w]
        assert np.array_equal(Y, want)
    # only the centre tap non-zero: a plain Matmul over pixels
    Wc = si.normal_bits(g, (C, 7), 1.0, F16)
    Wt = np.zeros((3, 3, C, 7), dtype=np.uint16)
    Wt[1, 1] = Wc
    Y = oc.conv2d_nhwc(X, Wt, F16)
    assert np.array_equal(Y.reshape(-1, 7), oc.matmul(X.reshape(-1, C), Wc, F16))


def test_conv_sampled_pixels_match_full():
    g = np.random.default_rng(24)
    X = si.normal_bits(g, (2, 5, 6, 8), 1.0, F16)
    Wt = si.normal_bits(g, (3, 3, 8, 4), 1.0, F16)
    full = oc.conv2d_nhwc(X, Wt, F16).reshape(-1, 4)
    pix = np.array([0, 59, 17, 30], dtype=np.int64)
    assert np.array_equal(oc.conv2d_nhwc(X, Wt, F16, pixels=pix), full[pix])


def test_fp32_accumulation_bound_is_far_inside_tolerance():
    # a-priori bound for any fp32 accumulation order of exact products:
    # |err| <= K * 2^-24 * sum|a||b| (first order); 2e-3 is looser even at K = 4096
    assert 4096 * 2.0 ** -24 < 2e-3
