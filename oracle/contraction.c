/*
 * CPU oracle for the contraction values (TEST INFRASTRUCTURE ONLY).
 *
 * Plain, slow, obviously-correct definitions of the three operators the
 * uKernel patchwork computes.  Tiling and padding never change the
 * mathematics, so the oracle is the definition written out:
 *
 *   Matmul       C[i,j]   = sum_k A[i,k]   * B[k,j]      (Sec. 4.1; Fig. 9 caption)
 *   BatchMatmul  C[b,i,j] = sum_k A[b,i,k] * B[b,k,j]    (Fig. 12 caption)
 *   Conv2d       space axes (n,k,p,q), reduce axes (c,r,s) (Fig. 7 caption):
 *                Y[n,p,q,k] = sum_{r,s,c} X[n, p*stride-pad+r, q*stride-pad+s, c] * W[r,s,c,k]
 *                with out-of-range X taken as zero (NHWC input, RSCK weights).
 *
 * Inputs are fp16 or bf16 bit patterns, decoded exactly to fp64 here (own
 * decoder, no library); every product of two such values is exact in fp64
 * (11x11 or 8x8 bit significands); sums are accumulated in fp64 in plain
 * ascending reduce-axis order.  A second output holds sum |a|*|b| per element
 * so that a test can apply an a-priori rounding bound.
 *
 * Nothing here is shared with the GPU library: no headers, no tables, no helpers.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

/* IEEE binary16 -> double, by the format's definition. */
static double dec_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int exp = (h >> 10) & 0x1f;
    int man = h & 0x3ff;
    double v;
    if (exp == 0)
        v = ldexp((double)man, -24);                 /* subnormal: man * 2^-10 * 2^-14 */
    else if (exp == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)man / 1024.0, exp - 15);
    return sign ? -v : v;
}

/* bfloat16 = upper half of an IEEE binary32. */
static double dec_bf16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int exp = (h >> 7) & 0xff;
    int man = h & 0x7f;
    double v;
    if (exp == 0)
        v = ldexp((double)man, -133);                /* man * 2^-7 * 2^-126 */
    else if (exp == 255)
        v = man ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)man / 128.0, exp - 127);
    return sign ? -v : v;
}

static double dec(uint16_t h, int dtype) { return dtype == 0 ? dec_f16(h) : dec_bf16(h); }

/* exported for the decoder's own pin (compared with numpy's float16 view) */
void oracle_decode(const uint16_t *src, double *dst, int64_t n, int dtype)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = dec(src[i], dtype);
}

/*
 * Rows rows[0..nrows) of C = A*B (rows == NULL: rows 0..nrows-1).
 * A [M,K], B [K,N] row-major bit patterns; C, Cabs [nrows,N] fp64 (Cabs may be NULL).
 * Each C element is built by additions in ascending k, whatever the loop nest
 * order: the i-k-j nest below adds a[i,k]*b[k,j] to C[i,j] for k = 0,1,2,...
 */
int oracle_matmul_rows(const uint16_t *A, const uint16_t *B, double *C, double *Cabs,
                       int64_t M, int64_t N, int64_t K, const int64_t *rows, int64_t nrows,
                       int dtype)
{
    if (M < 0 || N < 0 || K < 0 || nrows < 0) return -1;
    if (nrows == 0 || N == 0) return 0;
    double *Bd = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1) * (size_t)N);
    if (!Bd) return -2;
    for (int64_t t = 0; t < K * N; ++t) Bd[t] = dec(B[t], dtype);
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t i = rows ? rows[r] : r;
        double *c = C + r * N;
        double *ca = Cabs ? Cabs + r * N : NULL;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        if (ca) for (int64_t j = 0; j < N; ++j) ca[j] = 0.0;
        if (i < 0 || i >= M) continue;
        for (int64_t k = 0; k < K; ++k) {
            double a = dec(A[i * K + k], dtype);
            const double *b = Bd + k * N;
            for (int64_t j = 0; j < N; ++j) c[j] += a * b[j];
            if (ca) {
                double aa = fabs(a);
                for (int64_t j = 0; j < N; ++j) ca[j] += aa * fabs(b[j]);
            }
        }
    }
    free(Bd);
    return 0;
}

int oracle_matmul(const uint16_t *A, const uint16_t *B, double *C, double *Cabs,
                  int64_t M, int64_t N, int64_t K, int dtype)
{
    return oracle_matmul_rows(A, B, C, Cabs, M, N, K, NULL, M, dtype);
}

int oracle_bmm(const uint16_t *A, const uint16_t *B, double *C, double *Cabs,
               int64_t batch, int64_t M, int64_t N, int64_t K, int dtype)
{
    for (int64_t b = 0; b < batch; ++b) {
        int rc = oracle_matmul(A + b * M * K, B + b * K * N, C + b * M * N,
                               Cabs ? Cabs + b * M * N : NULL, M, N, K, dtype);
        if (rc) return rc;
    }
    return 0;
}

/*
 * Output pixels pix[0..npix) (flattened (n*P + p)*Q + q; pix == NULL: 0..npix-1) of the
 * NHWC convolution.  X [Nimg,H,W,Cin], Wt [R,S,Cin,Cout], Y/Yabs [npix,Cout] fp64.
 * Reduce order: r, then s, then c (ascending), the order of the flattened reduce index
 * (r*S + s)*Cin + c.
 */
int oracle_conv2d_nhwc_pixels(const uint16_t *X, const uint16_t *Wt, double *Y, double *Yabs,
                              int64_t Nimg, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                              int64_t R, int64_t S, int64_t stride, int64_t pad,
                              const int64_t *pix, int64_t npix, int dtype)
{
    if (stride <= 0 || H + 2 * pad < R || W + 2 * pad < S) return -1;
    int64_t P = (H + 2 * pad - R) / stride + 1;
    int64_t Q = (W + 2 * pad - S) / stride + 1;
    int64_t nw = R * S * Cin * Cout;
    double *Wd = (double *)malloc(sizeof(double) * (size_t)(nw > 0 ? nw : 1));
    if (!Wd) return -2;
    for (int64_t t = 0; t < nw; ++t) Wd[t] = dec(Wt[t], dtype);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < npix; ++t) {
        int64_t o = pix ? pix[t] : t;
        double *y = Y + t * Cout;
        double *ya = Yabs ? Yabs + t * Cout : NULL;
        for (int64_t k = 0; k < Cout; ++k) y[k] = 0.0;
        if (ya) for (int64_t k = 0; k < Cout; ++k) ya[k] = 0.0;
        if (o < 0 || o >= Nimg * P * Q) continue;
        int64_t n = o / (P * Q), p = (o / Q) % P, q = o % Q;
        for (int64_t r = 0; r < R; ++r)
            for (int64_t s = 0; s < S; ++s) {
                int64_t h = p * stride - pad + r, w = q * stride - pad + s;
                if (h < 0 || h >= H || w < 0 || w >= W) continue;   /* zero padding */
                for (int64_t c = 0; c < Cin; ++c) {
                    double x = dec(X[((n * H + h) * W + w) * Cin + c], dtype);
                    const double *wr = Wd + ((r * S + s) * Cin + c) * Cout;
                    for (int64_t k = 0; k < Cout; ++k) y[k] += x * wr[k];
                    if (ya) {
                        double ax = fabs(x);
                        for (int64_t k = 0; k < Cout; ++k) ya[k] += ax * fabs(wr[k]);
                    }
                }
            }
    }
    free(Wd);
    return 0;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
