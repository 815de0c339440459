/*
 * CPU oracle for the Shfl-BW hot path.  TEST INFRASTRUCTURE ONLY: nothing in
 * the product (the HIP library, its Python binding) may include, link or call
 * this file; only the tests, the smoke check and the benchmark's CPU-baseline
 * leg do.  It shares no code with the GPU path.
 *
 * What it computes.  The paper's kernels are an exact reformulation of a
 * masked matrix product (Section 2.1: "GEMM turns into an SpMM"; Algorithm 1:
 * data A.values/A.metadata/A.row_indices, B[K][N], result C[M][N]; Section
 * 4.2: the row order of the output is restored at write-back).  The result
 * therefore has a plain definition that never mentions the compressed
 * format or the permutation:
 *
 *     Y[i][j] = sum over k with mask[i][k] != 0 of  W[i][k] * X[k][j]
 *
 * and for convolution (Section 4.1, implicit GEMM: the feature map is
 * unfolded to matrix form, cross-correlation, zero padding)
 *
 *     out[b][o][y][x] = sum over (c,r,s) with mask[o][(c*R+r)*S+s] != 0 of
 *         W[o][(c*R+r)*S+s] * in[b][c][y*sh + r - ph][x*sw + s - pw]
 *
 * with out-of-range input positions contributing zero.
 *
 * Precision: inputs are 16-bit patterns, IEEE binary16 (the half precision
 * the paper measures in) or bfloat16 (format 1, the other 16-bit operand type
 * of the matrix cores), widened exactly to double; every product of two such
 * values is exact in double; sums are accumulated in double.  Alongside Y the oracle returns the scale
 * S[i][j] = sum |W||X| over the same terms, which the parity tolerance
 * (|Y_gpu - Y| <= 2^-10 * S) is stated against.
 *
 * Loop order is i (rows, OpenMP) - k (kept columns only) - j, so the work
 * done is the useful 2*nnz*N multiply-adds, nothing blocked or fused.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE 754 binary16 -> double, written out from the format's definition:
 * 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits; exponent 0 is
 * subnormal (no hidden one), exponent 31 is Inf/NaN. */
double oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 31;
    int f = h & 1023;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);               /* f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 25);   /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* bfloat16 -> double from the format's definition: 1 sign bit, 8 exponent
 * bits (bias 127), 7 fraction bits; exponent 0 is subnormal, 255 is Inf/NaN. */
double oracle_bfloat16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 7) & 255;
    int f = h & 127;
    double v;
    if (e == 0)
        v = ldexp((double)f, -133);              /* f * 2^-7 * 2^-126 */
    else if (e == 255)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(128 + f), e - 134);   /* (1 + f/128) * 2^(e-127) */
    return sign ? -v : v;
}

/* format 0 = binary16, 1 = bfloat16 */
static inline double widen(uint16_t h, int format)
{
    return format == 1 ? oracle_bfloat16_to_double(h) : oracle_half_to_double(h);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Masked product.  W: M x K binary16 bits, row-major, leading dimension K.
 * mask: M x K bytes (non-zero = kept).  X: K x N binary16 bits, row-major.
 * Y, S: M x N doubles, row-major (S may be NULL).  Returns 0, or -1 when a
 * work buffer cannot be allocated.
 */
int oracle_spmm_fmt(const uint16_t *W, const uint8_t *mask, const uint16_t *X,
                    int64_t M, int64_t K, int64_t N, double *Y, double *S, int format)
{
    double *Xd = (double *)malloc(sizeof(double) * (size_t)(K * N > 0 ? K * N : 1));
    if (!Xd) return -1;
    for (int64_t t = 0; t < K * N; ++t) Xd[t] = widen(X[t], format);

#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < M; ++i) {
        double *y = Y + i * N;
        double *s = S ? S + i * N : NULL;
        for (int64_t j = 0; j < N; ++j) y[j] = 0.0;
        if (s) for (int64_t j = 0; j < N; ++j) s[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            if (!mask[i * K + k]) continue;
            double w = widen(W[i * K + k], format);
            const double *x = Xd + k * N;
            for (int64_t j = 0; j < N; ++j) y[j] += w * x[j];
            if (s) {
                double aw = fabs(w);
                for (int64_t j = 0; j < N; ++j) s[j] += aw * fabs(x[j]);
            }
        }
    }
    free(Xd);
    return 0;
}

int oracle_spmm(const uint16_t *W, const uint8_t *mask, const uint16_t *X,
                int64_t M, int64_t K, int64_t N, double *Y, double *S)
{
    return oracle_spmm_fmt(W, mask, X, M, K, N, Y, S, 0);
}

/* Element (b, c, y, x) of an activation tensor in one of two layouts:
 * layout 0 = NCHW (x innermost), layout 1 = CHWN (batch innermost, the
 * layout the paper assumes for convolution, Section 4.3 discussion). */
static inline int64_t act_index(int layout, int64_t B, int64_t C, int64_t H, int64_t Wd,
                                int64_t b, int64_t c, int64_t y, int64_t x)
{
    if (layout == 0) return ((b * C + c) * H + y) * Wd + x;
    return ((c * H + y) * Wd + x) * B + b;
}

/*
 * Masked 2-D convolution by its definition.  Wt: Cout x (Cin*R*S) binary16,
 * flattened as k = (c*R + r)*S + s.  mask: same shape, bytes.  in: activation
 * tensor (B, Cin, H, Wd) in `layout`.  out / scale: (B, Cout, Ho, Wo) doubles
 * in the same layout (scale may be NULL).  Ho = (H + 2*ph - R)/sh + 1, same
 * for Wo.  Returns 0, -1 on allocation failure, -2 on an empty output shape.
 */
int oracle_conv2d_fmt(const uint16_t *Wt, const uint8_t *mask, const uint16_t *in,
                      int64_t B, int64_t Cin, int64_t H, int64_t Wd, int64_t Cout,
                      int64_t R, int64_t Sk, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                      int layout, double *out, double *scale, int format)
{
    if (H + 2 * ph < R || Wd + 2 * pw < Sk) return -2;
    int64_t Ho = (H + 2 * ph - R) / sh + 1;
    int64_t Wo = (Wd + 2 * pw - Sk) / sw + 1;
    int64_t K = Cin * R * Sk;
    int64_t nin = B * Cin * H * Wd;
    double *ind = (double *)malloc(sizeof(double) * (size_t)(nin > 0 ? nin : 1));
    if (!ind) return -1;
    for (int64_t t = 0; t < nin; ++t) ind[t] = widen(in[t], format);

#pragma omp parallel for collapse(2) schedule(dynamic, 4)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t o = 0; o < Cout; ++o) {
            for (int64_t y = 0; y < Ho; ++y)
                for (int64_t x = 0; x < Wo; ++x) {
                    int64_t q = act_index(layout, B, Cout, Ho, Wo, b, o, y, x);
                    out[q] = 0.0;
                    if (scale) scale[q] = 0.0;
                }
            for (int64_t c = 0; c < Cin; ++c)
                for (int64_t r = 0; r < R; ++r)
                    for (int64_t s = 0; s < Sk; ++s) {
                        int64_t k = (c * R + r) * Sk + s;
                        if (!mask[o * K + k]) continue;
                        double w = widen(Wt[o * K + k], format);
                        for (int64_t y = 0; y < Ho; ++y) {
                            int64_t iy = y * sh + r - ph;
                            if (iy < 0 || iy >= H) continue;
                            for (int64_t x = 0; x < Wo; ++x) {
                                int64_t ix = x * sw + s - pw;
                                if (ix < 0 || ix >= Wd) continue;
                                double v = ind[act_index(layout, B, Cin, H, Wd, b, c, iy, ix)];
                                int64_t q = act_index(layout, B, Cout, Ho, Wo, b, o, y, x);
                                out[q] += w * v;
                                if (scale) scale[q] += fabs(w) * fabs(v);
                            }
                        }
                    }
        }
    }
    free(ind);
    return 0;
}

int oracle_conv2d(const uint16_t *Wt, const uint8_t *mask, const uint16_t *in,
                  int64_t B, int64_t Cin, int64_t H, int64_t Wd, int64_t Cout,
                  int64_t R, int64_t Sk, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                  int layout, double *out, double *scale)
{
    return oracle_conv2d_fmt(Wt, mask, in, B, Cin, H, Wd, Cout, R, Sk, sh, sw, ph, pw, layout,
                             out, scale, 0);
}
