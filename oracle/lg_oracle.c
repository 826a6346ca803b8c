/*
 * lg_oracle.c -- plain CPU oracle for the structured tensor ops.
 *
 * TEST INFRASTRUCTURE ONLY.  This file exists to check the GPU library; it is
 * never part of the product path.  It shares no code, header, table or helper
 * with the HIP sources, and the GPU library never calls it.
 *
 * Every function is the naive loop nest of the op's index-notation definition
 * in the paper, over the full rectangular iteration domain, with no blocking,
 * fusion or reordering.  The reduction iterators run innermost in the order the
 * definition lists them.  The scalar body (one multiply, one add) is evaluated
 * in fp64 and the sum is rounded to fp32 once, so the oracle's own error is at
 * most half an ulp of the exact result; the paper leaves the reduction order
 * unspecified (its iterators are unordered "parallel"/"reduction" iterators,
 * Section 2.3, linalg dialect), so the exact sum is the reference every
 * admissible order is measured against.
 *
 * All pointers are HOST pointers to row-major fp32 data; extents and leading
 * dimensions are in elements.  `accumulate` != 0 adds the computed value to
 * what the output already holds (destination-passing style, Section 3.4);
 * `accumulate` == 0 overwrites it.  Return value: 0 on success, -1 on an
 * invalid argument.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (brute force in exact rational arithmetic, closed forms, identities between
 * the ops).  Nothing in this file is "parity unpinned".
 *
 * The only concession to run time is an OpenMP `parallel for` over the
 * outermost parallel iterator; it does not change any value.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define LGO_OK 0
#define LGO_ERR_INVALID_ARG (-1)

/* Number of host threads the parallel-for loops below use. */
int lgo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Output extent of a strided, dilated window over an input extent with no
 * padding: the largest extent for which every access in*S + k*D stays inside
 * the input (Section 3, iteration-domain rule "iterators span the entire data
 * of the operands").  Returns 0 when the dilated window does not fit. */
int64_t lgo_conv_out_extent(int64_t in, int64_t k, int64_t s, int64_t d)
{
    if (in <= 0 || k <= 0 || s <= 0 || d <= 0) return 0;
    int64_t span = d * (k - 1) + 1;
    if (span > in) return 0;
    return (in - span) / s + 1;
}

/* Section 4.6.1, equation (AB):  C[m,n] = sum_k A[m,k] * B[k,n]. */
int lgo_matmul(const float *A, const float *B, float *C,
               int64_t M, int64_t N, int64_t K,
               int64_t lda, int64_t ldb, int64_t ldc, int accumulate)
{
    if (M < 0 || N < 0 || K < 0) return LGO_ERR_INVALID_ARG;
    if (lda < K || ldb < N || ldc < N) return LGO_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return LGO_OK;
    if (!C || (K > 0 && (!A || !B))) return LGO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k)
                s += (double)A[m * lda + k] * (double)B[k * ldb + n];
            if (accumulate) s += (double)C[m * ldc + n];
            C[m * ldc + n] = (float)s;
        }
    }
    return LGO_OK;
}

/* Section 4.6.1, equations (A^T B) and (A B^T):
 *   transA: C[m,n] = sum_k A[k,m] * B[k,n]   (A stored K x M)
 *   transB: C[m,n] = sum_k A[m,k] * B[n,k]   (B stored N x K)
 * Both flags clear is equation (AB); both set is rejected (not one of the paper's variants). */
int lgo_matmul_t(const float *A, const float *B, float *C,
                 int64_t M, int64_t N, int64_t K,
                 int64_t lda, int64_t ldb, int64_t ldc,
                 int transA, int transB, int accumulate)
{
    if (M < 0 || N < 0 || K < 0 || ldc < N) return LGO_ERR_INVALID_ARG;
    if (transA && transB) return LGO_ERR_INVALID_ARG;
    if (lda < (transA ? M : K) || ldb < (transB ? K : N)) return LGO_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return LGO_OK;
    if (!C || (K > 0 && (!A || !B))) return LGO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double a = transA ? (double)A[k * lda + m] : (double)A[m * lda + k];
                double b = transB ? (double)B[n * ldb + k] : (double)B[k * ldb + n];
                s += a * b;
            }
            if (accumulate) s += (double)C[m * ldc + n];
            C[m * ldc + n] = (float)s;
        }
    }
    return LGO_OK;
}

/* Section 4.6.2, equation (2-D):
 *   O[n,h,w,f] = sum_{kh,kw,c} I[n, h*SH + kh*DH, w*SW + kw*DW, c] * K[kh,kw,c,f]
 * I is [N,H,W,C], K is [KH,KW,C,F], O is [N,OH,OW,F], all contiguous. */
int lgo_conv2d_nhwc_hwcf(const float *I, const float *Kf, float *O,
                         int64_t N, int64_t H, int64_t W, int64_t C,
                         int64_t KH, int64_t KW, int64_t F,
                         int64_t SH, int64_t SW, int64_t DH, int64_t DW,
                         int accumulate)
{
    if (N < 0 || H < 0 || W < 0 || C < 0 || KH < 0 || KW < 0 || F < 0)
        return LGO_ERR_INVALID_ARG;
    if (SH < 1 || SW < 1 || DH < 1 || DW < 1) return LGO_ERR_INVALID_ARG;
    if (KH == 0 || KW == 0) return LGO_ERR_INVALID_ARG;
    if (N == 0 || F == 0) return LGO_OK;
    int64_t OH = lgo_conv_out_extent(H, KH, SH, DH);
    int64_t OW = lgo_conv_out_extent(W, KW, SW, DW);
    if (OH == 0 || OW == 0) return LGO_ERR_INVALID_ARG;
    if (!O || (C > 0 && (!I || !Kf))) return LGO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t h = 0; h < OH; ++h) {
            for (int64_t w = 0; w < OW; ++w) {
                for (int64_t f = 0; f < F; ++f) {
                    double s = 0.0;
                    for (int64_t kh = 0; kh < KH; ++kh)
                        for (int64_t kw = 0; kw < KW; ++kw)
                            for (int64_t c = 0; c < C; ++c) {
                                int64_t ih = h * SH + kh * DH;
                                int64_t iw = w * SW + kw * DW;
                                s += (double)I[((n * H + ih) * W + iw) * C + c] *
                                     (double)Kf[((kh * KW + kw) * C + c) * F + f];
                            }
                    int64_t o = ((n * OH + h) * OW + w) * F + f;
                    if (accumulate) s += (double)O[o];
                    O[o] = (float)s;
                }
            }
        }
    }
    return LGO_OK;
}

/* Section 3 (running example) and Section 4.6.2, equation (1-D):
 *   O[n,w,f] = sum_{kw,c} I[n, w*SW + kw*DW, c] * K[kw,c,f]
 * I is [N,W,C], K is [KW,C,F], O is [N,OW,F], all contiguous. */
int lgo_conv1d_nwc_wcf(const float *I, const float *Kf, float *O,
                       int64_t N, int64_t W, int64_t C, int64_t KW, int64_t F,
                       int64_t SW, int64_t DW, int accumulate)
{
    if (N < 0 || W < 0 || C < 0 || KW < 1 || F < 0) return LGO_ERR_INVALID_ARG;
    if (SW < 1 || DW < 1) return LGO_ERR_INVALID_ARG;
    if (N == 0 || F == 0) return LGO_OK;
    int64_t OW = lgo_conv_out_extent(W, KW, SW, DW);
    if (OW == 0) return LGO_ERR_INVALID_ARG;
    if (!O || (C > 0 && (!I || !Kf))) return LGO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t w = 0; w < OW; ++w) {
            for (int64_t f = 0; f < F; ++f) {
                double s = 0.0;
                for (int64_t kw = 0; kw < KW; ++kw)
                    for (int64_t c = 0; c < C; ++c) {
                        int64_t x = w * SW + kw * DW;
                        s += (double)I[(n * W + x) * C + c] * (double)Kf[(kw * C + c) * F + f];
                    }
                int64_t o = (n * OW + w) * F + f;
                if (accumulate) s += (double)O[o];
                O[o] = (float)s;
            }
        }
    }
    return LGO_OK;
}

/* Section 4.6.2 asks for conv against an independent formulation: materialise
 * the window matrix col[(n,h,w),(kh,kw,c)] = I[n,h*SH+kh*DH,w*SW+kw*DW,c]
 * explicitly; the caller then multiplies it with K viewed as [KH*KW*C, F]
 * through lgo_matmul.  col must hold N*OH*OW rows of KH*KW*C floats. */
int lgo_im2col_nhwc(const float *I, float *col,
                    int64_t N, int64_t H, int64_t W, int64_t C,
                    int64_t KH, int64_t KW,
                    int64_t SH, int64_t SW, int64_t DH, int64_t DW)
{
    if (N < 0 || H < 0 || W < 0 || C < 0 || KH < 1 || KW < 1) return LGO_ERR_INVALID_ARG;
    if (SH < 1 || SW < 1 || DH < 1 || DW < 1) return LGO_ERR_INVALID_ARG;
    int64_t OH = lgo_conv_out_extent(H, KH, SH, DH);
    int64_t OW = lgo_conv_out_extent(W, KW, SW, DW);
    if (OH == 0 || OW == 0) return LGO_ERR_INVALID_ARG;
    if (N == 0 || C == 0) return LGO_OK;
    if (!I || !col) return LGO_ERR_INVALID_ARG;
    int64_t Kg = KH * KW * C;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t h = 0; h < OH; ++h)
            for (int64_t w = 0; w < OW; ++w) {
                int64_t row = (n * OH + h) * OW + w;
                for (int64_t kh = 0; kh < KH; ++kh)
                    for (int64_t kw = 0; kw < KW; ++kw)
                        for (int64_t c = 0; c < C; ++c)
                            col[row * Kg + (kh * KW + kw) * C + c] =
                                I[((n * H + h * SH + kh * DH) * W + w * SW + kw * DW) * C + c];
            }
    return LGO_OK;
}

/* Section 4.7, equation (1-D):
 *   O[n,w,c] = sum_kw I[n, w*SW + kw*DW, c] * K[kw,c]
 * I is [N,W,C], K is [KW,C], O is [N,OW,C]. */
int lgo_dwconv1d_nwc_wc(const float *I, const float *Kf, float *O,
                        int64_t N, int64_t W, int64_t C, int64_t KW,
                        int64_t SW, int64_t DW, int accumulate)
{
    if (N < 0 || W < 0 || C < 0 || KW < 1) return LGO_ERR_INVALID_ARG;
    if (SW < 1 || DW < 1) return LGO_ERR_INVALID_ARG;
    if (N == 0 || C == 0) return LGO_OK;
    int64_t OW = lgo_conv_out_extent(W, KW, SW, DW);
    if (OW == 0) return LGO_ERR_INVALID_ARG;
    if (!I || !Kf || !O) return LGO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t w = 0; w < OW; ++w) {
            for (int64_t c = 0; c < C; ++c) {
                double s = 0.0;
                for (int64_t kw = 0; kw < KW; ++kw)
                    s += (double)I[(n * W + w * SW + kw * DW) * C + c] *
                         (double)Kf[kw * C + c];
                int64_t o = (n * OW + w) * C + c;
                if (accumulate) s += (double)O[o];
                O[o] = (float)s;
            }
        }
    }
    return LGO_OK;
}

/* Section 4.7, equation (2-D):
 *   O[n,h,w,c] = sum_{kh,kw} I[n, h*SH + kh*DH, w*SW + kw*DW, c] * K[kh,kw,c]
 * I is [N,H,W,C], K is [KH,KW,C], O is [N,OH,OW,C]. */
int lgo_dwconv2d_nhwc_hwc(const float *I, const float *Kf, float *O,
                          int64_t N, int64_t H, int64_t W, int64_t C,
                          int64_t KH, int64_t KW,
                          int64_t SH, int64_t SW, int64_t DH, int64_t DW,
                          int accumulate)
{
    if (N < 0 || H < 0 || W < 0 || C < 0 || KH < 1 || KW < 1) return LGO_ERR_INVALID_ARG;
    if (SH < 1 || SW < 1 || DH < 1 || DW < 1) return LGO_ERR_INVALID_ARG;
    if (N == 0 || C == 0) return LGO_OK;
    int64_t OH = lgo_conv_out_extent(H, KH, SH, DH);
    int64_t OW = lgo_conv_out_extent(W, KW, SW, DW);
    if (OH == 0 || OW == 0) return LGO_ERR_INVALID_ARG;
    if (!I || !Kf || !O) return LGO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t h = 0; h < OH; ++h) {
            for (int64_t w = 0; w < OW; ++w) {
                for (int64_t c = 0; c < C; ++c) {
                    double s = 0.0;
                    for (int64_t kh = 0; kh < KH; ++kh)
                        for (int64_t kw = 0; kw < KW; ++kw)
                            s += (double)I[((n * H + h * SH + kh * DH) * W +
                                            w * SW + kw * DW) * C + c] *
                                 (double)Kf[(kh * KW + kw) * C + c];
                    int64_t o = ((n * OH + h) * OW + w) * C + c;
                    if (accumulate) s += (double)O[o];
                    O[o] = (float)s;
                }
            }
        }
    }
    return LGO_OK;
}

/* Section 4.4, RowRed2D: out[i] = sum_j in[i,j].  The reduced dimension is the
 * contiguous one; the result has one entry per row (Section 4.5.3: a 250x960
 * input gives a 250-element output). */
int lgo_reduce_rows(const float *in, float *out, int64_t R, int64_t Cn, int64_t ld,
                    int accumulate)
{
    if (R < 0 || Cn < 0 || ld < Cn) return LGO_ERR_INVALID_ARG;
    if (R == 0) return LGO_OK;
    if (!out || (Cn > 0 && !in)) return LGO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < R; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < Cn; ++j) s += (double)in[i * ld + j];
        if (accumulate) s += (double)out[i];
        out[i] = (float)s;
    }
    return LGO_OK;
}

/* Section 4.4, ColRed2D: out[j] = sum_i in[i,j]; one entry per column
 * (a 250x960 input gives a 960-element output). */
int lgo_reduce_cols(const float *in, float *out, int64_t R, int64_t Cn, int64_t ld,
                    int accumulate)
{
    if (R < 0 || Cn < 0 || ld < Cn) return LGO_ERR_INVALID_ARG;
    if (Cn == 0) return LGO_OK;
    if (!out || (R > 0 && !in)) return LGO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < Cn; ++j) {
        double s = 0.0;
        for (int64_t i = 0; i < R; ++i) s += (double)in[i * ld + j];
        if (accumulate) s += (double)out[j];
        out[j] = (float)s;
    }
    return LGO_OK;
}

/* Section 4.4, Transpose2D: out[j,i] = in[i,j].  Pure data movement: the
 * 32-bit pattern is copied, never interpreted as a number. */
int lgo_transpose(const float *in, float *out, int64_t R, int64_t Cn,
                  int64_t ld_in, int64_t ld_out)
{
    if (R < 0 || Cn < 0 || ld_in < Cn || ld_out < R) return LGO_ERR_INVALID_ARG;
    if (R == 0 || Cn == 0) return LGO_OK;
    if (!in || !out) return LGO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < R; ++i)
        for (int64_t j = 0; j < Cn; ++j)
            memcpy(&out[j * ld_out + i], &in[i * ld_in + j], sizeof(float));
    return LGO_OK;
}

/* Section 4.4: a transpose of more than two dimensions written as B0 x B1 2-D
 * transposes placed by element strides,
 *   out[b0*os0 + b1*os1 + j*ld_out + i] = in[b0*is0 + b1*is1 + i*ld_in + j]. */
int lgo_transpose_batched(const float *in, float *out, int64_t R, int64_t Cn,
                          int64_t ld_in, int64_t ld_out, int64_t B0, int64_t B1,
                          int64_t is0, int64_t is1, int64_t os0, int64_t os1)
{
    if (R < 0 || Cn < 0 || B0 < 0 || B1 < 0 || ld_in < Cn || ld_out < R) return LGO_ERR_INVALID_ARG;
    if (is0 < 0 || is1 < 0 || os0 < 0 || os1 < 0) return LGO_ERR_INVALID_ARG;
    if (R == 0 || Cn == 0 || B0 == 0 || B1 == 0) return LGO_OK;
    if (!in || !out) return LGO_ERR_INVALID_ARG;
    for (int64_t b0 = 0; b0 < B0; ++b0)
        for (int64_t b1 = 0; b1 < B1; ++b1)
            for (int64_t i = 0; i < R; ++i)
                for (int64_t j = 0; j < Cn; ++j)
                    memcpy(&out[b0 * os0 + b1 * os1 + j * ld_out + i],
                           &in[b0 * is0 + b1 * is1 + i * ld_in + j], sizeof(float));
    return LGO_OK;
}

/* Section 4.4, Copy2D: out[i,j] = in[i,j]; the paper's bandwidth yardstick. */
int lgo_copy2d(const float *in, float *out, int64_t R, int64_t Cn,
               int64_t ld_in, int64_t ld_out)
{
    if (R < 0 || Cn < 0 || ld_in < Cn || ld_out < Cn) return LGO_ERR_INVALID_ARG;
    if (R == 0 || Cn == 0) return LGO_OK;
    if (!in || !out) return LGO_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < R; ++i)
        for (int64_t j = 0; j < Cn; ++j)
            memcpy(&out[i * ld_out + j], &in[i * ld_in + j], sizeof(float));
    return LGO_OK;
}
