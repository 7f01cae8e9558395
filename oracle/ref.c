/*
 * CPU oracle for the dense contraction and the convolution lowered to it.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is checked against; nothing on the product path may call it.  It shares
 * no code, header, table or helper with the HIP sources.
 *
 * What it computes (paper, Case Study 4, Fig. 7: the loop nest
 * C[b,i,j] += A[b,i,k] * B[b,k,j]; Case Study 3: the rewrites that fold a
 * transpose into the matmul operand, sink a negate, and skip elements produced by
 * zero padding):
 *
 *   R[i][j] = sum_k opA(i,k) * B[k][j]          accumulated in fp64
 *   S[i][j] = sum_k |opA(i,k)| * |B[k][j]|      (forward-error denominator)
 *
 * with opA(i,k) = A[i*lda + k] (plain) or A[k*lda + i] (left operand stored
 * transposed).  The convolution is the direct seven-loop form, NOT an implicit
 * GEMM, so the GPU's index map is checked by an independent route.
 *
 * Pins (tests marked "not gpu"): identity and all-ones closed forms, one-hot
 * locality probes, A^T.B = (B^T.A)^T, explicit zero padding, literal Python
 * brute force on tiny integer inputs, and numpy's fp64 matmul.  The bf16 branch of
 * the convolution has pins of its own: bf16 bit patterns must give exactly what
 * the same values give as fp32, and a brute-force geometry on bf16 inputs.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int ref_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline float bf16_to_f32(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Element (i,k) of op(A) as a double.  is_bf16: A holds bfloat16 bit patterns. */
static inline double load_a(const void *A, int is_bf16, int64_t idx) {
    return is_bf16 ? (double)bf16_to_f32(((const uint16_t *)A)[idx])
                   : (double)((const float *)A)[idx];
}

/*
 * Triple loop of Fig. 7 (batch index dropped), one output row at a time with an
 * fp64 row accumulator (loop order i, k, j: still the same sum for every (i,j)).
 * S may be NULL.
 */
void ref_gemm(int is_bf16, int trans_a, int64_t M, int64_t N, int64_t K,
              const void *A, int64_t lda, const void *B, int64_t ldb,
              double *R, double *S) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *r = R + i * N;
        double *s = S ? S + i * N : NULL;
        for (int64_t j = 0; j < N; ++j) r[j] = 0.0;
        if (s) for (int64_t j = 0; j < N; ++j) s[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = load_a(A, is_bf16, trans_a ? k * lda + i : i * lda + k);
            const double aa = fabs(a);
            if (is_bf16) {
                const uint16_t *b = (const uint16_t *)B + k * ldb;
                for (int64_t j = 0; j < N; ++j) r[j] += a * (double)bf16_to_f32(b[j]);
                if (s) for (int64_t j = 0; j < N; ++j) s[j] += aa * fabs((double)bf16_to_f32(b[j]));
            } else {
                const float *b = (const float *)B + k * ldb;
                for (int64_t j = 0; j < N; ++j) r[j] += a * (double)b[j];
                if (s) for (int64_t j = 0; j < N; ++j) s[j] += aa * fabs((double)b[j]);
            }
        }
    }
}

/*
 * The same product with the right operand stored transposed as well (B is N x K,
 * row-major, and op(B)(k,j) = B[j*ldb + k] is read in place): the plain i, j, k loop.
 */
void ref_gemm_transB(int is_bf16, int trans_a, int64_t M, int64_t N, int64_t K,
                     const void *A, int64_t lda, const void *B, int64_t ldb,
                     double *R, double *S) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0, mag = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const double a = load_a(A, is_bf16, trans_a ? k * lda + i : i * lda + k);
                const double b = load_a(B, is_bf16, j * ldb + k);
                acc += a * b;
                mag += fabs(a) * fabs(b);
            }
            R[i * N + j] = acc;
            if (S) S[i * N + j] = mag;
        }
    }
}

/*
 * Direct NHWC convolution.  x [N][H][W][Cin], w [KH][KW][Cin][Cout],
 * R,S [N][Ho][Wo][Cout] with Ho = (H + 2*ph - KH)/sh + 1 (floor), same for Wo.
 * A tap whose input coordinate falls in the zero padding is skipped: the padded
 * element is never formed, read or added (Case Study 3, the zero-pad rewrite).
 */
void ref_conv2d_nhwc(int is_bf16, int64_t N, int64_t H, int64_t W, int64_t Cin,
                     int64_t Cout, int64_t KH, int64_t KW, int64_t sh, int64_t sw,
                     int64_t ph, int64_t pw, const void *x, const void *w,
                     double *R, double *S) {
    const int64_t Ho = (H + 2 * ph - KH) / sh + 1;
    const int64_t Wo = (W + 2 * pw - KW) / sw + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t ho = 0; ho < Ho; ++ho) {
            for (int64_t wo = 0; wo < Wo; ++wo) {
                double *r = R + ((n * Ho + ho) * Wo + wo) * Cout;
                double *s = S ? S + ((n * Ho + ho) * Wo + wo) * Cout : NULL;
                for (int64_t co = 0; co < Cout; ++co) r[co] = 0.0;
                if (s) for (int64_t co = 0; co < Cout; ++co) s[co] = 0.0;
                for (int64_t kh = 0; kh < KH; ++kh) {
                    const int64_t hi = ho * sh + kh - ph;
                    if (hi < 0 || hi >= H) continue;
                    for (int64_t kw = 0; kw < KW; ++kw) {
                        const int64_t wi = wo * sw + kw - pw;
                        if (wi < 0 || wi >= W) continue;
                        for (int64_t ci = 0; ci < Cin; ++ci) {
                            const double xv = load_a(x, is_bf16, ((n * H + hi) * W + wi) * Cin + ci);
                            const int64_t wbase = ((kh * KW + kw) * Cin + ci) * Cout;
                            for (int64_t co = 0; co < Cout; ++co) {
                                const double wv = load_a(w, is_bf16, wbase + co);
                                r[co] += xv * wv;
                                if (s) s[co] += fabs(xv) * fabs(wv);
                            }
                        }
                    }
                }
            }
        }
    }
}

/*
 * Index map of the lowering: for output pixel m = (n*Ho + ho)*Wo + wo and tap
 * t = kh*KW + kw, off[m*KH*KW + t] is the element offset of x[n][hi][wi][0], or -1
 * when (hi,wi) lies in the padding.  Integer work: compared bit-exactly.
 */
void ref_conv2d_index_map(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t KH,
                          int64_t KW, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                          int32_t *off) {
    const int64_t Ho = (H + 2 * ph - KH) / sh + 1;
    const int64_t Wo = (W + 2 * pw - KW) / sw + 1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo)
                for (int64_t kh = 0; kh < KH; ++kh)
                    for (int64_t kw = 0; kw < KW; ++kw) {
                        const int64_t m = (n * Ho + ho) * Wo + wo;
                        const int64_t hi = ho * sh + kh - ph, wi = wo * sw + kw - pw;
                        const int inside = hi >= 0 && hi < H && wi >= 0 && wi < W;
                        off[m * KH * KW + kh * KW + kw] =
                            inside ? (int32_t)(((n * H + hi) * W + wi) * Cin) : -1;
                    }
}

/*
 * Loop split of Fig. 1 / Fig. 8: the main part has the largest trip count that is
 * a multiple of d, the remainder has fewer than d iterations.  d == 0 means "do not
 * tile": everything is main, one tile.
 */
void ref_split(int64_t ub, int64_t d, int64_t *main_part, int64_t *rest, int64_t *tiles) {
    if (d <= 0) { *main_part = ub; *rest = 0; *tiles = 1; return; }
    *tiles = ub / d;
    *main_part = *tiles * d;
    *rest = ub - *main_part;
}
