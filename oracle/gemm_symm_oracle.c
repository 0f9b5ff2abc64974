/*
 * CPU oracle for the product with a symmetric operand given by one triangle
 *
 *     S[m,k]    = A[m,k] if k <= m else A[k,m]        (uplo = lower: the stored lower triangle, mirrored)
 *                 A[m,k] if k >= m else A[k,m]        (uplo = upper)
 *     P[b][m,n] = sum_{k<M} S[b][m,k] * opB(B[b])[k,n]
 *     v         = alpha * row_scale[m] * P[b][m,n] + bias[n] + beta * R[b][m,n]
 *     C[b][m,n] = round_out( min(max(act(v), lo), hi) )
 *
 * TEST INFRASTRUCTURE ONLY.  Slow, plain reference for the GPU library's
 * symmetric-operand path; nothing on the product path may call it and it shares
 * no code, header, table or helper with the HIP kernels.
 *
 * The paper's optimisation prompt ("Rules for GEMM") asks to use what is known
 * about an operand and names the symmetric case: the reads of such an operand can
 * be reduced, because one triangle determines the matrix.  What is computed is
 * the ordinary product with the full symmetric matrix S; this file writes that
 * definition out, taking S element by element from the stored triangle, so that
 * the other triangle of the array is never touched (it may hold anything).  The
 * consumer chain and its order are those of the widened operator's oracle
 * (gemm_fused_oracle.c), restated here so that the two files stay independent.
 * A is square (M x M, leading dimension lda, batches packed M*lda apart).
 *
 * Loop order m, n, k: one fp64 accumulator per output, k ascending.
 *
 * Pins (tests/test_oracle_symm_pins.py): exact rational brute force, the widened
 * operator's oracle on the explicitly mirrored dense matrix, NaN in the unread
 * triangle, all-ones and diagonal closed forms, agreement of the two readings on a
 * symmetric array and their disagreement on an asymmetric one.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { SYMM_ACT_NONE = 0, SYMM_ACT_RELU = 1, SYMM_ACT_GELU_TANH = 2 };
enum { SYMM_IN_F64 = 0, SYMM_IN_F32 = 1, SYMM_IN_BF16 = 2 };
enum { SYMM_OUT_F64 = 0, SYMM_OUT_F32 = 1, SYMM_OUT_BF16 = 2 };
enum { SYMM_LOWER = 0, SYMM_UPPER = 1 };

static double value_at(const void *base, int kind, size_t index)
{
    if (kind == SYMM_IN_F64) return ((const double *)base)[index];
    if (kind == SYMM_IN_F32) return (double)((const float *)base)[index];
    uint32_t w = ((uint32_t)((const uint16_t *)base)[index]) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* nearest bf16 (ties to even) of a finite fp32 value, as that value */
static double to_bf16(float x)
{
    uint32_t w;
    memcpy(&w, &x, sizeof w);
    if ((w & 0x7F800000u) != 0x7F800000u) {
        uint32_t lower = w & 0xFFFFu;
        w &= 0xFFFF0000u;
        if (lower > 0x8000u || (lower == 0x8000u && (w & 0x10000u))) w += 0x10000u;
    } else {
        w &= 0xFFFF0000u;
    }
    float r;
    memcpy(&r, &w, sizeof r);
    return (double)r;
}

int oracle_gemm_symm(int M, int N, int batch,
                     const void *A, long lda, int uplo,
                     const void *B, long ldb, int transB, int in_kind,
                     double alpha, const double *row_scale, const double *bias,
                     const void *R, long ldr, int r_kind, double beta,
                     int act, double lo, double hi, int out_kind,
                     double *C, long ldc)
{
    if (M < 1 || N < 1 || batch < 1 || !A || !B || !C) return -1;
    if (lda < M || ldb < (transB ? M : N) || ldc < N) return -1;
    if (R && ldr < N) return -1;
    if (uplo != SYMM_LOWER && uplo != SYMM_UPPER) return -1;
    if (act < SYMM_ACT_NONE || act > SYMM_ACT_GELU_TANH) return -1;
    if (in_kind < SYMM_IN_F64 || in_kind > SYMM_IN_BF16) return -1;
    if (R && (r_kind < SYMM_IN_F64 || r_kind > SYMM_IN_BF16)) return -1;
    if (out_kind < SYMM_OUT_F64 || out_kind > SYMM_OUT_BF16) return -1;
    if (!(lo <= hi)) return -1;

    const size_t batchA = (size_t)M * (size_t)lda;
    const size_t batchB = (size_t)(transB ? N : M) * (size_t)ldb;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < batch; ++b) {
        for (int m = 0; m < M; ++m) {
            for (int n = 0; n < N; ++n) {
                double p = 0.0;
                for (int k = 0; k < M; ++k) {
                    /* the element of the stored triangle that S[m,k] is */
                    const int stored = uplo == SYMM_LOWER ? (k <= m) : (k >= m);
                    const size_t row = stored ? (size_t)m : (size_t)k, col = stored ? (size_t)k : (size_t)m;
                    const size_t ib = b * batchB + (transB ? (size_t)n * ldb + k : (size_t)k * ldb + n);
                    p += value_at(A, in_kind, b * batchA + row * lda + col) * value_at(B, in_kind, ib);
                }
                double v = alpha * p;
                if (row_scale) v = row_scale[m] * v;
                if (bias) v = v + bias[n];
                if (R) v = v + beta * value_at(R, r_kind, ((size_t)b * M + m) * (size_t)ldr + n);
                double y = v;
                if (act == SYMM_ACT_RELU) y = v > 0.0 ? v : 0.0;
                if (act == SYMM_ACT_GELU_TANH) y = 0.5 * v * (1.0 + tanh(0.7978845608028654 * (v + 0.044715 * v * v * v)));
                if (y < lo) y = lo;
                if (y > hi) y = hi;
                if (out_kind == SYMM_OUT_F32) y = (double)(float)y;
                if (out_kind == SYMM_OUT_BF16) y = to_bf16((float)y);
                C[((size_t)b * M + m) * (size_t)ldc + n] = y;
            }
        }
    }
    return 0;
}
