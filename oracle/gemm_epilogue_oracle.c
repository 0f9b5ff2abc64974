/*
 * CPU oracle for the fused operator  C = act(alpha * A*B + bias).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU
 * library is checked against.  Nothing on the product path may call it, and it
 * shares no code, header, table or helper with the HIP kernels.
 *
 * What it computes, and where the paper fixes it:
 *   - the contraction is the plain row-major definition of the paper's naive
 *     baseline kernel (appendix "Comparison of CuTe and CUDA Representations
 *     for Square GEMM", Fig. simp_cuda): C[m,n] = sum_k A[m*lda+k]*B[k*ldb+n],
 *     k ascending, A is [M,K] row-major and B is [K,N] row-major (also the
 *     operand convention of the optimisation prompt's GEMM section);
 *   - the writeback scales the accumulator and adds no previous C (the initial
 *     CuTe kernel's epilogue is 1.0*acc + 0.0*C, Fig. simple_cute);
 *   - bias, scale and activation are applied to the producer value before the
 *     single store (Level-2 optimisation prompt, "Fusion": bias/add/scale/
 *     activation fused into the producer writeback).  The order scale -> bias
 *     -> activation, the per-column bias and the tanh form of GELU are this
 *     repository's reading; the paper only names the operations;
 *   - precision is never lowered (Experiments, "Manual Correctness Audit"):
 *     every product and sum here is fp64, operands are widened exactly.
 *
 * Loop order is m, k, n with one fp64 accumulator per output column of the
 * current row: still the triple loop, each output still sums k = 0..K-1 in
 * ascending order, so the result does not depend on the thread count (OpenMP
 * splits rows and batches only).
 *
 * Pins (tests/test_oracle_pins.py): exact rational brute force on tiny inputs,
 * integer-valued inputs, identity B, all-ones closed form, linearity in alpha,
 * transposition identity, bias difference, relu and gelu_tanh identities, a
 * library gelu, batch slicing, padded leading dimensions.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_RELU = 1, ORACLE_ACT_GELU_TANH = 2 };
enum { ORACLE_IN_F64 = 0, ORACLE_IN_F32 = 1, ORACLE_IN_BF16 = 2 };

/* A bf16 value is the upper half of an IEEE binary32 pattern: widening is exact. */
static double widen_bf16(uint16_t bits)
{
    uint32_t w = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

static double widen_f64(double x) { return x; }
static double widen_f32(float x) { return (double)x; }

/*
 * One output row: acc[n] = sum_k A[m,k] * B[k,n], k ascending, fp64.
 * Written once per operand type so the inner loop carries no type switch.
 */
#define ORACLE_ROW_KERNEL(NAME, T, WIDEN)                                      \
    static void NAME(int N, int K, const T *a_row, const T *b_mat, long ldb,   \
                     double *acc)                                              \
    {                                                                          \
        for (int n = 0; n < N; ++n) acc[n] = 0.0;                              \
        for (int k = 0; k < K; ++k) {                                          \
            double a = WIDEN(a_row[k]);                                        \
            const T *b_row = b_mat + (size_t)k * ldb;                          \
            for (int n = 0; n < N; ++n) acc[n] += a * WIDEN(b_row[n]);         \
        }                                                                      \
    }
ORACLE_ROW_KERNEL(row_f64, double, widen_f64)
ORACLE_ROW_KERNEL(row_f32, float, widen_f32)
ORACLE_ROW_KERNEL(row_bf16, uint16_t, widen_bf16)

/* gelu_tanh(v) = 0.5 v (1 + tanh( sqrt(2/pi) (v + 0.044715 v^3) )) */
static double act_apply(double v, int act)
{
    if (act == ORACLE_ACT_RELU)
        return v > 0.0 ? v : 0.0;
    if (act == ORACLE_ACT_GELU_TANH) {
        const double c = 0.7978845608028654; /* sqrt(2/pi) */
        double u = c * (v + 0.044715 * v * v * v);
        return 0.5 * v * (1.0 + tanh(u));
    }
    return v;
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
 * C[b][m,n] = act(alpha * sum_k A[b][m,k] * B[b][k,n] + bias[n])   (fp64 out)
 *
 * kind: element type of A and B (ORACLE_IN_*).  bias (nullable, length N,
 * shared by every batch) and alpha are fp64 already (the caller widens the
 * fp32 values exactly).  Batch b starts at A + b*M*lda, B + b*K*ldb,
 * C + b*M*ldc (packed strides).  Returns 0, or -1 on a bad argument.
 */
int oracle_gemm_epilogue(int M, int N, int K,
                         const void *A, long lda, const void *B, long ldb,
                         int kind, const double *bias, double alpha, int act,
                         double *C, long ldc, int batch)
{
    if (M < 1 || N < 1 || K < 1 || batch < 1 || !A || !B || !C) return -1;
    if (lda < K || ldb < N || ldc < N) return -1;
    if (act < ORACLE_ACT_NONE || act > ORACLE_ACT_GELU_TANH) return -1;
    if (kind < ORACLE_IN_F64 || kind > ORACLE_IN_BF16) return -1;

    long rows = (long)batch * M;
    int failed = 0;
#pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)N);
        if (!acc) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (long r = 0; r < rows; ++r) {
            if (!acc) continue;
            long b = r / M, m = r % M;
            size_t a_off = (size_t)b * M * lda + (size_t)m * lda;
            size_t b_off = (size_t)b * K * ldb;
            double *c_row = C + (size_t)b * M * ldc + (size_t)m * ldc;
            if (kind == ORACLE_IN_F64)
                row_f64(N, K, (const double *)A + a_off, (const double *)B + b_off, ldb, acc);
            else if (kind == ORACLE_IN_F32)
                row_f32(N, K, (const float *)A + a_off, (const float *)B + b_off, ldb, acc);
            else
                row_bf16(N, K, (const uint16_t *)A + a_off, (const uint16_t *)B + b_off, ldb, acc);
            for (int n = 0; n < N; ++n) {
                double v = alpha * acc[n] + (bias ? bias[n] : 0.0);
                c_row[n] = act_apply(v, act);
            }
        }
        free(acc);
    }
    return failed ? -1 : 0;
}
