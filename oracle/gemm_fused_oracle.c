/*
 * CPU oracle for the widened operator
 *
 *     P[b][m,n] = sum_{k<K} opA(A[b])[m,k] * opB(B[b])[k,n]
 *     v         = alpha * row_scale[m] * P[b][m,n] + bias[n] + beta * R[b][m,n]
 *     C[b][m,n] = round_out( min(max(act(v), lo), hi) )
 *
 * TEST INFRASTRUCTURE ONLY.  Slow, plain reference for the GPU library's fused
 * entry point; nothing on the product path may call it and it shares no code,
 * header, table or helper with the HIP kernels.
 *
 * Where the paper fixes it, and this repository's readings:
 *   - the contraction is the plain matmul definition of the naive baseline
 *     (appendix "Comparison of CuTe and CUDA Representations for Square GEMM",
 *     Fig. simp_cuda).  opA / opB select how the operand is stored, not what is
 *     computed: transA = 0 reads A[m,k] at A[m*lda + k], transA = 1 at
 *     A[k*lda + m]; transB = 0 reads B[k,n] at B[k*ldb + n], transB = 1 at
 *     B[n*ldb + k] (the strided "transposed view" operands of the initial CuTe
 *     kernel, Fig. simple_cute, and the layout section of the coding guide);
 *   - everything after the product is the consumer chain that the Level-2
 *     optimisation prompt asks to fold into the producer's writeback
 *     ("Fusion": bias / add / scale / activation, and "clamp" in its list of
 *     consumer operations): computed on the producer value, stored once.  The
 *     ORDER (scale -> row scale -> bias -> residual -> activation -> clamp ->
 *     output rounding), the per-row / per-column broadcast axes and the meaning
 *     of beta are readings of this repository; the paper names the operations
 *     only.  row_scale on the product alone is what makes diag(d) * (A*B) a
 *     special case (the paper's diagonal-matrix multiply);
 *   - precision is never lowered inside (Experiments, "Manual Correctness
 *     Audit"): products, sums and the chain are fp64.  Only the final store may
 *     round: to fp32, or to bf16 by rounding that fp32 value to nearest-even
 *     (the decision is taken from the fp32 value because that is the precision
 *     the kernel holds it in).
 *
 * Loop order m, n, k: one fp64 accumulator per output, k ascending.
 *
 * Pins (tests/test_oracle_fused_pins.py): exact rational brute force on tiny
 * inputs for every combination of transposition flags, agreement with the
 * separately pinned plain oracle when the extras are off, numpy matmul on
 * transposed copies, row scale folded into A by hand, residual and clamp
 * identities, library bfloat16 conversion and hand-made ties for the rounding.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { FUSED_ACT_NONE = 0, FUSED_ACT_RELU = 1, FUSED_ACT_GELU_TANH = 2 };
enum { FUSED_IN_F64 = 0, FUSED_IN_F32 = 1, FUSED_IN_BF16 = 2 };
enum { FUSED_OUT_F64 = 0, FUSED_OUT_F32 = 1, FUSED_OUT_BF16 = 2 };

static double bf16_value(uint16_t bits)
{
    uint32_t w = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

static double element(const void *base, int kind, size_t index)
{
    if (kind == FUSED_IN_F64) return ((const double *)base)[index];
    if (kind == FUSED_IN_F32) return (double)((const float *)base)[index];
    return bf16_value(((const uint16_t *)base)[index]);
}

/* Nearest bf16 (ties to even) of an fp32 value, returned as that value. */
float oracle_round_f32_to_bf16(float x)
{
    uint32_t w;
    memcpy(&w, &x, sizeof w);
    if ((w & 0x7F800000u) == 0x7F800000u) {          /* inf or NaN: keep, quieten a NaN */
        if (w & 0x007FFFFFu) w |= 0x00400000u;
        w &= 0xFFFF0000u;
    } else {
        uint32_t lower = w & 0xFFFFu;                /* the 16 bits that are dropped */
        w &= 0xFFFF0000u;
        if (lower > 0x8000u || (lower == 0x8000u && (w & 0x10000u))) w += 0x10000u;
    }
    float r;
    memcpy(&r, &w, sizeof r);
    return r;
}

static double act_apply(double v, int act)
{
    if (act == FUSED_ACT_RELU) return v > 0.0 ? v : 0.0;
    if (act == FUSED_ACT_GELU_TANH) {
        const double c = 0.7978845608028654; /* sqrt(2/pi) */
        return 0.5 * v * (1.0 + tanh(c * (v + 0.044715 * v * v * v)));
    }
    return v;
}

/*
 * All sizes in elements.  in_kind: type of A and B; r_kind: type of R
 * (FUSED_IN_*), ignored when R is NULL.  row_scale (length M), bias (length N)
 * are fp64 and shared by every batch; either may be NULL.  Batches are packed:
 * A advances by rowsA*lda where rowsA = transA ? K : M, B by rowsB*ldb where
 * rowsB = transB ? N : K, R by M*ldr, C by M*ldc.  lo <= hi; pass -inf / +inf
 * for no clamp.  C receives fp64 values (already rounded when out_kind asks for
 * it).  Returns 0, or -1 on a bad argument.
 */
int oracle_gemm_fused(int M, int N, int K, int batch,
                      const void *A, long lda, int transA,
                      const void *B, long ldb, int transB, int in_kind,
                      double alpha, const double *row_scale, const double *bias,
                      const void *R, long ldr, int r_kind, double beta,
                      int act, double lo, double hi, int out_kind,
                      double *C, long ldc)
{
    if (M < 1 || N < 1 || K < 1 || batch < 1 || !A || !B || !C) return -1;
    if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N) return -1;
    if (R && ldr < N) return -1;
    if (act < FUSED_ACT_NONE || act > FUSED_ACT_GELU_TANH) return -1;
    if (in_kind < FUSED_IN_F64 || in_kind > FUSED_IN_BF16) return -1;
    if (R && (r_kind < FUSED_IN_F64 || r_kind > FUSED_IN_BF16)) return -1;
    if (out_kind < FUSED_OUT_F64 || out_kind > FUSED_OUT_BF16) return -1;
    if (!(lo <= hi)) return -1;

    const size_t batchA = (size_t)(transA ? K : M) * (size_t)lda;
    const size_t batchB = (size_t)(transB ? N : K) * (size_t)ldb;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < batch; ++b) {
        for (int m = 0; m < M; ++m) {
            for (int n = 0; n < N; ++n) {
                double p = 0.0;
                for (int k = 0; k < K; ++k) {
                    size_t ia = b * batchA + (transA ? (size_t)k * lda + m : (size_t)m * lda + k);
                    size_t ib = b * batchB + (transB ? (size_t)n * ldb + k : (size_t)k * ldb + n);
                    p += element(A, in_kind, ia) * element(B, in_kind, ib);
                }
                double v = alpha * p;
                if (row_scale) v = row_scale[m] * v;
                if (bias) v = v + bias[n];
                if (R) v = v + beta * element(R, r_kind, ((size_t)b * M + m) * (size_t)ldr + n);
                double y = act_apply(v, act);
                if (y < lo) y = lo;
                if (y > hi) y = hi;
                if (out_kind == FUSED_OUT_F32) y = (double)(float)y;
                if (out_kind == FUSED_OUT_BF16) y = (double)oracle_round_f32_to_bf16((float)y);
                C[((size_t)b * M + m) * (size_t)ldc + n] = y;
            }
        }
    }
    return 0;
}
