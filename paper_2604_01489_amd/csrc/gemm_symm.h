// Product with a symmetric operand given by one stored triangle, for few output columns (N <= 32):
// the partial products of  S * B,  S the symmetric M x M matrix whose lower (upper) triangle is
// stored in A, with every element of the stored triangle fetched from memory once.
//
// The paper's optimisation prompt ("Rules for GEMM") names the symmetric operand as a structure to
// exploit: its reads can be reduced.  With few columns the product is a stream of A and bound by HBM,
// so halving the bytes read is what pays.  The stored triangle is cut into super-tiles of ST x ST; one
// workgroup owns one super-tile T = A[I-rows, J-columns] and uses every 128 x 128 sub-tile of it twice
// while it sits in LDS:
//     P1[rows of I] += T   * B[rows of J]        (fragments read along the rows of the image)
//     P2[rows of J] += T^T * B[rows of I]        (fragments read across them, by transposing reads)
// For a super-tile on the diagonal both products belong to the same rows, only the sub-tiles of the
// stored triangle are walked, and in the sub-tiles on the diagonal the elements of the other triangle
// (which may hold anything) are cleared in the fragments: P1 keeps the diagonal, P2 does not.
// Row block X of the result is the sum of T_s terms, T_s the number of super-tile rows: term t comes
// from super-tile (max(X, t), min(X, t)) -- its P1 if it is the super-tile's row block, its P2 if it is
// its column block.  Every term is written to the workspace W[t][batch][M][N] by exactly one
// workgroup and the terms are added in the order of t, with the consumer chain, by the second pass of
// split-K (splitk_reduce_fused_kernel): no atomics, bitwise repeatable.  The partial results cost
// 8 N / ST bytes per byte of A (written once, read once): a quarter at N = 16 with ST = 512.
#pragma once
#include "gemm_bf16_fast.h"
#include "symm_layout.h"

namespace ge {

struct SymmParams {
    const void *A;             // bf16 [batch][M][lda]
    const void *B;             // bf16, K x N (ldb >= N) or, transB, N x K (ldb >= M)
    float *W;                  // [terms][batch][M][N] fp32
    int M, N, lda, ldb, transB, upper, batch;
    int tiles;                 // super-tile rows
    int bVec;                  // B can be read in 16-byte pieces along n (N % 8 == 0, aligned, not transposed)
    long long bytesA;          // extent of one batch of A: ((M - 1) lda + M) * 2
};

// keep element e of a fragment register pair iff keepLo / keepHi
__device__ __forceinline__ unsigned symm_mask_pair(unsigned w, bool keepLo, bool keepHi)
{
    return w & ((keepLo ? 0x0000FFFFu : 0u) | (keepHi ? 0xFFFF0000u : 0u));
}

// ST: side of a super-tile (a multiple of 128: 256, 512 or 768); NP: columns of the small operand's image (16 or 32);
// UPPER: the upper triangle is the stored one.
template <int ST, int NP, bool UPPER>
__global__ void __launch_bounds__(256)
gemm_symm_bf16_kernel(const SymmParams p)
{
    using namespace ge_symm;
    constexpr int NS = ST / SUB;            // sub-tiles per side of a super-tile
    constexpr int NJ = NP / 16;             // 16-column blocks of the result
    constexpr int SMALL_BYTES = ST * NP * 2;
    // two sub-tiles on their way while one is multiplied, where the LDS has room for three stages (one otherwise)
    constexpr int STAGES = 3 * STAGE_BYTES + 2 * SMALL_BYTES <= 152 * 1024 ? 3 : 2, AHEAD = STAGES - 1;
    __shared__ __attribute__((aligned(1024))) char smem[STAGES * STAGE_BYTES + 2 * SMALL_BYTES];
    const unsigned ldsBase = (unsigned)(size_t)(GE_LDS char *)smem;
    const unsigned smallJ = ldsBase + STAGES * STAGE_BYTES;

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.y;

    // super-tile (a, c), a >= c, of linear index blockIdx.x = a (a + 1) / 2 + c
    unsigned a = (unsigned)((__builtin_sqrtf(8.0f * (float)blockIdx.x + 1.0f) - 1.0f) * 0.5f);
    while (a * (a + 1) / 2 > blockIdx.x) --a;
    while ((a + 1) * (a + 2) / 2 <= blockIdx.x) ++a;
    const unsigned c = blockIdx.x - a * (a + 1) / 2;
    const int I = __builtin_amdgcn_readfirstlane(UPPER ? (int)c : (int)a);     // super-tile row
    const int J = __builtin_amdgcn_readfirstlane(UPPER ? (int)a : (int)c);     // super-tile column
    const bool diag = I == J;
    const unsigned smallI = diag ? smallJ : smallJ + SMALL_BYTES;

    const char *gA = (const char *)p.A + (long long)b * p.M * p.lda * 2;
    const uint16_t *gB = (const uint16_t *)p.B + (long long)b * (p.transB ? (long long)p.N * p.ldb : (long long)p.M * p.ldb);

    // ---- the blocks of the small operand: its rows (k) k0 .. k0 + ST - 1, zero beyond M and beyond N --------
    auto stage_small = [&](unsigned dst, int k0) __attribute__((always_inline)) {
        if (p.bVec) {
            for (int q = threadIdx.x; q < ST * (NP / 8); q += 256) {
                const int kk = q / (NP / 8), n = (q % (NP / 8)) * 8;
                i32x4_t v = {0, 0, 0, 0};
                if (k0 + kk < p.M && n < p.N) v = *(const i32x4_t *)(gB + (long long)(k0 + kk) * p.ldb + n);
                *(GE_LDS i32x4_t *)(size_t)(dst + (unsigned)small_offset(NP, kk, n)) = v;
            }
        } else {
            for (int q = threadIdx.x; q < ST * NP; q += 256) {
                const int kk = q / NP, n = q % NP;
                unsigned short v = 0;
                if (k0 + kk < p.M && n < p.N)
                    v = p.transB ? gB[(long long)n * p.ldb + (k0 + kk)] : gB[(long long)(k0 + kk) * p.ldb + n];
                *(GE_LDS unsigned short *)(size_t)(dst + (unsigned)small_offset(NP, kk, n)) = v;
            }
        }
    };

    // ---- loads of sub-tile (rs, cs) of the super-tile into stage st: 8 per wave ---------------------------
    auto issue_sub = [&](int rs, int cs, int st) __attribute__((always_inline)) {
        const int r0 = I * ST + rs * SUB, c0 = J * ST + cs * SUB;
        const long long origin = ((long long)r0 * p.lda + c0) * 2;
        // a sub-tile wholly outside the matrix (a ragged last super-tile) goes through an empty resource
        const bool live = r0 < p.M && c0 < p.M;
        const rsrc_words_t res = make_rsrc(gA + (live ? origin : 0), live ? records_left(p.bytesA, origin) : 0u);
#pragma unroll
        for (int q = 0; q < SLABS / 4; ++q) {
            const int slab = q * 4 + w;
            const int row = slab_row(slab, lane), ch = slab_chunk(slab, lane);
            unsigned v = (unsigned)row * (unsigned)p.lda * 2u + (unsigned)ch * 16u;
            if (r0 + row >= p.M || c0 + ch * 8 >= p.M) v = OOB_OFFSET;
            lds_dma16(res, ldsBase + (unsigned)(st * STAGE_BYTES + slab * 1024), v);
        }
    };

    f32x4_t acc1[NS][2][NJ], acc2[NS][2][NJ];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) { acc1[s][i][j][r] = 0.0f; acc2[s][i][j][r] = 0.0f; }

    // fragment of a small-operand image: the 32 k from kBase, column block j
    auto small_frag = [&](unsigned img, int kBase, int j) __attribute__((always_inline)) {
        const GE_LDS char *p0 = (const GE_LDS char *)(size_t)(img + (unsigned)small_frag_offset(NP, kBase, j, lane, 0));
        const GE_LDS char *p1 = (const GE_LDS char *)(size_t)(img + (unsigned)small_frag_offset(NP, kBase, j, lane, 1));
        short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)p0);
        short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)p1);
        return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    // (Every lambda below is forced inline: called from dozens of unrolled places the large ones would
    // otherwise stay functions, and the accumulator arrays they index would live in scratch memory.)
    // Sub-tile (rs, cs) from stage st: P1 into acc1[rs], P2 into acc2[cs].  onDiag: the sub-tile lies on the
    // diagonal of the matrix and the fragments are cleared of the other triangle.  (Called from fully
    // unrolled loops: rs, cs and onDiag are constants by then.)
    auto multiply = [&](int rs, int cs, bool onDiag, int st) __attribute__((always_inline)) {
        const unsigned img = ldsBase + (unsigned)(st * STAGE_BYTES);
#pragma unroll
        for (int ks = 0; ks < SUB / 32; ++ks) {
            // ---- P1: rows 32 w + 16 i + l%16 of the sub-tile, k = its columns 32 ks + 8 (l/16) + e
            bf16x8_t fbJ[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j) fbJ[j] = small_frag(smallJ, cs * SUB + 32 * ks, j);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int rowBase = 32 * w + 16 * i;
                i32x4_t raw = *(const GE_LDS i32x4_t *)(size_t)(img + (unsigned)row_frag_offset(rowBase, ks, lane));
                if (onDiag) {
                    const int r = rowBase + (lane & 15), col = 32 * ks + 8 * (lane >> 4);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int c0 = col + 2 * q, c1 = c0 + 1;
                        raw[q] = (int)symm_mask_pair((unsigned)raw[q], UPPER ? c0 >= r : c0 <= r, UPPER ? c1 >= r : c1 <= r);
                    }
                }
                const bf16x8_t fa = __builtin_bit_cast(bf16x8_t, raw);
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc1[rs][i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fbJ[j], acc1[rs][i][j], 0, 0, 0);
            }
            // ---- P2: output rows = columns 32 w + 16 i + l%16 of the sub-tile, k = its rows 32 ks + 8 (l/16) + e
            bf16x8_t fbI[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j) fbI[j] = small_frag(smallI, rs * SUB + 32 * ks, j);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int colBase = 32 * w + 16 * i;
                const GE_LDS char *p0 = (const GE_LDS char *)(size_t)(img + (unsigned)col_frag_offset(colBase, ks, lane, 0));
                const GE_LDS char *p1 = (const GE_LDS char *)(size_t)(img + (unsigned)col_frag_offset(colBase, ks, lane, 1));
                short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)p0);
                short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)p1);
                i32x4_t raw = __builtin_bit_cast(i32x4_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                if (onDiag) {
                    // the mirrored part only: the diagonal itself belongs to P1
                    const int cc = colBase + (lane & 15), row = 32 * ks + 8 * (lane >> 4);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int r0 = row + 2 * q, r1 = r0 + 1;
                        raw[q] = (int)symm_mask_pair((unsigned)raw[q], UPPER ? cc > r0 : cc < r0, UPPER ? cc > r1 : cc < r1);
                    }
                }
                const bf16x8_t fa = __builtin_bit_cast(bf16x8_t, raw);
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc2[cs][i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fbI[j], acc2[cs][i][j], 0, 0, 0);
            }
        }
    };

    // ---- the walk over the sub-tiles, two loading while one is multiplied --------------------------------
    // Off the diagonal every sub-tile of the super-tile, (u, v) = (row, column).  On it only those of the
    // stored triangle: v <= u with (row, column) = (u, v) for the lower, (v, u) for the upper triangle.
    // Both loops are fully unrolled, so the accumulators are indexed by constants.  Per sub-tile t: its data
    // have landed (the loads complete in order: all but those of t + 1) and every wave is past the multiply
    // of t - 1 -- one barrier for both -- then the loads of t + AHEAD go into the stage t - 1 occupied.
    auto walk = [&](auto diagC) __attribute__((always_inline)) {
        constexpr bool DIAG = decltype(diagC)::value;
        auto row_of = [](int u, int v) { return (DIAG && UPPER) ? v : u; };
        auto col_of = [](int u, int v) { return (DIAG && UPPER) ? u : v; };
        // (u, v) one step on; u == NS: past the end
        auto step_u = [](int u, int v) { return (DIAG ? v == u : v == NS - 1) ? u + 1 : u; };
        auto step_v = [](int u, int v) { return (DIAG ? v == u : v == NS - 1) ? 0 : v + 1; };
        issue_sub(0, 0, 0);
        if (AHEAD == 2 && step_u(0, 0) < NS) issue_sub(row_of(step_u(0, 0), step_v(0, 0)), col_of(step_u(0, 0), step_v(0, 0)), 1);
        stage_small(smallJ, J * ST);
        if (!DIAG) stage_small(smallI, I * ST);
        int t = 0;
#pragma unroll
        for (int u = 0; u < NS; ++u) {
#pragma unroll
            for (int v = 0; v < NS; ++v) {
                if (DIAG && v > u) continue;
                const int u1 = step_u(u, v), v1 = step_v(u, v);
                const int u2 = u1 < NS ? step_u(u1, v1) : NS, v2 = u1 < NS ? step_v(u1, v1) : 0;
                if (AHEAD == 2 && u1 < NS) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(SLABS / 4) : "memory");
                else                       asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
                if (AHEAD == 2) {
                    if (u2 < NS) issue_sub(row_of(u2, v2), col_of(u2, v2), (t + 2) % STAGES);
                } else if (u1 < NS) {
                    issue_sub(row_of(u1, v1), col_of(u1, v1), (t + 1) % STAGES);
                }
                multiply(row_of(u, v), col_of(u, v), DIAG && u == v, t % STAGES);
                ++t;
            }
        }
    };

    if (diag) walk(std::true_type{});
    else walk(std::false_type{});

    // ---- the terms: P1 is term J of row block I, P2 term I of row block J; on the diagonal their sum is
    // term I of row block I.  Register r of lane l: row 4 (l/16) + r, column l%16 of its 16 x 16 block.
    const long long slice = (long long)p.batch * p.M * p.N;
    auto store_term = [&](f32x4_t (&acc)[NS][2][NJ], int rowBlock, int term) __attribute__((always_inline)) {
        float *dst = p.W + (long long)term * slice + (long long)b * p.M * p.N;
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int m = rowBlock * ST + s * SUB + 32 * w + 16 * i + 4 * (lane >> 4) + r, n = 16 * j + (lane & 15);
                        if (m < p.M && n < p.N) dst[(long long)m * p.N + n] = acc[s][i][j][r];
                    }
    };
    if (diag) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc1[s][i][j][r] += acc2[s][i][j][r];
        store_term(acc1, I, I);
    } else {
        store_term(acc1, I, J);
        store_term(acc2, J, I);
    }
}

}  // namespace ge
