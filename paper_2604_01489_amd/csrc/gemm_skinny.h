// Tall-skinny bf16 GEMM with the fused epilogue: many rows, at most 32 output columns, any K.
//
// With so few columns the product is a stream of A, bound by HBM, and the optimisation prompt's rule
// for skinny shapes applies: tile over the large dimension, keep the small one whole inside the
// block.  A 128-wide tile wastes three quarters of its matrix instructions on padding here and needs
// K slices (a second launch) to make enough blocks.  This kernel: a workgroup owns 32 rows and every
// column, walks K in stages of 128 through a ring of four (three stages on their way while one is
// multiplied; 12 or 16 KB a stage, so that two or three workgroups share a CU and cover each other's
// start and end: with stages of 256 and one workgroup to a CU the kernel was slower than the 128 x 128
// tiles it replaces), A in 256-byte row pieces by direct-to-LDS loads carrying the non-temporal hint
// (A is read once), the matching rows of B from L2 the same way.  Four waves: two row blocks of 16 x
// two halves of a stage's k; the halves are added through LDS in a fixed order at the end, then
// scale, bias and activation, and C is written once.  M / 32 workgroups are enough for a tall matrix;
// for a long K with fewer rows the plan may still slice K (partial tiles for the common second pass).
#pragma once
#include "gemm_bf16_fast.h"
#include "skinny_layout.h"

namespace ge {

// as lds_dma16, with the non-temporal hint: the operand is streamed once
__device__ inline void lds_dma16_nt(rsrc_words_t rs, unsigned ldsAddr, unsigned voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen nt lds"
                 :: "s"(ldsAddr), "v"(voff), "s"(rs) : "memory", "m0");
}

// NP: columns of the B image (16 or 32); RAW: fp32 partial sums of one K slice instead of the epilogue;
// STAGES: depth of the ring, 4 or 8.  Four stages leave room for two or three workgroups on a CU, which is
// what a launch of many short workgroups wants; a launch with one long-lived workgroup to a CU needs the
// bytes in flight from its own ring: eight stages, seven on their way.
template <int NP, bool RAW, int STAGES>
__global__ void __launch_bounds__(256)
gemm_skinny_bf16_kernel(const GemmParams p)
{
    using namespace ge_skinny;
    constexpr int NJ = NP / 16, B_BYTES = KS * NP * 2, B_SLABS = B_BYTES / 1024, STAGE = A_BYTES + B_BYTES;
    constexpr int LOADS = A_SLABS / 4 + B_SLABS / 4;       // loads per wave and stage
    static_assert((STAGES == 4 || STAGES == 8) && (STAGES - 2) * LOADS <= 63, "ring depth; range of the load counter");
    static_assert(A_SLABS % 4 == 0 && B_SLABS % 4 == 0, "the loads divide over the four waves");
    __shared__ __attribute__((aligned(1024))) char smem[STAGES * STAGE];
    const unsigned ldsBase = (unsigned)(size_t)(GE_LDS char *)smem;

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rg = w & 1, kh = w >> 1;                   // row block of 16, half of the stage's k
    const int tilesM = (p.M + BM - 1) / BM;
    const int tm = blockIdx.x % tilesM, s = blockIdx.x / tilesM, b = blockIdx.y;
    const int m0 = tm * BM;
    const int kBegin = s * p.kPerSlice, kEnd = min(p.K, kBegin + p.kPerSlice);
    const int steps = (kEnd - kBegin + KS - 1) / KS;

    const long long offA = 2 * ((long long)b * p.strideA + (long long)m0 * p.lda + kBegin);
    const long long offB = 2 * ((long long)b * p.strideB + (long long)kBegin * p.ldb);
    const char *gA = (const char *)p.A + offA;
    const char *gB = (const char *)p.B + offB;

    // per-lane offsets within a stage's piece of A and of B (inverse of the images' layouts)
    unsigned voffA[A_SLABS / 4], voffB[B_SLABS / 4];
    int kA[A_SLABS / 4], kB[B_SLABS / 4];            // first k of the lane's chunk within the stage
#pragma unroll
    for (int q = 0; q < A_SLABS / 4; ++q) {
        const int slab = q * 4 + w, row = a_slab_row(slab, lane), ch = a_slab_chunk(slab, lane);
        voffA[q] = (unsigned)row * (unsigned)p.lda * 2u + (unsigned)ch * 16u;
        if (m0 + row >= p.M) voffA[q] = OOB_OFFSET;
        kA[q] = ch * 8;
    }
#pragma unroll
    for (int q = 0; q < B_SLABS / 4; ++q) {
        const int slab = q * 4 + w, k = b_slab_k(NP, slab, lane), ch = b_slab_chunk(NP, lane);
        voffB[q] = (unsigned)k * (unsigned)p.ldb * 2u + (unsigned)ch * 16u;
        if (ch * 8 >= p.N) voffB[q] = OOB_OFFSET;
        kB[q] = k;
    }

    // Every workgroup starts its walk over K at another stage and wraps around.  The rows of A are a power
    // of two apart in memory more often than not, so workgroups walking K in step would ask the same few
    // memory channels for everything at once (measured at 8192 x 32 x 8192, rows 16 KB apart: 36 us in step,
    // against 31 us for the sliced 128 x 128 plan whose slices are at different k by construction).  The order
    // of a workgroup's additions depends on its index only: results stay repeatable bit for bit.
    const int rot = steps > 1 ? (int)((blockIdx.x * 5u + blockIdx.y) % (unsigned)steps) : 0;
    // the t-th stage of this workgroup's walk (k from kBegin + KS ((t + rot) mod steps)) into ring slot
    // t % STAGES; past the end of the walk through an empty resource
    auto issue = [&](int t0) __attribute__((always_inline)) {
        const bool live = t0 < steps;
        const int t = live ? (t0 + rot >= steps ? t0 + rot - steps : t0 + rot) : 0;
        const long long stepA = (long long)t * (KS * 2), stepB = (long long)t * KS * p.ldb * 2;
        const rsrc_words_t rA = make_rsrc(gA + (live ? stepA : 0), live ? records_left(p.bytesA, offA + stepA) : 0u);
        const rsrc_words_t rB = make_rsrc(gB + (live ? stepB : 0), live ? records_left(p.bytesB, offB + stepB) : 0u);
        const int kLeft = kEnd - kBegin - t * KS;        // valid k in this stage
        const unsigned dst = ldsBase + (unsigned)((t0 & (STAGES - 1)) * STAGE);
#pragma unroll
        for (int q = 0; q < A_SLABS / 4; ++q) {
            unsigned v = voffA[q];
            if (kA[q] >= kLeft) v = OOB_OFFSET;
            lds_dma16_nt(rA, dst + (unsigned)((q * 4 + w) * 1024), v);
        }
#pragma unroll
        for (int q = 0; q < B_SLABS / 4; ++q) {
            unsigned v = voffB[q];
            if (kB[q] >= kLeft) v = OOB_OFFSET;
            lds_dma16(rB, dst + (unsigned)(A_BYTES + (q * 4 + w) * 1024), v);
        }
    };

    f32x4_t acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[j][r] = 0.0f;

#pragma unroll
    for (int t = 0; t < STAGES - 1; ++t) issue(t);
    for (int t = 0; t < steps; ++t) {
        // stage t has landed (the loads complete in order: all but those of the STAGES - 2 stages after it) and
        // every wave is past the multiply of t - 1, whose ring slot the loads of t + STAGES - 1 now refill
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((STAGES - 2) * LOADS) : "memory");
        issue(t + STAGES - 1);
        const unsigned img = ldsBase + (unsigned)((t & (STAGES - 1)) * STAGE);
#pragma unroll
        for (int ks = 0; ks < KS / 64; ++ks) {       // this wave's half of the stage, 32 k at a time
            const int kk = kh * (KS / 2) + 32 * ks;
            const bf16x8_t fa = *(const GE_LDS bf16x8_t *)(size_t)(img + (unsigned)ge_skinny::a_frag_offset(16 * rg, kk, lane));
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const GE_LDS char *p0 = (const GE_LDS char *)(size_t)(img + (unsigned)(A_BYTES + ge_skinny::b_frag_offset(NP, kk, j, lane, 0)));
                const GE_LDS char *p1 = (const GE_LDS char *)(size_t)(img + (unsigned)(A_BYTES + ge_skinny::b_frag_offset(NP, kk, j, lane, 1)));
                short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)p0);
                short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)p1);
                const bf16x8_t fb = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, acc[j], 0, 0, 0);
            }
        }
    }
    // the empty loads of the stages past the end have retired; every wave is done with the ring
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // the two halves of k: the waves of the second half park their sums, those of the first add them (first
    // half + second half, always in this order) and finish the tile
    GE_LDS f32x4_t *park = (GE_LDS f32x4_t *)(GE_LDS char *)smem;
    if (kh == 1) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) park[(rg * NJ + j) * 64 + lane] = acc[j];
    }
    __syncthreads();
    if (kh == 1) return;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const f32x4_t other = park[(rg * NJ + j) * 64 + lane];
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[j][r] += other[r];
    }
    // register r of lane l: row 4 (l/16) + r, column l%16 of its 16 x 16 block
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int n = 16 * j + (lane & 15);
        if (n >= p.N) continue;
        const float bv = (!RAW && p.bias != nullptr) ? p.bias[n] : 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = m0 + 16 * rg + 4 * (lane >> 4) + r;
            if (m >= p.M) continue;
            if (RAW) p.C[(long long)s * p.sliceStride + (long long)b * p.M * p.N + (long long)m * p.N + n] = acc[j][r];
            else p.C[(long long)b * p.strideC + (long long)m * p.ldc + n] = epilogue_value_rt(acc[j][r], p.alpha, bv, p.act);
        }
    }
}

}  // namespace ge
