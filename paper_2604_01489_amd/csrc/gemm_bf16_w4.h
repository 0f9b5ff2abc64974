// bf16 x bf16 -> fp32 GEMM kernel for full 256 x 256 tiles over a long K range on gfx950: four
// waves, one per SIMD, each owning a 128 x 128 quarter of the tile.
//
// Same ingredients as the eight-wave kernel in gemm_bf16_fast.h (direct-to-LDS loads, XOR-swizzled
// stages, v_mfma_f32_16x16x32_bf16, the fused epilogues), arranged for what the counters and the
// shader clock show at 8192^3: the chip runs into its power limit, so a cycle in which the matrix
// pipes wait costs little (the clock rises) while every byte moved and every instruction issued
// costs time.  Hence
//   * 128 x 128 per wave: a step of 32 k reads 16 KB of fragments per wave, 64 KB per tile, where
//     eight waves of 128 x 64 read 96 KB;
//   * an operand whose memory rows run along k is staged 64 k at a time in rows of 128 bytes (two
//     "pair" stages), so that every request to the L2 is a whole line (half lines with 32-k
//     stages); an operand whose rows run along m or n keeps four stages of 32 k rows, which are
//     whole lines anyway;
//   * the fragments of step t+1 are read into a second register set while the MFMAs of step t
//     issue.  A stage is then free one step earlier than its data is multiplied, which gives the
//     loads the slack that the two-stage ring of 64 k lacks with eight waves: a 32-k stage is
//     refilled four steps ahead, a pair stage (steps 2P, 2P+1) is refilled from step 2P+1 on with
//     the pair of steps 2P+4, 2P+5, needed when step 2P+3 reads its fragments;
//   * the loads and the fragment reads of a step are spread between its 64 MFMAs, one every few
//     MFMAs (measured: the same loads issued back to back at the head of the step cost 9 %);
//   * the accumulators (256 registers per lane) live in the accumulation registers, which the
//     compiler does not do by itself for this many: the MFMAs are written as inline assembly.
// Plain variant: full tiles, every block's K range a multiple of 128 (the loop body is four steps of
// 32).  EDGE: tiles may hang over M or N -- the rows and column chunks beyond are never fetched (their
// lanes carry the out-of-range offset from the start, which costs the loop nothing) and never
// stored.  EDGEK: the K range may be any multiple of 8 -- chunks at or beyond its end are masked load
// by load (two vector instructions each), steps beyond it load nothing, which leaves zeros in their
// stages, and the loop runs on to the next multiple of four steps over those zeros.
#pragma once
#include <type_traits>

#include "gemm_bf16_fast.h"

namespace ge {

// s_waitcnt vmcnt(N) lgkmcnt(0) as an instruction the compiler sees.  As inline assembly the wait is opaque
// to the compiler's bookkeeping of LDS reads: it goes on believing that the fragment reads of the step
// before are still on their way and guards the first MFMAs of every step with waits of its own ("at most
// 3, 2, 1 LDS operations outstanding").  Those are satisfied when they are reached, so this buys
// instructions, not time (34 -> 4 waits per four steps; 8192^3 measured the same).
template <int N>
__device__ __forceinline__ void w4_wait_loads_and_lds()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    // vmcnt[3:0] | expcnt[6:4] = 7 (none) | lgkmcnt[11:8] = 0 | vmcnt[5:4] at [15:14]
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (0 << 8) | ((N >> 4) << 14));
}

struct W4Tile {
    static constexpr int BM = 256, BN = 256, BK = 32, NW = 4, WTM = 128, WTN = 128, TM = 8, TN = 8;
    static constexpr int STAGE_BYTES = 256 * BK * 2;        // one operand, 32 k: 16 KB
    static constexpr int OPERAND_BYTES = 4 * STAGE_BYTES;   // four stages of 32 k or two of 64 k
    static constexpr int LDS_BYTES = 2 * OPERAND_BYTES;     // 128 KB
};

// EDGEMODE: 0 none, 1 tiles may hang over M or N (EDGE above), 2 also any K range (EDGEK above; the
// masks of the K edge are vector instructions among the MFMAs of the one wave a SIMD has, about 10 %
// of the run at 8192^3, so shapes that only need the first do not pay for the second).
// RAW / ACT / FUSED / OUTBF16 / TA / TB as in gemm_bf16_kernel.
template <int EDGEMODE, bool RAW, int ACT, bool TA, bool TB, bool FUSED, bool OUTBF16>
__global__ void __launch_bounds__(256)
gemm_bf16_w4_kernel(const GemmParams p)
{
    using T = W4Tile;
    constexpr bool EDGE = EDGEMODE >= 1, EDGEK = EDGEMODE == 2;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NW = T::NW, TM = T::TM, TN = T::TN;
    constexpr bool APAIR = !TA, BPAIR = TB;                 // operand staged 64 k at a time
    constexpr int NLA = APAIR ? 8 : 4, NLB = BPAIR ? 8 : 4; // loads per wave and stage
    // loads of an odd step (pair stages first, they are needed sooner), of an even step
    constexpr int PAIR_LOADS = (APAIR ? 8 : 0) + (BPAIR ? 8 : 0), RING_LOADS = (APAIR ? 0 : 4) + (BPAIR ? 0 : 4);
    constexpr int ODD_LOADS = PAIR_LOADS + RING_LOADS, EVEN_LOADS = RING_LOADS;
    constexpr int ODD_STRIDE = ODD_LOADS > 8 ? 4 : 8, EVEN_STRIDE = EVEN_LOADS > 4 ? 8 : 16;
    static_assert(!(RAW && FUSED) && (FUSED || !OUTBF16), "partial tiles carry no epilogue; bf16 output is the fused one's");
    static_assert(ODD_LOADS * ODD_STRIDE <= 64 && EVEN_LOADS * EVEN_STRIDE <= 64, "a step has 64 slots");

    __shared__ __attribute__((aligned(1024))) char smem[T::LDS_BYTES];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = w / 2, wn = w % 2;

    const TileCoord tc = map_block(p);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;
    int kBegin = tc.s * p.kPerSlice;
    int kEnd = min(p.K, kBegin + p.kPerSlice);
    if constexpr (FUSED) triangular_k_range(p, m0, BM, kBegin, kEnd);
    const int kLen = kEnd - kBegin;
    const int nk = (kLen + BK - 1) / BK;                    // a multiple of 4 unless EDGEK (the host checks)

    const long long offA = 2 * ((long long)tc.b * p.strideA +
                                (TA ? (long long)kBegin * p.lda + m0 : (long long)m0 * p.lda + kBegin));
    const long long offB = 2 * ((long long)tc.b * p.strideB +
                                (TB ? (long long)n0 * p.ldb + kBegin : (long long)kBegin * p.ldb + n0));
    const char *gA = (const char *)p.A + offA;
    const char *gB = (const char *)p.B + offB;

    // per-lane offsets of the 16-byte chunks this lane fetches (inverse of the LDS layouts)
    unsigned voffA[NLA], voffB[NLB];
    int kA[EDGEK ? NLA : 1], kB[EDGEK ? NLB : 1];   // first k of the chunk within its stage, for the K-edge mask
#pragma unroll
    for (int j = 0; j < NLA; ++j) {
        if (APAIR) {
            const int row = a64_slot_row(j * NW + w, lane), c = a64_slot_chunk(j * NW + w, lane);
            voffA[j] = (unsigned)row * (unsigned)p.lda * 2u + (unsigned)c * 16u;
            if (EDGE && m0 + row >= p.M) voffA[j] = OOB_OFFSET;
            if (EDGEK) kA[j] = c * 8;
        } else {
            const int k = b_slot_k<BM>(j * NW + w, lane), c = b_slot_chunk<BM>(j * NW + w, lane);
            voffA[j] = (unsigned)k * (unsigned)p.lda * 2u + (unsigned)c * 16u;
            if (EDGE && m0 + c * 8 >= p.M) voffA[j] = OOB_OFFSET;
            if (EDGEK) kA[j] = k;
        }
    }
#pragma unroll
    for (int j = 0; j < NLB; ++j) {
        if (BPAIR) {
            const int row = a64_slot_row(j * NW + w, lane), c = a64_slot_chunk(j * NW + w, lane);
            voffB[j] = (unsigned)row * (unsigned)p.ldb * 2u + (unsigned)c * 16u;
            if (EDGE && n0 + row >= p.N) voffB[j] = OOB_OFFSET;
            if (EDGEK) kB[j] = c * 8;
        } else {
            const int k = b_slot_k<BN>(j * NW + w, lane), c = b_slot_chunk<BN>(j * NW + w, lane);
            voffB[j] = (unsigned)k * (unsigned)p.ldb * 2u + (unsigned)c * 16u;
            if (EDGE && n0 + c * 8 >= p.N) voffB[j] = OOB_OFFSET;
            if (EDGEK) kB[j] = k;
        }
    }

    const unsigned ldsA = (unsigned)(size_t)(GE_LDS char *)smem, ldsB = ldsA + T::OPERAND_BYTES;

    // Resource words of the tile being loaded: the pair of steps kt, kt+1 (kt even) for a pair
    // stage, step kt for a ring stage; zero length past the K range (nothing is read).
    rsrc_words_t rA, rB;
    int kLeftPair = 0, kLeftRing = 0;               // valid k from the first k of the stage being loaded (EDGEK only)
    auto set_rsrc_pair = [&](int kt) {
        const unsigned rec = kt < nk ? RSRC_RECORDS : 0u;
        kLeftPair = kLen - kt * BK;
        if (APAIR) rA = make_rsrc(gA + (long long)kt * (BK * 2), rec);
        if (BPAIR) rB = make_rsrc(gB + (long long)kt * (BK * 2), rec);
    };
    auto set_rsrc_ring = [&](int kt) {
        const unsigned rec = kt < nk ? RSRC_RECORDS : 0u;
        kLeftRing = kLen - kt * BK;
        if (!APAIR) rA = make_rsrc(gA + (long long)kt * BK * p.lda * 2, rec);
        if (!BPAIR) rB = make_rsrc(gB + (long long)kt * BK * p.ldb * 2, rec);
    };
    // load d of the pair loads (A's first) into pair stage pst; load d of the ring loads into ring stage st
    auto dma_pair = [&](int d, int pst) {
        if (APAIR && d < 8) {
            unsigned v = voffA[d & (NLA - 1)];
            if (EDGEK && kA[EDGEK ? (d & (NLA - 1)) : 0] >= kLeftPair) v = OOB_OFFSET;
            lds_dma16(rA, ldsA + (unsigned)(pst * 2 * T::STAGE_BYTES + (d * NW + w) * 1024), v);
        } else {
            const int l = APAIR ? d - 8 : d;
            unsigned v = voffB[l & (NLB - 1)];
            if (EDGEK && kB[EDGEK ? (l & (NLB - 1)) : 0] >= kLeftPair) v = OOB_OFFSET;
            lds_dma16(rB, ldsB + (unsigned)(pst * 2 * T::STAGE_BYTES + (l * NW + w) * 1024), v);
        }
    };
    auto dma_ring = [&](int d, int st) {
        if (!APAIR && d < 4) {
            unsigned v = voffA[d & (NLA - 1)];
            if (EDGEK && kA[EDGEK ? (d & (NLA - 1)) : 0] >= kLeftRing) v = OOB_OFFSET;
            lds_dma16(rA, ldsA + (unsigned)(st * T::STAGE_BYTES + (d * NW + w) * 1024), v);
        } else {
            const int l = !APAIR ? d - 4 : d;
            unsigned v = voffB[l & (NLB - 1)];
            if (EDGEK && kB[EDGEK ? (l & (NLB - 1)) : 0] >= kLeftRing) v = OOB_OFFSET;
            lds_dma16(rB, ldsB + (unsigned)(st * T::STAGE_BYTES + (l * NW + w) * 1024), v);
        }
    };

    // Lane bases of the fragment reads, opaque to the compiler so that each read is "base +
    // immediate": a pair stage needs one per k half (the half is part of the XOR), a ring stage
    // one per 16-wide block (its stepping is an XOR).
    constexpr int NA = APAIR ? 2 : TM, NB = BPAIR ? 2 : TN;
    unsigned aAddr[NA], bAddr[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        aAddr[i] = ldsA + (APAIR ? (unsigned)a64_frag_offset(wm * T::WTM, lane, i)
                                 : ((unsigned)b_frag_offset<BM>(wm * T::WTM, lane, 0) ^ (unsigned)(i * 32)));
        asm volatile("" : "+v"(aAddr[i]));
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        bAddr[j] = ldsB + (BPAIR ? (unsigned)a64_frag_offset(wn * T::WTN, lane, j)
                                 : ((unsigned)b_frag_offset<BN>(wn * T::WTN, lane, 0) ^ (unsigned)(j * 32)));
        asm volatile("" : "+v"(bAddr[j]));
    }

    f32x4_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

    bf16x8_t fa[2][TM], fb[2][TN];

    // fragment r (0..7: A's, 8..15: B's) of the step whose data sit in ring stage st (pair stage
    // st / 2, half st % 2), into register set NX
#define GE_W4_READ_STRIDED(dst, base, rowBytes)                                                        \
    do {                                                                                               \
        const GE_LDS char *ptr_ = (const GE_LDS char *)(size_t)(base);                                 \
        short4_t lo_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)ptr_);               \
        short4_t hi_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)(ptr_ + 4 * (rowBytes))); \
        short8_t both_ = __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7);                    \
        dst = __builtin_bit_cast(bf16x8_t, both_);                                                     \
    } while (0)
#define GE_W4_READ(r, st, NX)                                                                          \
    do {                                                                                               \
        const int f_ = (r) & 7, st_ = (st);                                                            \
        if ((r) < 8) {                                                                                 \
            if (APAIR) fa[NX][f_] = *(const GE_LDS bf16x8_t *)(size_t)(aAddr[APAIR ? (st_ & 1) : 0] + (unsigned)((st_ >> 1) * 2 * T::STAGE_BYTES + f_ * 2048)); \
            else GE_W4_READ_STRIDED(fa[NX][f_], aAddr[APAIR ? 0 : f_] + (unsigned)(st_ * T::STAGE_BYTES), BM * 2); \
        } else {                                                                                       \
            if (BPAIR) fb[NX][f_] = *(const GE_LDS bf16x8_t *)(size_t)(bAddr[BPAIR ? (st_ & 1) : 0] + (unsigned)((st_ >> 1) * 2 * T::STAGE_BYTES + f_ * 2048)); \
            else GE_W4_READ_STRIDED(fb[NX][f_], bAddr[BPAIR ? 0 : f_] + (unsigned)(st_ * T::STAGE_BYTES), BN * 2); \
        }                                                                                              \
    } while (0)

    // accumulator register r of lane l is C[m = 16 i + 4*(l/16) + r][n = 16 j + l%16]; with the
    // operands swapped (OUTBF16) the block comes out transposed
#define GE_W4_MFMA(i, j, CU)                                                                           \
    do {                                                                                               \
        if (OUTBF16) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fb[CU][j]), "v"(fa[CU][i])); \
        else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fa[CU][i]), "v"(fb[CU][j])); \
    } while (0)

    // Step t (t % 4 == S): the fragments of step t are in register set CU.  64 MFMAs with, in
    // between, the loads of this step (odd S: the pair stages of steps t+3, t+4 into pair stage
    // S / 2, whose last fragments were read during step t-1; every S: ring stage S, step t+4) and
    // the fragment reads of step t+1 into register set NX.  Then: own part of step t+2's data
    // landed (the loads complete in order, so "all but the N youngest"), own fragment reads done,
    // barrier.  After the barrier the data of step t+2 are visible to all waves and the stages
    // read during this step are free.
#define GE_W4_STEP(S, t, CU, NX)                                                                       \
    {                                                                                                  \
        if (RING_LOADS > 0) set_rsrc_ring((t) + 4);                                                    \
        if (((S) & 1) && PAIR_LOADS > 0) set_rsrc_pair((t) + 3);                                       \
        __builtin_amdgcn_sched_barrier(0);                                                             \
        _Pragma("unroll") for (int q = 0; q < 64; ++q) {                                               \
            GE_W4_MFMA(q >> 3, q & 7, CU);                                                             \
            if ((S) & 1) {                                                                             \
                if (q % ODD_STRIDE == 0 && q / ODD_STRIDE < ODD_LOADS) {                               \
                    const int d = q / ODD_STRIDE;                                                      \
                    if (d < PAIR_LOADS) dma_pair(d, (S) >> 1);                                         \
                    else dma_ring(d - PAIR_LOADS, (S));                                                \
                }                                                                                      \
            } else if (q % EVEN_STRIDE == 0 && q / EVEN_STRIDE < EVEN_LOADS) dma_ring(q / EVEN_STRIDE, (S)); \
            if ((q & 1) && q < 32) GE_W4_READ(q >> 1, ((S) + 1) & 3, NX);                              \
            __builtin_amdgcn_sched_barrier(0);                                                         \
        }                                                                                              \
        w4_wait_loads_and_lds<((S) & 1) ? PAIR_LOADS + 2 * RING_LOADS : 2 * RING_LOADS>();             \
        asm volatile("s_barrier" ::: "memory");                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                             \
    }

    if (nk > 0) {
        // both pair stages, all four ring stages
        if (PAIR_LOADS > 0) {
            set_rsrc_pair(0);
#pragma unroll
            for (int d = 0; d < PAIR_LOADS; ++d) dma_pair(d, 0);
            set_rsrc_pair(2);
#pragma unroll
            for (int d = 0; d < PAIR_LOADS; ++d) dma_pair(d, 1);
        }
        if (RING_LOADS > 0) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                set_rsrc_ring(t);
#pragma unroll
                for (int d = 0; d < RING_LOADS; ++d) dma_ring(d, t);
            }
        }
        // step 0 landed -> its fragments; step 1 landed -> the loop
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(RING_LOADS > 0 ? 3 * RING_LOADS : PAIR_LOADS) : "memory");
#pragma unroll
        for (int r = 0; r < 16; ++r) GE_W4_READ(r, 0, 0);
        w4_wait_loads_and_lds<(RING_LOADS > 0 ? 2 * RING_LOADS : PAIR_LOADS)>();
        asm volatile("s_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        // one back edge, no exit from the middle: with more the register allocator spills the accumulators
        for (int kt = 0; kt < nk; kt += 4) {
            GE_W4_STEP(0, kt, 0, 1);
            GE_W4_STEP(1, kt + 1, 1, 0);
            GE_W4_STEP(2, kt + 2, 0, 1);
            GE_W4_STEP(3, kt + 3, 1, 0);
        }
    }
    // The zero-length loads of the steps past the end must have retired before the LDS is released,
    // and the accumulation registers of the last MFMAs must be readable (the compiler does not see
    // the MFMAs, so it inserts no wait states of its own).
    asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");

#undef GE_W4_STEP
#undef GE_W4_MFMA
#undef GE_W4_READ
#undef GE_W4_READ_STRIDED

    // ---- epilogue in registers ----------------------------------------------------
    // the lane index as a value born here: nothing of the epilogue's address arithmetic or edge
    // tests can be hoisted above the main loop, where it would only be carried along
    int laneE = lane, waveE = (int)(threadIdx.x >> 6);
    asm volatile("" : "+v"(laneE), "+v"(waveE));
    const int rowLane = m0 + (waveE / 2) * T::WTM + 4 * (laneE >> 4);
    const int colLane = n0 + (waveE % 2) * T::WTN + (laneE & 15);
    if constexpr (FUSED) {
        if constexpr (OUTBF16) {
            const bool resInLds = stage_residual_bf16<BM, BN, NW>(p, tc.b, (GE_LDS char *)smem, m0, n0, p.M, waveE, laneE);
            fused_epilogue_bf16_through_lds<BM, BN, NW, T::LDS_BYTES, TM, TN, EDGE, true>(
                p, tc.b, acc, (GE_LDS char *)smem, m0, n0, (waveE / 2) * T::WTM + (laneE & 15),
                (waveE % 2) * T::WTN + 4 * (laneE >> 4), waveE, laneE, resInLds);
        } else {
            // only the tiles that hang over M or N pay for masked stores (a uniform branch; masked, the
            // stores of an 8192^3-sized launch cost 10 % of its run)
            if (!EDGE || (m0 + BM <= p.M && n0 + BN <= p.N)) fused_epilogue_f32_direct<TM, TN, false>(p, tc.b, acc, rowLane, colLane);
            else fused_epilogue_f32_direct<TM, TN, EDGE>(p, tc.b, acc, rowLane, colLane);
        }
    } else {
        float *cBase;
        long long ldc;
        if (RAW) {
            ldc = p.N;
            cBase = p.C + (long long)tc.s * p.sliceStride + (long long)tc.b * p.M * p.N;
        } else {
            ldc = p.ldc;
            cBase = p.C + (long long)tc.b * p.strideC;
        }
        auto store_tile = [&](auto masked) {
            constexpr bool MASK = decltype(masked)::value;
            float bv[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bv[j] = (!RAW && p.bias != nullptr && (!MASK || colLane + j * 16 < p.N)) ? p.bias[colLane + j * 16] : 0.0f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = rowLane + i * 16 + r;
                    float *rowPtr = cBase + (long long)m * ldc + colLane;
                    // the row's values first, stage by stage over the column blocks, then its stores
                    float v[TN];
#pragma unroll
                    for (int j = 0; j < TN; ++j) v[j] = acc[i][j][r];
                    if (!RAW) epilogue_values<ACT, TN>(v, p.alpha, bv);
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        if (!MASK || (m < p.M && colLane + j * 16 < p.N)) rowPtr[j * 16] = v[j];
                }
        };
        if (!EDGE || (m0 + BM <= p.M && n0 + BN <= p.N)) store_tile(std::false_type{});
        else store_tile(std::true_type{});
    }
}

}  // namespace ge
