// bf16 x bf16 -> fp32 GEMM main kernel for gfx950 (MI355X).
//
// The optimisation list for GEMM-like kernels in the paper's optimisation prompt
// (block tiling, wave tiling, matrix instructions, bank-conflict-free staging,
// multi-stage asynchronous loads) and its square-GEMM case study (staging
// buffers per operand, the next K tile prefetched while the current one is
// consumed) are kept as ideas; the realisation is CDNA4's own:
//   * one workgroup owns a BM x BN tile of C and walks K in steps of 32;
//   * WM x WN wavefronts of 64 lanes, each owning a (BM/WM) x (BN/WN) sub-tile as
//     a grid of 16x16 v_mfma_f32_16x16x32_bf16 accumulators (fp32).  Of the bf16
//     shapes this one draws the least power per FLOP, and on this part the clock
//     under load, not the issue rate, is what bounds a dense GEMM;
//   * A and B tiles go global -> LDS with buffer_load_dwordx4 ... lds (16 bytes
//     per lane, no register round trip) into a ring of four stages, three tiles
//     in flight; completion is tracked with explicit s_waitcnt vmcnt(N);
//   * A fragments are ds_read_b128, B fragments ds_read_b64_tr_b16 (B is [K,N]
//     row-major while the matrix unit wants 8 consecutive k per lane);
//   * both LDS layouts are XOR-swizzled so fragment reads spread over all banks
//     (measured: SQ_LDS_BANK_CONFLICT = 0).  A direct-to-LDS load lands at
//     base + 16*lane, so the swizzle is applied by choosing which global chunk
//     each lane fetches;
//   * with 8 waves the two waves of every SIMD run half a step apart: one issues
//     its loads and LDS reads while the other issues back-to-back MFMAs, swapping
//     at each barrier, so the matrix pipe never waits on LDS latency;
//   * scale, bias and activation are applied to the accumulators in registers and C
//     is written once.  A lane holds one column of each 16x16 block, so a store
//     instruction writes 64 contiguous bytes of 4 rows; stores are issued row by
//     row across the wave's column blocks so whole 128-byte lines fill within a
//     few instructions (measured faster than 16-byte-per-lane stores whose
//     neighbouring lanes sit in different rows).
#pragma once
#include <type_traits>

#include "bf16_layout.h"
#include "ge_device.h"

namespace ge {

constexpr int BF16_BK = 32;
constexpr int BF16_STAGES = 4;
constexpr unsigned OOB_OFFSET = 0x80000000u;   // >= num_records: the load returns 0, touches no memory
constexpr unsigned RSRC_RECORDS = 0x80000000u;  // upper bound of num_records (keeps OOB_OFFSET out of range)
constexpr unsigned RSRC_FLAGS = 0x00020000u;   // raw buffer, 32-bit data format

typedef __attribute__((ext_vector_type(4))) int rsrc_words_t;

// 16 bytes per lane from a raw buffer straight into LDS at ldsAddr + 16*lane.
// Written as inline assembly so the compiler does not track it: its own
// bookkeeping of LDS DMA forces vmcnt(0) at loop headers, which would serialise
// the pipeline.  The caller awaits completion with s_waitcnt vmcnt(N).
__device__ inline void lds_dma16(rsrc_words_t rs, unsigned ldsAddr, unsigned voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(ldsAddr), "v"(voff), "s"(rs) : "memory", "m0");
}

// num_records for a resource that starts `consumed` bytes into an allocation of `total` bytes:
// what is left of the allocation, capped at RSRC_RECORDS.  With it an offset that is wrong for
// whatever reason reads zeros instead of faulting.
// Written on 32-bit halves so that it stays on the scalar unit (there is no 64-bit scalar
// compare, and vector instructions in the load phase would take issue slots from the MFMAs of
// the other wave group).  `consumed` never exceeds `total` for the tiles a block loads.
__device__ inline unsigned records_left(long long total, long long consumed)
{
    const unsigned long long left = (unsigned long long)(total - consumed);
    unsigned hi = (unsigned)(left >> 32), lo = (unsigned)left;
    asm volatile("" : "+s"(hi), "+s"(lo));     // keep the halves apart: no 64-bit (vector) compare
    const unsigned capped = lo < RSRC_RECORDS ? lo : RSRC_RECORDS;
    return hi != 0u ? RSRC_RECORDS : capped;
}

__device__ inline rsrc_words_t make_rsrc(const void *base, unsigned records)
{
    const unsigned long long a = (unsigned long long)base;
    rsrc_words_t r;
    r[0] = (int)(unsigned)a;
    r[1] = (int)((unsigned)(a >> 32) & 0xFFFFu);
    r[2] = (int)records;
    r[3] = (int)RSRC_FLAGS;
    return r;
}

// A bf16 residual on its way into the LDS image of a tile's bf16 output (fused_epilogue_bf16_through_lds with
// resInLds): whole rows of the tile by the same 16-byte-per-lane direct-to-LDS loads as the operands, 1 KB
// per wave instruction, all of a wave's loads on their way at once, landing where the image's row and chunk
// swizzle wants them.  Read from memory by the lanes that need it, the residual comes as 8 bytes a lane from
// 16 rows per instruction: the 112 KB of a 224 x 256 tile then take 4.8 us where the stores of the same
// bytes take 2 (the 3 x 3 convolution workload: 0.128 -> 0.124 ms).  Returns whether the residual is of the
// kind this takes (bf16, rows readable in 16-byte pieces, offsets within 31 bits); the caller passes that on.
// Every wave of the block calls this after the last read of the stages; rows at or beyond rowLimit and
// columns at or beyond p.N are not fetched.
template <int BM, int BN, int NW>
__device__ __forceinline__ bool stage_residual_bf16(const GemmParams &p, int b, GE_LDS char *lds, int m0, int n0, int rowLimit, int w, int lane)
{
    constexpr int PITCH = BN * 2, CHUNKS = PITCH / 16, ROWS_PER_INSTR = 1024 / PITCH;
    static_assert((BM / ROWS_PER_INSTR) % NW == 0, "the image's kilobytes divide over the waves");
    // (rVec: R is 16-byte aligned and its rows are multiples of 16 bytes; a batch's first row must be as well)
    const bool take = p.R != nullptr && p.rVec && p.rType == DT_BF16 && (long long)BM * p.ldr * 2 < (1ll << 31) &&
                      (((long long)b * p.strideR) & 7) == 0;
    if (!take) return false;
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // every wave is done with the stages
    const rsrc_words_t rR = make_rsrc((const char *)p.R + ((long long)b * p.strideR + (long long)m0 * p.ldr + n0) * 2, RSRC_RECORDS);
    const unsigned ldsBase = (unsigned)(size_t)lds + (unsigned)__builtin_amdgcn_readfirstlane(w) * 1024u;
#pragma unroll
    for (int it = 0; it < BM / ROWS_PER_INSTR / NW; ++it) {
        const int row = (it * NW + w) * ROWS_PER_INSTR + lane / CHUNKS, chunk = (lane % CHUNKS) ^ (row & (CHUNKS - 1));
        unsigned v = (unsigned)row * (unsigned)p.ldr * 2u + (unsigned)chunk * 16u;
        if (m0 + row >= rowLimit || n0 + chunk * 8 >= p.N) v = OOB_OFFSET;
        lds_dma16(rR, ldsBase + (unsigned)(it * NW * 1024), v);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    return true;
}

template <int BM, int BN, int WM, int WN>
struct Bf16Tile {
    static constexpr int BK = BF16_BK, NS = BF16_STAGES;
    static constexpr int NW = WM * WN;
    static constexpr int THREADS = NW * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int TM = WTM / 16, TN = WTN / 16;
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BK * BN * 2;
    static constexpr int A_LOADS = A_BYTES / 1024 / NW;  // wave-wide 1 KB loads per wave and tile
    static constexpr int B_LOADS = B_BYTES / 1024 / NW;
    static constexpr int LOADS = A_LOADS + B_LOADS;
    static constexpr int LDS_BYTES = NS * (A_BYTES + B_BYTES);
    static constexpr bool PINGPONG = (NW == 8);
    static_assert(NW == 4 || NW == 8, "4 or 8 waves");
    static_assert(WTM % 16 == 0 && WTN % 32 == 0, "wave tile shape");
    static_assert((A_BYTES / 1024) % NW == 0 && (B_BYTES / 1024) % NW == 0, "loads must divide over waves");
    static_assert(BM % 16 == 0 && BN % 32 == 0 && (BN & (BN - 1)) == 0, "block tile shape");
    static_assert(((WTN / 32) & (WTN / 32 - 1)) == 0, "WTN/32 must be a power of two");
    static_assert(2 * LOADS <= 63, "vmcnt range");
};

// EDGE: the tile may hang over M, N or the K range (loads are zero filled through
// the buffer bounds check, stores are masked).  RAW: write fp32 partial sums for
// the split-K reduction (no scale, bias or activation) instead of C.
//
// TA / TB: the operand is stored transposed (A as K x M, B as N x K).  Only the staging differs:
// an operand whose rows run along k uses the "k-contiguous" stage (rows of 64 bytes, fragments
// by ds_read_b128), one whose rows run along m or n the "k-strided" stage (k rows of the tile
// width, fragments by transposing reads); the matrix instruction sees the same fragments.
// FUSED: the run-time epilogue of the widened operator (row scale, residual, clamp) instead of the
// compile-time scale/bias/activation, with fp32 output straight from the accumulators or
// (OUTBF16) bf16 output through LDS, for which the operands of the MFMA are swapped.
// CONV: implicit-GEMM convolution (optimisation prompt, convolution section): the rows of A are
// output positions of a channels-last input and are gathered on the fly -- K step t covers 32
// channels of one filter tap, so the lane's chunk of a row is 16 contiguous bytes at
// position base + tap offset, or zeros where the tap falls into the padding (the out-of-range
// offset of the buffer load).  B is the filter bank stored [Cout][KH*KW*Cin] (TB), C the
// channels-last output.
// K64: the loads move 64 k at a time into a ring of two stages (same LDS as four of 32).  A
// k-contiguous operand is then staged in rows of 128 bytes, so that eight neighbouring lanes of a
// load fetch one whole line of the operand instead of half of it now and the other half a step
// later; a k-strided operand keeps its layout (a 64-k stage is two of its 32-k stages back to back).
// The multiply still advances 32 k per phase.  One tile of 64 is in flight while one is consumed:
// less slack than the three-of-four ring, which the full lines more than repay when both operands
// are k-contiguous (measured: 8192^3 with both operands k-contiguous 0.85 -> 0.81 ms; with one
// or none 0.75 -> 0.81 ms; the 3x3 convolution over 256 channels 0.139 -> 0.147 ms, so it is used
// for the first only).  The K range of a block must be a multiple of 64 unless EDGE.
template <int BM, int BN, int WM, int WN, bool EDGE, bool RAW, int ACT, bool TA = false, bool TB = false,
          bool FUSED = false, bool OUTBF16 = false, bool CONV = false, bool K64 = false>
__global__ void __launch_bounds__(WM * WN * 64)
gemm_bf16_kernel(const GemmParams p)
{
    using T = Bf16Tile<BM, BN, WM, WN>;
    constexpr int BK = T::BK, NW = T::NW, TM = T::TM, TN = T::TN, LOADS = T::LOADS;
    constexpr bool PINGPONG = T::PINGPONG;
    constexpr bool A64 = K64 && !TA, B64 = K64 && TB;     // operands staged in 128-byte rows
    static_assert(!(RAW && FUSED) && (FUSED || !OUTBF16), "partial tiles carry no epilogue; bf16 output is the fused one's");
    static_assert(!CONV || (!TA && TB && (FUSED || RAW) && !K64), "convolution: gathered k-contiguous A, filters as N x K, 32 k per step");
    static_assert((BM & (BM - 1)) == 0 && ((T::WTM / 32) & (T::WTM / 32 - 1)) == 0, "k-strided A stage");

    // One LDS object with a fixed layout: A stages 0..3, then B stages 0..3.  Every fragment read is then "lane base + immediate" (the A stages
    // and, from a second lane base, the B stages each lie within the 64 KB immediate range), so
    // the main loop carries no address arithmetic on the vector unit.
    __shared__ __attribute__((aligned(1024))) char smem[T::LDS_BYTES];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = w / WN, wn = w % WN;

    const TileCoord tc = map_block(p);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;
    int kBegin = tc.s * p.kPerSlice;
    int kEnd = min(p.K, kBegin + p.kPerSlice);
    if constexpr (FUSED && !CONV) triangular_k_range(p, m0, BM, kBegin, kEnd);
    const int kLen = kEnd - kBegin;
    const int nk = (kLen + BK - 1) / BK;

    const long long offA = CONV ? 0ll : 2 * ((long long)tc.b * p.strideA +
                                (TA ? (long long)kBegin * p.lda + m0 : (long long)m0 * p.lda + kBegin));
    const long long offB = 2 * ((long long)tc.b * p.strideB +
                                (TB ? (long long)n0 * p.ldb + kBegin : (long long)kBegin * p.ldb + n0));
    const char *gA = (const char *)p.A + offA;
    const char *gB = (const char *)p.B + offB;

    // ---- per-lane global offsets of the 16-byte chunks this lane fetches (inverse of
    // the LDS layout: slot -> (row, chunk)); kA / kB hold what the K-edge mask compares:
    // the chunk along k (k-contiguous stage) or the k row (k-strided stage) ---------------
    constexpr int NLA = A64 ? 2 * T::A_LOADS : T::A_LOADS, NLB = B64 ? 2 * T::B_LOADS : T::B_LOADS;
    unsigned voffA[NLA], voffB[NLB];
    int kA[NLA], kB[NLB];
    // convolution: input row and column of filter tap (0, 0) for the lane's output position
    // (far out of range for rows past M, so that every tap test fails)
    int ih0[CONV ? NLA : 1], iw0[CONV ? NLA : 1];
#pragma unroll
    for (int j = 0; j < NLA; ++j) {
        if (CONV) {
            const int row = A64 ? a64_slot_row(j * NW + w, lane) : a_slot_row(j * NW + w, lane);
            const int c = A64 ? a64_slot_chunk(j * NW + w, lane) : a_slot_chunk(lane);
            const int m = m0 + row;
            const int pos = m % (p.convOH * p.convOW), img = m / (p.convOH * p.convOW);
            const int oh = pos / p.convOW, ow = pos % p.convOW;
            const int ihTap0 = oh * p.convSh - p.convPh;
            ih0[j] = m < p.M ? ihTap0 : -(1 << 24);
            iw0[j] = ow * p.convSw - p.convPw;
            kA[j] = c * 8;
            // byte offset of (img, ih0, iw0, channel 8c) modulo 2^32: it may be "negative" for a tap
            // in the padding, and adding the tap offset of an inside tap brings it back into
            // [0, 2^31) (the host checks that the input is smaller than that)
            voffA[j] = ((unsigned)((img * p.convH + ihTap0) * p.convW + iw0[j]) * (unsigned)p.convCin + (unsigned)(c * 8)) * 2u;
        } else if (!TA) {
            // 1 KB slab = 16 rows of 64 bytes, or 8 rows of 128
            const int row = A64 ? a64_slot_row(j * NW + w, lane) : a_slot_row(j * NW + w, lane);
            const int c = A64 ? a64_slot_chunk(j * NW + w, lane) : a_slot_chunk(lane);
            kA[j] = c * 8;
            voffA[j] = (unsigned)row * (unsigned)p.lda * 2u + (unsigned)c * 16u;
            if (EDGE && m0 + row >= p.M) voffA[j] = OOB_OFFSET;
        } else {
            const int k = b_slot_k<BM>(j * NW + w, lane), c = b_slot_chunk<BM>(j * NW + w, lane);
            kA[j] = k;
            voffA[j] = (unsigned)k * (unsigned)p.lda * 2u + (unsigned)c * 16u;
            if (EDGE && m0 + c * 8 >= p.M) voffA[j] = OOB_OFFSET;
        }
    }
#pragma unroll
    for (int j = 0; j < NLB; ++j) {
        if (!TB) {
            const int k = b_slot_k<BN>(j * NW + w, lane), c = b_slot_chunk<BN>(j * NW + w, lane);
            kB[j] = k;
            voffB[j] = (unsigned)k * (unsigned)p.ldb * 2u + (unsigned)c * 16u;
            if (EDGE && n0 + c * 8 >= p.N) voffB[j] = OOB_OFFSET;
        } else {
            const int row = B64 ? a64_slot_row(j * NW + w, lane) : a_slot_row(j * NW + w, lane);
            const int c = B64 ? a64_slot_chunk(j * NW + w, lane) : a_slot_chunk(lane);
            kB[j] = c * 8;
            voffB[j] = (unsigned)row * (unsigned)p.ldb * 2u + (unsigned)c * 16u;
            if (EDGE && n0 + row >= p.N) voffB[j] = OOB_OFFSET;
        }
    }

    // Tiles past the end of the K range are fetched through a zero-length resource:
    // every lane is out of range, nothing is read and zeros land in a stage nobody
    // consumes, so the number of loads in flight is the same in every step.
    // convolution: filter tap and first channel of the next K step to be issued (the steps are
    // issued in ascending order, so the state advances by 32 channels per call, on the scalar unit)
    int tapH = 0, tapW = 0, tapC = 0;
    if (CONV) {
        const int tap = kBegin / p.convCin;
        tapC = kBegin % p.convCin;
        tapH = tap / p.convKW;
        tapW = tap % p.convKW;
    }
    // issue_prep(kt) sets up tile kt (resource words, K-edge limit, tap offsets); issue_one(l, ...) then
    // issues its load l (A's first, then B's); issue() is both for all loads.
    rsrc_words_t rA, rB;
    int kLeft = 0, dIh = 0, dIw = 0;                 // valid k in the tile (EDGE only); tap displacement (CONV only)
    unsigned tapOff = 0u;
    auto issue_prep = [&](int kt) {
        const long long stepA = CONV ? 0ll : TA ? (long long)kt * BK * p.lda * 2 : (long long)kt * (BK * 2);
        const long long stepB = TB ? (long long)kt * (BK * 2) : (long long)kt * BK * p.ldb * 2;
        // Full tiles: every offset lies inside the operand by construction, and the exact extent
        // (ten scalar instructions per step, measured at 1-3 % of the 8192^3 run) is skipped.
        // Edge tiles: the resource ends where the operand ends, so a lane that is not masked for
        // whatever reason reads zeros instead of memory beyond the allocation.  Computed
        // unconditionally, then selected: a conditional around it would be a scalar branch.
        const unsigned leftA = (EDGE || CONV) ? records_left(p.bytesA, offA + stepA) : RSRC_RECORDS;
        const unsigned leftB = EDGE ? records_left(p.bytesB, offB + stepB) : RSRC_RECORDS;
        rA = make_rsrc(gA + stepA, kt < nk ? leftA : 0u);
        rB = make_rsrc(gB + stepB, kt < nk ? leftB : 0u);
        kLeft = kLen - kt * BK;
        if (CONV) {
            dIh = tapH * p.convDh;
            dIw = tapW * p.convDw;
            tapOff = (unsigned)(((dIh * p.convW + dIw) * p.convCin + tapC) * 2);
            tapC += BK;
            if (tapC >= p.convCin) { tapC = 0; ++tapW; }
            if (tapW >= p.convKW) { tapW = 0; ++tapH; }
        }
    };
    auto issue_one = [&](int l, GE_LDS char *dA, GE_LDS char *dB) {
        if (l < T::A_LOADS) {
            const int j = l < T::A_LOADS ? l : 0;
            unsigned v = voffA[j];
            if (CONV) {
                const bool inside = (unsigned)(ih0[CONV ? j : 0] + dIh) < (unsigned)p.convH && (unsigned)(iw0[CONV ? j : 0] + dIw) < (unsigned)p.convW;
                v = inside ? v + tapOff : OOB_OFFSET;
            }
            if (EDGE && kA[j] >= kLeft) v = OOB_OFFSET;
            lds_dma16(rA, (unsigned)(size_t)(dA + (j * NW + w) * 1024), v);
        } else {
            const int j = l < T::A_LOADS ? 0 : l - T::A_LOADS;
            unsigned v = voffB[j];
            if (EDGE && kB[j] >= kLeft) v = OOB_OFFSET;
            lds_dma16(rB, (unsigned)(size_t)(dB + (j * NW + w) * 1024), v);
        }
    };
    auto issue = [&](int kt, GE_LDS char *dA, GE_LDS char *dB) {
        issue_prep(kt);
#pragma unroll
        for (int l = 0; l < LOADS; ++l) issue_one(l, dA, dB);
    };

    // K64: tile t64 (64 k from kBegin + 64 t64) into stage `stage` of two.  A k-strided operand
    // goes in as its two 32-k halves, each through a resource of its own.
    const int nk64 = (kLen + 63) / 64;
    auto issue64 = [&](int t64, int stage) {
        GE_LDS char *dA = (GE_LDS char *)smem + stage * 2 * T::A_BYTES;
        GE_LDS char *dB = (GE_LDS char *)smem + 4 * T::A_BYTES + stage * 2 * T::B_BYTES;
        const int kLeft = kLen - t64 * 64;           // valid k in this tile (EDGE only)
        if constexpr (A64) {
            const long long stepA = (long long)t64 * 128;
            const unsigned leftA = EDGE ? records_left(p.bytesA, offA + stepA) : RSRC_RECORDS;
            const rsrc_words_t rA = make_rsrc(gA + stepA, t64 < nk64 ? leftA : 0u);
#pragma unroll
            for (int j = 0; j < NLA; ++j) {
                unsigned v = voffA[j];
                if (EDGE && kA[j] >= kLeft) v = OOB_OFFSET;
                lds_dma16(rA, (unsigned)(size_t)(dA + (j * NW + w) * 1024), v);
            }
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const long long stepA = (long long)(t64 * 64 + h * 32) * p.lda * 2;
                const bool live = t64 < nk64 && (h == 0 || !EDGE || kLeft > 32);
                const unsigned leftA = (EDGE && live) ? records_left(p.bytesA, offA + stepA) : RSRC_RECORDS;
                const rsrc_words_t rA = make_rsrc(gA + stepA, live ? leftA : 0u);
#pragma unroll
                for (int j = 0; j < NLA; ++j) {
                    unsigned v = voffA[j];
                    if (EDGE && kA[j] + 32 * h >= kLeft) v = OOB_OFFSET;
                    lds_dma16(rA, (unsigned)(size_t)(dA + h * T::A_BYTES + (j * NW + w) * 1024), v);
                }
            }
        }
        if constexpr (B64) {
            const long long stepB = (long long)t64 * 128;
            const unsigned leftB = EDGE ? records_left(p.bytesB, offB + stepB) : RSRC_RECORDS;
            const rsrc_words_t rB = make_rsrc(gB + stepB, t64 < nk64 ? leftB : 0u);
#pragma unroll
            for (int j = 0; j < NLB; ++j) {
                unsigned v = voffB[j];
                if (EDGE && kB[j] >= kLeft) v = OOB_OFFSET;
                lds_dma16(rB, (unsigned)(size_t)(dB + (j * NW + w) * 1024), v);
            }
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const long long stepB = (long long)(t64 * 64 + h * 32) * p.ldb * 2;
                const bool live = t64 < nk64 && (h == 0 || !EDGE || kLeft > 32);
                const unsigned leftB = (EDGE && live) ? records_left(p.bytesB, offB + stepB) : RSRC_RECORDS;
                const rsrc_words_t rB = make_rsrc(gB + stepB, live ? leftB : 0u);
#pragma unroll
                for (int j = 0; j < NLB; ++j) {
                    unsigned v = voffB[j];
                    if (EDGE && kB[j] + 32 * h >= kLeft) v = OOB_OFFSET;
                    lds_dma16(rB, (unsigned)(size_t)(dB + h * T::B_BYTES + (j * NW + w) * 1024), v);
                }
            }
        }
    };

    // The same tile in two parts, for the four-wave blocks, which issue its loads between their MFMAs:
    // issue64_prep sets up tile t64, issue64_one issues load l of it (both operands in 128-byte rows).
    rsrc_words_t rA64, rB64;
    int kLeft64 = 0;
    auto issue64_prep = [&](int t64) {
        const long long step = (long long)t64 * 128;
        const unsigned leftA = EDGE ? records_left(p.bytesA, offA + step) : RSRC_RECORDS;
        const unsigned leftB = EDGE ? records_left(p.bytesB, offB + step) : RSRC_RECORDS;
        rA64 = make_rsrc(gA + step, t64 < nk64 ? leftA : 0u);
        rB64 = make_rsrc(gB + step, t64 < nk64 ? leftB : 0u);
        kLeft64 = kLen - t64 * 64;
    };
    auto issue64_one = [&](int l, int stage) {
        if (l < NLA) {
            const int j = l < NLA ? l : 0;
            unsigned v = voffA[j];
            if (EDGE && kA[j] >= kLeft64) v = OOB_OFFSET;
            lds_dma16(rA64, (unsigned)(size_t)((GE_LDS char *)smem + stage * 2 * T::A_BYTES + (j * NW + w) * 1024), v);
        } else {
            const int j = l < NLA ? 0 : l - NLA;
            unsigned v = voffB[j];
            if (EDGE && kB[j] >= kLeft64) v = OOB_OFFSET;
            lds_dma16(rB64, (unsigned)(size_t)((GE_LDS char *)smem + 4 * T::A_BYTES + stage * 2 * T::B_BYTES + (j * NW + w) * 1024), v);
        }
    };

    // ---- per-lane LDS read addresses ---------------------------------------------
    // k-contiguous stage, fragment i: rows base + 16 i + lane%16, k chunk lane/16
    // (k = 8*(lane/16) + e): one ds_read_b128, stepping i adds 1 KB.
    // k-strided stage, fragment j, read r in {0,1}: the 16-lane group g = lane/16 covers
    // k = 8g + 4r .. +3 of columns base + 16 j .. +15; lane i of the group addresses k row i/4,
    // the 4 columns from 4*(i%4), and receives column i of the 4x16 block (k = 8g + 4r + e).
    // Stepping j moves 16 columns: an XOR with 32 j on the hashed half (bit 5) and segment
    // (bits 6..8) fields; stepping r adds 4 k rows.
    // 128-byte-row stage (K64): the k half is carried by the lane part of the address (an XOR),
    // so there is one lane base per half; stepping the row block adds 2 KB.
    const unsigned aBase = TA ? (unsigned)b_frag_offset<BM>(wm * T::WTM, lane, 0)
                              : A64 ? (unsigned)a64_frag_offset(wm * T::WTM, lane, 0) : (unsigned)a_frag_offset(wm * T::WTM, lane);
    const unsigned bBase = TB ? (B64 ? (unsigned)a64_frag_offset(wn * T::WTN, lane, 0) : (unsigned)a_frag_offset(wn * T::WTN, lane))
                              : (unsigned)b_frag_offset<BN>(wn * T::WTN, lane, 0);

    f32x4_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

    bf16x8_t fa[TM], fb[TN];

    // Lane bases held in registers the compiler cannot see through, so that each read below is
    // "base + immediate": one base covers every fragment of a k-contiguous operand, a
    // k-strided operand needs one per 16-column block (its stepping is an XOR, not an add).
    constexpr int NA = TA ? TM : A64 ? 2 : 1, NB = TB ? (B64 ? 2 : 1) : TN;
    unsigned aAddr[NA], bAddr[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        if (A64) aAddr[i] = (unsigned)(size_t)(GE_LDS char *)smem + (unsigned)a64_frag_offset(wm * T::WTM, lane, i);
        else aAddr[i] = (unsigned)(size_t)(GE_LDS char *)smem + (aBase ^ (unsigned)(i * 32));
        asm volatile("" : "+v"(aAddr[i]));
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        if (B64) bAddr[j] = (unsigned)(size_t)(GE_LDS char *)smem + 4 * T::A_BYTES + (unsigned)a64_frag_offset(wn * T::WTN, lane, j);
        else bAddr[j] = (unsigned)(size_t)(GE_LDS char *)smem + 4 * T::A_BYTES + (bBase ^ (unsigned)(j * 32));
        asm volatile("" : "+v"(bAddr[j]));
    }
    auto read_strided = [&](unsigned addr, int rowBytes) {
        const GE_LDS char *ptr = (const GE_LDS char *)(size_t)addr;
        short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)ptr);
        short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)(ptr + 4 * rowBytes));
        short8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8_t, both);
    };
    auto read_frags = [&](int stage) {
#pragma unroll
        // `stage` counts 32-k pieces: under K64, piece q is half q%2 of the 64-k stage q/2
        for (int i = 0; i < TM; ++i) {
            if (TA) fa[i] = read_strided(aAddr[TA ? i : 0] + (unsigned)(stage * T::A_BYTES), BM * 2);
            else if (A64) fa[i] = *(const GE_LDS bf16x8_t *)(size_t)(aAddr[A64 ? (stage & 1) : 0] + (unsigned)((stage >> 1) * 2 * T::A_BYTES + i * 2048));
            else fa[i] = *(const GE_LDS bf16x8_t *)(size_t)(aAddr[0] + (unsigned)(stage * T::A_BYTES + i * 1024));
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (B64) fb[j] = *(const GE_LDS bf16x8_t *)(size_t)(bAddr[B64 ? (stage & 1) : 0] + (unsigned)((stage >> 1) * 2 * T::B_BYTES + j * 2048));
            else if (TB) fb[j] = *(const GE_LDS bf16x8_t *)(size_t)(bAddr[0] + (unsigned)(stage * T::B_BYTES + j * 1024));
            else fb[j] = read_strided(bAddr[TB ? 0 : j] + (unsigned)(stage * T::B_BYTES), BN * 2);
        }
    };
    // accumulator register r of lane l is C[m = 16 i + 4*(l/16) + r][n = 16 j + l%16]; with the
    // operands swapped (OUTBF16) the block comes out transposed: C[m = 16 i + l%16][n = 16 j + 4*(l/16) + r]
    auto mma = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (OUTBF16) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
    };

    // The same with the loads of the tile set up by issue_prep issued between the MFMAs, one every
    // fourth (four-wave blocks: issued back to back at the head of the step they cost 4-7 % on the
    // mid-size shapes these blocks serve, 2048^3 25.7 -> 24.2 us).
    auto mma_with_loads = [&](GE_LDS char *dA, GE_LDS char *dB) {
        constexpr int SPREAD = (TM * TN) / LOADS >= 4 ? 4 : (TM * TN) / LOADS >= 2 ? 2 : 1;
        static_assert(LOADS <= TM * TN, "a load slot per MFMA at most");
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (OUTBF16) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
                const int q = i * TN + j;
                if (q % SPREAD == 0 && q / SPREAD < LOADS) issue_one(q / SPREAD, dA, dB);
                __builtin_amdgcn_sched_barrier(0);
            }
    };

    auto mma_with_loads64 = [&](int stage) {
        constexpr int N64 = NLA + NLB, SPREAD = (TM * TN) / N64 >= 2 ? 2 : 1;
        static_assert(!K64 || N64 <= TM * TN, "a load slot per MFMA at most");
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (OUTBF16) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
                const int q = i * TN + j;
                if (q % SPREAD == 0 && q / SPREAD < N64) issue64_one(q / SPREAD, stage);
                __builtin_amdgcn_sched_barrier(0);
            }
    };

    GE_LDS char *const ldsBase = (GE_LDS char *)smem;
    GE_LDS char *lA[4], *lB[4];
#pragma unroll
    for (int st = 0; st < 4; ++st) {
        lA[st] = ldsBase + st * T::A_BYTES;
        lB[st] = ldsBase + 4 * T::A_BYTES + st * T::B_BYTES;
    }
    // waves w and w+4 share a SIMD: they form the two phase groups
    const int group = w >> 2;

    // One K tile t held in stage S (compile time).  Loads of tile t+3 refill the stage of
    // tile t-1, which every wave has finished reading (barrier of the previous step).
    //  8 waves: [LDS reads t, loads t+3, wait own part of t+1] barrier [MFMAs t] barrier (the LDS
    //           reads go first: their latency, not the load issue, is what the phase waits for),
    //           the two groups half a step apart (one extra barrier for group 1 up front);
    //  4 waves: [wait own part of t] barrier [LDS reads t, MFMAs t with the loads of t+3 between them].
#define GE_BF16_STEP(S, t)                                                                          \
    if (PINGPONG) {                                                                                 \
        read_frags(S);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        issue((t) + 3, lA[((S) + 3) & 3], lB[((S) + 3) & 3]);                                       \
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * LOADS) : "memory");    \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        __builtin_amdgcn_s_setprio(1);                                                              \
        mma();                                                                                      \
        __builtin_amdgcn_s_setprio(0);                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        asm volatile("s_barrier" ::: "memory");                                                     \
        __builtin_amdgcn_sched_barrier(0);                                                          \
    } else {                                                                                        \
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * LOADS) : "memory");    \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        issue_prep((t) + 3);                                                                        \
        read_frags(S);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        mma_with_loads(lA[((S) + 3) & 3], lB[((S) + 3) & 3]);                                       \
        __builtin_amdgcn_sched_barrier(0);                                                          \
    }

    // K64, piece Q (compile time) of the ring, belonging to 64-k tile t64.  Loads of tile t64 + 1
    // are issued in the even piece, into the stage whose second half every wave finished reading
    // before the last barrier, and awaited in the odd piece.
    //  8 waves: [LDS reads, (loads | wait)] barrier [MFMAs] barrier, the two groups half a piece apart;
    //  4 waves: even piece [wait own part of this tile] barrier [LDS reads, MFMAs with the loads of t64+1 between them],
    //           odd piece [LDS reads, MFMAs].
#define GE_BF16_STEP64(Q, t64)                                                                      \
    if (PINGPONG) {                                                                                 \
        read_frags(Q);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        if (((Q) & 1) == 0) {                                                                       \
            issue64((t64) + 1, (((Q) >> 1) ^ 1));                                                   \
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");                         \
        } else {                                                                                    \
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");                \
        }                                                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        __builtin_amdgcn_s_setprio(1);                                                              \
        mma();                                                                                      \
        __builtin_amdgcn_s_setprio(0);                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                          \
        asm volatile("s_barrier" ::: "memory");                                                     \
        __builtin_amdgcn_sched_barrier(0);                                                          \
    } else {                                                                                        \
        if (((Q) & 1) == 0) {                                                                       \
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");                \
            __builtin_amdgcn_sched_barrier(0);                                                      \
            if (A64 && B64) {                                                                       \
                issue64_prep((t64) + 1);                                                            \
                read_frags(Q);                                                                      \
                __builtin_amdgcn_sched_barrier(0);                                                  \
                mma_with_loads64(((Q) >> 1) ^ 1);                                                   \
            } else {                                                                                \
                issue64((t64) + 1, (((Q) >> 1) ^ 1));                                               \
                read_frags(Q);                                                                      \
                mma();                                                                              \
            }                                                                                       \
        } else {                                                                                    \
            read_frags(Q);                                                                          \
            mma();                                                                                  \
        }                                                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                          \
    }

    if constexpr (K64) {
        if (nk64 <= 2) {
            // the whole K range (K <= 128) fits the two stages: one load phase, then the multiply
            issue64(0, 0);
            if (nk64 > 1) issue64(1, 1);
            asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (t < nk) {
                    read_frags(t);
                    mma();
                }
        } else {
            issue64(0, 0);
            if (PINGPONG) {
                asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
                if (group == 1) asm volatile("s_barrier" ::: "memory");
            }
            for (int t = 0;; t += 2) {
                GE_BF16_STEP64(0, t);
                GE_BF16_STEP64(1, t);
                if (t + 1 >= nk64) break;
                GE_BF16_STEP64(2, t + 1);
                GE_BF16_STEP64(3, t + 1);
                if (t + 2 >= nk64) break;
            }
            if (PINGPONG && group == 0) asm volatile("s_barrier" ::: "memory");
        }
    } else if (nk <= 4) {
        // The whole K range fits the four stages (K <= 128, always bound by the C stores): one
        // load phase, one barrier, then the multiply; no ring, no phase groups.
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (t < nk) issue(t, lA[t], lB[t]);
        asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (t < nk) {
                read_frags(t);
                mma();
            }
    } else {
        issue(0, lA[0], lB[0]);
        issue(1, lA[1], lB[1]);
        issue(2, lA[2], lB[2]);
        if (PINGPONG) {
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * LOADS) : "memory");
            if (group == 1) asm volatile("s_barrier" ::: "memory");
        }
        for (int kt = 0;; kt += 4) {
            GE_BF16_STEP(0, kt);
            if (kt + 1 >= nk) break;
            GE_BF16_STEP(1, kt + 1);
            if (kt + 2 >= nk) break;
            GE_BF16_STEP(2, kt + 2);
            if (kt + 3 >= nk) break;
            GE_BF16_STEP(3, kt + 3);
            if (kt + 4 >= nk) break;
        }
        if (PINGPONG && group == 0) asm volatile("s_barrier" ::: "memory");
    }
    // the zero-length loads of the padding tiles must have retired before the LDS is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- epilogue in registers ----------------------------------------------------
    const int rowLane = m0 + wm * T::WTM + 4 * (lane >> 4);
    const int colLane = n0 + wn * T::WTN + (lane & 15);
    if constexpr (FUSED) {
        if constexpr (OUTBF16) {
            // the lane index as a value born here: nothing of the epilogue's address arithmetic can
            // be hoisted above the main loop, where the accumulators leave no registers to hold it
            int laneE = lane, waveE = (int)(threadIdx.x >> 6);
            asm volatile("" : "+v"(laneE), "+v"(waveE));
            const bool resInLds = stage_residual_bf16<BM, BN, NW>(p, tc.b, (GE_LDS char *)smem, m0, n0, p.M, waveE, laneE);
            fused_epilogue_bf16_through_lds<BM, BN, NW, T::LDS_BYTES, TM, TN, EDGE>(
                p, tc.b, acc, (GE_LDS char *)smem, m0, n0, (waveE / WN) * T::WTM + (laneE & 15),
                (waveE % WN) * T::WTN + 4 * (laneE >> 4), waveE, laneE, resInLds);
        } else {
            // only the tiles that hang over M or N pay for masked stores (a uniform branch)
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
            for (int j = 0; j < TN; ++j) {
                const int n = colLane + j * 16;
                bv[j] = (!RAW && p.bias != nullptr && (!MASK || n < p.N)) ? p.bias[n] : 0.0f;
            }
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
        // only the tiles that hang over M or N pay for masked stores (a uniform branch)
        if (!EDGE || (m0 + BM <= p.M && n0 + BN <= p.N)) store_tile(std::false_type{});
        else store_tile(std::true_type{});
    }
}

#undef GE_BF16_STEP
#undef GE_BF16_STEP64

}  // namespace ge
