// 3 x 3, stride-1 convolution of a channels-last bf16 input as an implicit GEMM whose gathered operand
// is staged once per channel slab (optimisation prompt, convolution section: direct -> tiled ->
// implicit GEMM; the tile of the input with its halo is what the "tiled" step keeps on chip).
//
// The gathering kernel (gemm_bf16_fast.h, CONV) fetches the 64 bytes of an input position nine times,
// once per filter tap, and its K step is bound by those loads.  Here a tile is R whole output rows of
// one image and 256 output channels; per slab of 32 input channels the R + 2 input rows the tile needs
// go into LDS once (conv_halo_layout.h), and the nine taps of the slab are nine K steps whose row
// fragments are read from that halo at shifted positions.  Per slab a tile then moves 4 KB per input
// row plus nine filter stages of 16 KB, where the gathering kernel moves nine times 16 KB + 16 KB.
//
// Four waves, one per SIMD, each owning all rows of the tile and 64 of its 256 output channels
// (accumulators in the accumulation registers, fragments of step t + 1 read during the MFMAs of step t,
// loads and fragment reads issued between the MFMAs, one wait and one barrier per step: the schedule of
// gemm_bf16_w4.h).  The filters go through a ring of six stages of 16 KB, fetched six steps ahead (a ring of
// three measured the same: the loads are not late), the halo through two buffers: the seven rows of slab
// s + 1 are fetched during steps 0..3 of slab s and have landed by the end of step 7.  152 KB of LDS in all.
//
// Tiles of two heights share a launch (conv_halo_layout.h: the plan): TMB1 and TMB2 are the row blocks
// of 16 positions that the MFMA loop of either kind covers; positions beyond R * OW are multiplied
// (they read position 0) and never stored.
//
// Needs: 3 x 3 filter, unit strides and dilations, OW + 2 <= 64, Cin a multiple of 64, Cout a multiple
// of 256, X and Wt 16-byte aligned, the input smaller than 2 GiB; bf16 output in 16-byte row pieces.
#pragma once
#include "conv_halo_launch.h"
#include "conv_halo_layout.h"
#include "gemm_bf16_fast.h"

namespace ge {

struct HaloGeom {
    static constexpr int NSTG = 6;                                 // filter stages: loads run six steps ahead
    static constexpr int B_STAGE = 256 * 64;                       // 256 filters x 32 k
    static constexpr int HALO_BUF = ge_halo::HALO_BUF_BYTES;        // 28 KB
    static constexpr int B_BASE = 2 * HALO_BUF;                    // behind the two halo buffers
    static constexpr int RING_BYTES = B_BASE + NSTG * B_STAGE;     // 152 KB
    static constexpr int lds_bytes(int tmb) { return tmb * 16 * 512 > RING_BYTES ? tmb * 16 * 512 : RING_BYTES; }
};

// halo rows of the next slab fetched in step `tap` of a slab: rows 2 tap and 2 tap + 1 in steps 0..2, row 6 in step 3
constexpr int halo_loads_in_step(int tap) { return tap < 3 ? 2 : tap == 3 ? 1 : 0; }
// loads a wave issues in the four steps that end with step `tap` of a slab (four filter loads per step)
constexpr int loads_in_last_four_steps(int tap)
{
    int n = 0;
    for (int d = 0; d < 4; ++d) n += 4 + halo_loads_in_step((tap + 9 - d) % 9);
    return n;
}
static_assert(ge_halo::HALO_ROWS == 7, "the halo loads of steps 0..3 cover seven rows");

// s_waitcnt vmcnt(N) lgkmcnt(0) as an instruction the compiler sees.  Written as inline assembly, the wait
// is opaque to the compiler's own bookkeeping of LDS reads: it goes on believing that the fragment reads of
// the step before are still on their way and guards the first MFMAs of a step with waits of its own ("at
// most 3, 2, 1 LDS operations outstanding").  Those waits are satisfied when they are reached (the counter is
// already below their bound), so this buys instructions, not time: 88 -> 17 waits per 18 steps.
template <int N>
__device__ __forceinline__ void wait_loads_and_lds()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    // vmcnt[3:0] | expcnt[6:4] = 7 (none) | lgkmcnt[11:8] = 0 | vmcnt[5:4] at [15:14]
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (0 << 8) | ((N >> 4) << 14));
}

// lds_dma16 with a scalar byte offset into the buffer on top of the lane's
__device__ inline void lds_dma16_at(rsrc_words_t rs, unsigned ldsAddr, unsigned voff, unsigned soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(ldsAddr), "v"(voff), "s"(rs), "s"(__builtin_amdgcn_readfirstlane(soff)) : "memory", "m0");
}

// ids of a launch's blocks go round the 8 XCDs; give each XCD a contiguous run of the `total` logical ids
__device__ inline unsigned xcd_contiguous(unsigned id, unsigned total)
{
    const unsigned q = total / 8u, rem = total % 8u, xcd = id % 8u;
    return xcd * q + (xcd < rem ? xcd : rem) + id / 8u;
}

template <int TMB, bool OUTBF16, int LDS_BYTES>
__device__ __forceinline__ void conv_halo_tile(const GemmParams &p, GE_LDS char *smem, int img, int oh0, int R, int n0, int posMul)
{
    using namespace ge_halo;
    using G = HaloGeom;
    constexpr int TN = 4, NW = 4, NMFMA = TMB * TN, NREAD = TMB + TN, NSTG = G::NSTG;
    static_assert(2 * NREAD <= NMFMA && NMFMA >= 28, "a step has room for its loads and fragment reads");
    static_assert(18 % NSTG == 0 && NSTG == 6, "the ring divides the 18 steps of the loop body; two lane bases cover six stages");

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int OW = p.convOW, Cin = p.convCin;
    const int nSlabs = Cin / 32;                                   // even (the host checks)
    const int rowsValid = R * OW;
    const int m0 = (img * p.convOH + oh0) * OW;
    const int ihTop = oh0 - p.convPh;                              // input row of halo row 0

    // ---- halo loads: one input row per load, this lane's 16 bytes of it --------------------------
    unsigned voffH;
    {
        const int iw = halo_slot_col(w, lane) - p.convPw;
        voffH = (iw >= 0 && iw < p.convW) ? (unsigned)(iw * Cin * 2 + halo_slot_chunk(w, lane) * 16) : OOB_OFFSET;
    }
    // One resource for the halo and one for the filters for the whole tile; a load's place in the operand is
    // its scalar offset (halo: row j of channel slab `slab`; filters: 32 channels of tap `tap` in slab `slab`),
    // so a step spends a handful of scalar instructions on its loads.  A load that must fetch nothing (a
    // halo row outside the image or beyond the tile's R + 2, a slab past the last) has the out-of-range
    // bit ORed into its lane offsets: zeros land, no memory is touched.
    const long long rowBytes = (long long)p.convW * Cin * 2;
    const long long haloBase = ((long long)img * p.convH + ihTop) * rowBytes;      // may lie before X: rows above the image are dead
    unsigned liveRows = 0u;
#pragma unroll
    for (int j = 0; j < HALO_ROWS; ++j) {
        const int ih = ihTop + j;
        liveRows |= ((unsigned)(j < R + 2) & (unsigned)(ih >= 0) & (unsigned)(ih < p.convH)) << j;
    }
    const rsrc_words_t rH = make_rsrc((const char *)p.A + haloBase, RSRC_RECORDS);
    const unsigned rowBytes32 = (unsigned)rowBytes;                                 // the input is smaller than 2 GiB
    auto halo_soff = [&](int j, int slab) { return (unsigned)j * rowBytes32 + (unsigned)slab * 64u; };
    auto halo_dead = [&](int j, int slab) { return (0u - (1u ^ ((liveRows >> j) & (unsigned)(slab < nSlabs) & 1u))) & OOB_OFFSET; };

    // ---- filter loads: 256 rows of 64 bytes, the k-contiguous stage of the GEMM kernels ----------
    const char *gB = (const char *)p.B + (long long)n0 * p.ldb * 2;
    unsigned voffB[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        voffB[j] = (unsigned)a_slot_row(j * NW + w, lane) * (unsigned)p.ldb * 2u + (unsigned)a_slot_chunk(lane) * 16u;
    const rsrc_words_t rB = make_rsrc(gB, RSRC_RECORDS);
    const unsigned cin2 = (unsigned)Cin * 2u;
    auto filt_soff = [&](int tap, int slab) { return (unsigned)tap * cin2 + (unsigned)slab * 64u; };
    auto filt_dead = [&](int slab) { return (0u - (unsigned)(slab >= nSlabs)) & OOB_OFFSET; };

    const unsigned ldsBase = (unsigned)(size_t)smem;

    // the halo of slab 0 and the filter stages of steps 0..5 are on their way before anything else is set up
#pragma unroll
    for (int j = 0; j < HALO_ROWS; ++j)
        lds_dma16_at(rH, ldsBase + (unsigned)(j * HALO_ROW_BYTES + w * 1024), voffH | halo_dead(j, 0), halo_soff(j, 0));
#pragma unroll
    for (int t = 0; t < NSTG; ++t) {
#pragma unroll
        for (int d = 0; d < 4; ++d)
            lds_dma16_at(rB, ldsBase + (unsigned)(G::B_BASE + t * G::B_STAGE + (d * NW + w) * 1024), voffB[d] | filt_dead(0), filt_soff(t, 0));
    }

    // ---- fragment read addresses: one lane base per row block and filter column ------------------
    unsigned aAddr[3][TMB], bAddr[2];
#pragma unroll
    for (int i = 0; i < TMB; ++i) {
        int pos = 16 * i + (lane & 15);
        if (pos >= rowsValid) pos = 0;
        const int ro = (pos * posMul) >> 16;
        const int h0 = ro * HALO_PITCH + (pos - ro * OW);
#pragma unroll
        for (int dw = 0; dw < 3; ++dw) {
            aAddr[dw][i] = ldsBase + (unsigned)halo_offset(h0 + dw, lane >> 4);
            asm volatile("" : "+v"(aAddr[dw][i]));
        }
    }
    bAddr[0] = ldsBase + G::B_BASE + (unsigned)a_frag_offset(w * 64, lane);
    bAddr[1] = bAddr[0] + 3 * G::B_STAGE;            // a read's immediate offset reaches 64 KB: three stages per base
    asm volatile("" : "+v"(bAddr[0]), "+v"(bAddr[1]));

    f32x4_t acc[TMB][TN];
#pragma unroll
    for (int i = 0; i < TMB; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

    bf16x8_t fa[2][TMB], fb[2][TN];

    // fragment r (row blocks first, then the wave's four filter blocks) of tap TAP, halo buffer BUF, filter
    // stage STG, into register set NX
#define GE_HALO_READ(r, TAP, BUF, STG, NX)                                                             \
    do {                                                                                               \
        if ((r) < TMB)                                                                                 \
            fa[NX][(r) < TMB ? (r) : 0] = *(const GE_LDS bf16x8_t *)(size_t)(aAddr[(TAP) % 3][(r) < TMB ? (r) : 0] + \
                                              (unsigned)((BUF) * G::HALO_BUF + ((TAP) / 3) * HALO_ROW_BYTES)); \
        else                                                                                           \
            fb[NX][(r) < TMB ? 0 : (r) - TMB] = *(const GE_LDS bf16x8_t *)(size_t)(bAddr[(STG) / 3] + (unsigned)(((STG) % 3) * G::B_STAGE + ((r) < TMB ? 0 : (r) - TMB) * 1024)); \
    } while (0)

    // accumulator register r of lane l is Y[pos = 16 i + 4*(l/16) + r][channel = 16 j + l%16]; with the
    // operands swapped (OUTBF16) the block comes out transposed
#define GE_HALO_MFMA(i, j, CU)                                                                         \
    do {                                                                                               \
        if (OUTBF16) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fb[CU][j]), "v"(fa[CU][i])); \
        else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fa[CU][i]), "v"(fb[CU][j])); \
    } while (0)

    // Step TAP of the slab with parity PAR in the loop body (step K = 9 PAR + TAP of its 18; slab s + PAR,
    // halo buffer PAR): the MFMAs of the step on register set CU, with in between
    //   * the halo rows of the next slab that this step fetches (two each in steps 0..2, the seventh in
    //     step 3; the other buffer, last read two steps before this slab began),
    //   * the filter stage of step K + 6 (stage K % 6, whose fragments were read during the step before),
    //   * the fragment reads of step K + 1.
    // Then: every load issued four or more steps ago has landed (the loads complete in order: "all but
    // those of the last four steps"), which covers the filter stage of step K + 2 and the halo rows
    // issued in steps 0..3 by the end of step 7; own fragment reads done; barrier.
#define GE_HALO_STEP(TAP, PAR, CU, NX)                                                                 \
    {                                                                                                  \
        constexpr int K_ = (PAR) * 9 + (TAP);                                                          \
        unsigned soffB_ = 0u, deadB_ = 0u, soffH0_ = 0u, deadH0_ = 0u, soffH1_ = 0u, deadH1_ = 0u;     \
        _Pragma("unroll") for (int q = 0; q < NMFMA; ++q) {                                            \
            GE_HALO_MFMA(q / TN, q % TN, CU);                                                          \
            if (q == 0) {                                                                              \
                /* the scalar work of the step's loads, behind its first MFMA */                       \
                soffB_ = filt_soff(((TAP) + NSTG) % 9, s + (PAR) + ((TAP) + NSTG) / 9);                \
                deadB_ = filt_dead(s + (PAR) + ((TAP) + NSTG) / 9);                                    \
                if (halo_loads_in_step(TAP) > 0) { soffH0_ = halo_soff(2 * (TAP), s + (PAR) + 1); deadH0_ = halo_dead(2 * (TAP), s + (PAR) + 1); } \
                if (halo_loads_in_step(TAP) > 1) { soffH1_ = halo_soff(2 * (TAP) + 1, s + (PAR) + 1); deadH1_ = halo_dead(2 * (TAP) + 1, s + (PAR) + 1); } \
            }                                                                                          \
            if (q == 2 && halo_loads_in_step(TAP) > 0)                                                 \
                lds_dma16_at(rH, ldsBase + (unsigned)((((PAR) + 1) & 1) * G::HALO_BUF + 2 * (TAP) * HALO_ROW_BYTES + w * 1024), voffH | deadH0_, soffH0_); \
            if (q == 4 && halo_loads_in_step(TAP) > 1)                                                 \
                lds_dma16_at(rH, ldsBase + (unsigned)((((PAR) + 1) & 1) * G::HALO_BUF + (2 * (TAP) + 1) * HALO_ROW_BYTES + w * 1024), voffH | deadH1_, soffH1_); \
            if (q % 2 == 0 && q >= 6 && q < 14)                                                        \
                lds_dma16_at(rB, ldsBase + (unsigned)(G::B_BASE + (K_ % NSTG) * G::B_STAGE + (((q - 6) / 2) * NW + w) * 1024), voffB[((q - 6) / 2) & 3] | deadB_, soffB_); \
            if ((q & 1) && q < 2 * NREAD)                                                              \
                GE_HALO_READ(q >> 1, ((TAP) + 1) % 9, (TAP) == 8 ? (((PAR) + 1) & 1) : (PAR), (K_ + 1) % NSTG, NX); \
            __builtin_amdgcn_sched_barrier(0);                                                         \
        }                                                                                              \
        wait_loads_and_lds<loads_in_last_four_steps(TAP)>();                                           \
        asm volatile("s_barrier" ::: "memory");                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                             \
    }

    {
        // halo and step 0 landed -> its fragments; step 1 landed -> the loop
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(4 * (NSTG - 1)) : "memory");
#pragma unroll
        for (int r = 0; r < NREAD; ++r) GE_HALO_READ(r, 0, 0, 0, 0);
        wait_loads_and_lds<4 * (NSTG - 2)>();
        asm volatile("s_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        // one back edge, no exit from the middle (with more the register allocator spills the accumulators)
        for (int s = 0; s < nSlabs; s += 2) {
            GE_HALO_STEP(0, 0, 0, 1);
            GE_HALO_STEP(1, 0, 1, 0);
            GE_HALO_STEP(2, 0, 0, 1);
            GE_HALO_STEP(3, 0, 1, 0);
            GE_HALO_STEP(4, 0, 0, 1);
            GE_HALO_STEP(5, 0, 1, 0);
            GE_HALO_STEP(6, 0, 0, 1);
            GE_HALO_STEP(7, 0, 1, 0);
            GE_HALO_STEP(8, 0, 0, 1);
            GE_HALO_STEP(0, 1, 1, 0);
            GE_HALO_STEP(1, 1, 0, 1);
            GE_HALO_STEP(2, 1, 1, 0);
            GE_HALO_STEP(3, 1, 0, 1);
            GE_HALO_STEP(4, 1, 1, 0);
            GE_HALO_STEP(5, 1, 0, 1);
            GE_HALO_STEP(6, 1, 1, 0);
            GE_HALO_STEP(7, 1, 0, 1);
            GE_HALO_STEP(8, 1, 1, 0);
        }
    }
    // the zero-length loads past the end must have retired before the LDS is reused, and the
    // accumulation registers of the last MFMAs must be readable (the compiler does not see the MFMAs)
    asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");

#undef GE_HALO_STEP
#undef GE_HALO_MFMA
#undef GE_HALO_READ

    // ---- consumer chain and stores: the epilogues of the GEMM kernels on a tile of rowsValid rows ----
    int laneE = lane, waveE = (int)(threadIdx.x >> 6);
    asm volatile("" : "+v"(laneE), "+v"(waveE));
    GemmParams q = p;
    q.M = m0 + rowsValid;
    if constexpr (OUTBF16) {
        // a bf16 residual goes into the LDS image of the tile first (gemm_bf16_fast.h: stage_residual_bf16)
        const bool resInLds = stage_residual_bf16<TMB * 16, 256, NW>(p, 0, smem, m0, n0, m0 + rowsValid, waveE, laneE);
        fused_epilogue_bf16_through_lds<TMB * 16, 256, NW, LDS_BYTES, TMB, TN, true>(
            q, 0, acc, smem, m0, n0, laneE & 15, waveE * 64 + 4 * (laneE >> 4), waveE, laneE, resInLds);
    } else {
        const int rowLane = m0 + 4 * (laneE >> 4), colLane = n0 + waveE * 64 + (laneE & 15);
        if (rowsValid == TMB * 16) fused_epilogue_f32_direct<TMB, TN, false>(q, 0, acc, rowLane, colLane);
        else fused_epilogue_f32_direct<TMB, TN, true>(q, 0, acc, rowLane, colLane);
    }
}

template <int TMB1, int TMB2, bool OUTBF16>
__global__ void __launch_bounds__(256)
conv_halo_bf16_kernel(const GemmParams p, const HaloTiles ht)
{
    constexpr int LDS_BYTES = HaloGeom::lds_bytes(TMB1 > TMB2 ? TMB1 : TMB2);
    __shared__ __attribute__((aligned(1024))) char smem[LDS_BYTES];
    const unsigned bid = blockIdx.x;
    const bool first = bid < (unsigned)ht.tiles1;
    const unsigned idx = first ? bid : bid - (unsigned)ht.tiles1;
    // logical id within the kind: tile column fastest, then the row groups of an image, then the images
    const unsigned L = xcd_contiguous(idx, (unsigned)(first ? ht.tiles1 : ht.tiles2));
    const unsigned g = (unsigned)(first ? ht.g1 : ht.g2);
    const unsigned tn = L % (unsigned)ht.tilesN, t = L / (unsigned)ht.tilesN;
    const int img = __builtin_amdgcn_readfirstlane((int)(t / g));
    const int grp = __builtin_amdgcn_readfirstlane((int)(t % g));
    const int n0 = __builtin_amdgcn_readfirstlane((int)tn * 256);
    const int oh0 = first ? grp * ht.R1 : ht.g1 * ht.R1 + grp * ht.R2, R = first ? ht.R1 : ht.R2;
    if constexpr (TMB1 == TMB2) {
        conv_halo_tile<TMB1, OUTBF16, LDS_BYTES>(p, (GE_LDS char *)smem, img, oh0, R, n0, ht.posMul);
    } else {
        if (first) conv_halo_tile<TMB1, OUTBF16, LDS_BYTES>(p, (GE_LDS char *)smem, img, oh0, R, n0, ht.posMul);
        else conv_halo_tile<TMB2, OUTBF16, LDS_BYTES>(p, (GE_LDS char *)smem, img, oh0, R, n0, ht.posMul);
    }
}

}  // namespace ge
