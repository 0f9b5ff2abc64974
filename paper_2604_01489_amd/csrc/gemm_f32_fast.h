// fp32 x fp32 -> fp32 GEMM main kernel for gfx950: v_mfma_f32_32x32x2_f32 (true fp32 products and
// sums; the paper's audit forbids lowering operand precision, and gfx950 has no reduced-precision
// fp32 matrix path anyway), fed the same way as the bf16 kernel:
//   * BM x BN workgroup tile, K step 16, 4 wavefronts (2 x 2), each a grid of 32x32 accumulators;
//   * A and B tiles go global -> LDS with buffer_load_dwordx4 ... lds into a ring of four stages,
//     three tiles in flight, awaited with s_waitcnt vmcnt(N);
//   * an A stage row is 16 floats = 64 bytes and a B stage row BN floats: byte for byte the
//     geometry of the bf16 stages (64-byte A rows, B rows of 2*(2 BN) bytes), so the same swizzled
//     slot maps are used, with a 16-byte chunk now holding 4 floats;
//   * A fragments: one ds_read_b128 gives a lane 4 consecutive k of its row, used by 4 successive
//     MFMAs; the k each lane group contributes to an MFMA is a free choice as long as A and B
//     agree, here k = 8*rho + 4*(lane/32) + e for read rho, element e.  B fragments: ds_read_b32 of
//     B[k][n = lane%32], consecutive lanes on consecutive addresses;
//   * epilogue in registers: a store instruction writes 128 contiguous bytes of 2 rows;
//   * K slices (few tiles, long K): block slice s walks k in [s kPerSlice, (s + 1) kPerSlice) and, RAW,
//     leaves its sums unscaled in the workspace W[s][batch][M][N] for the second pass.
// Resources carry the exact extent of the operands, so a wrong offset reads zeros, never faults.
#pragma once
#include "bf16_layout.h"
#include "ge_device.h"
#include "gemm_bf16_fast.h"

namespace ge {

template <int BM, int BN>
struct F32Tile {
    static constexpr int BK = 16, NW = 4, WM = 2, WN = 2;
    static constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
    static constexpr int A_BYTES = BM * BK * 4, B_BYTES = BK * BN * 4;
    static constexpr int A_LOADS = A_BYTES / 1024 / NW, B_LOADS = B_BYTES / 1024 / NW;
    static constexpr int LOADS = A_LOADS + B_LOADS;
    static constexpr int LDS_BYTES = 4 * (A_BYTES + B_BYTES);
    static constexpr int BNB = 2 * BN;     // width of the bf16 B stage with the same row bytes
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be 32x32 blocks");
    static_assert((A_BYTES / 1024) % NW == 0 && (B_BYTES / 1024) % NW == 0, "loads must divide over waves");
    static_assert((BN & (BN - 1)) == 0 && BN >= 64, "BN must be a power of two, at least 64");
};

template <int BM, int BN, bool EDGE, bool RAW = false>
__global__ void __launch_bounds__(256)
gemm_f32_fast_kernel(const GemmParams p)
{
    using T = F32Tile<BM, BN>;
    constexpr int BK = T::BK, NW = T::NW, TM = T::TM, TN = T::TN, LOADS = T::LOADS, BNB = T::BNB;

    __shared__ __attribute__((aligned(1024))) char smem[T::LDS_BYTES];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = w / T::WN, wn = w % T::WN;

    const TileCoord tc = map_block(p);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;
    const int kBegin = tc.s * p.kPerSlice;                  // the whole K range when there are no slices
    const int kLen = min(p.K, kBegin + p.kPerSlice) - kBegin;
    const int nk = (kLen + BK - 1) / BK;

    const long long offA = 4 * ((long long)tc.b * p.strideA + (long long)m0 * p.lda + kBegin);
    const long long offB = 4 * ((long long)tc.b * p.strideB + (long long)kBegin * p.ldb + n0);
    const char *gA = (const char *)p.A + offA;
    const char *gB = (const char *)p.B + offB;

    // per-lane global offsets of the 16-byte chunks (4 floats) this lane fetches
    unsigned voffA[T::A_LOADS], voffB[T::B_LOADS];
    int chA[T::A_LOADS], rowB[T::B_LOADS];
#pragma unroll
    for (int j = 0; j < T::A_LOADS; ++j) {
        const int row = a_slot_row(j * NW + w, lane), c = a_slot_chunk(lane);
        chA[j] = c;
        voffA[j] = (unsigned)row * (unsigned)p.lda * 4u + (unsigned)c * 16u;
        if (EDGE && m0 + row >= p.M) voffA[j] = OOB_OFFSET;
    }
#pragma unroll
    for (int j = 0; j < T::B_LOADS; ++j) {
        const int k = b_slot_k<BNB>(j * NW + w, lane), c = b_slot_chunk<BNB>(j * NW + w, lane);
        rowB[j] = k;
        voffB[j] = (unsigned)k * (unsigned)p.ldb * 4u + (unsigned)c * 16u;
        if (EDGE && n0 + c * 4 >= p.N) voffB[j] = OOB_OFFSET;
    }

    GE_LDS char *const ldsBase = (GE_LDS char *)smem;
    auto issue = [&](int kt, int stage) {
        const long long stepA = (long long)kt * (BK * 4), stepB = (long long)kt * BK * p.ldb * 4;
        const unsigned leftA = records_left(p.bytesA, offA + stepA);
        const unsigned leftB = records_left(p.bytesB, offB + stepB);
        const rsrc_words_t rA = make_rsrc(gA + stepA, kt < nk ? leftA : 0u);
        const rsrc_words_t rB = make_rsrc(gB + stepB, kt < nk ? leftB : 0u);
        const int kLeft = kLen - kt * BK;
        GE_LDS char *dA = ldsBase + stage * T::A_BYTES;
        GE_LDS char *dB = ldsBase + 4 * T::A_BYTES + stage * T::B_BYTES;
#pragma unroll
        for (int j = 0; j < T::A_LOADS; ++j) {
            unsigned v = voffA[j];
            if (EDGE && chA[j] * 4 >= kLeft) v = OOB_OFFSET;
            lds_dma16(rA, (unsigned)(size_t)(dA + (j * NW + w) * 1024), v);
        }
#pragma unroll
        for (int j = 0; j < T::B_LOADS; ++j) {
            unsigned v = voffB[j];
            if (EDGE && rowB[j] >= kLeft) v = OOB_OFFSET;
            lds_dma16(rB, (unsigned)(size_t)(dB + (j * NW + w) * 1024), v);
        }
    };

    // A fragment (i, rho): row wm*WTM + 32 i + lane%32, chunk 2*rho + lane/32
    const int g = lane >> 5, l32 = lane & 31;
    unsigned aAddr[2];
#pragma unroll
    for (int rho = 0; rho < 2; ++rho) {
        aAddr[rho] = (unsigned)(size_t)ldsBase + (unsigned)lds_a_offset(wm * T::WTM + l32, 2 * rho + g);
        asm volatile("" : "+v"(aAddr[rho]));
    }
    // B element (j, rho, e): k = 8 rho + 4 g + e, column wn*WTN + 32 j + lane%32
    unsigned bAddr[TN][2][4];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int rho = 0; rho < 2; ++rho)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = 8 * rho + 4 * g + e, n = wn * T::WTN + 32 * j + l32;
                bAddr[j][rho][e] = (unsigned)(size_t)ldsBase + 4 * T::A_BYTES +
                                   (unsigned)lds_b_offset<BNB>(k, n >> 2) + (unsigned)(n & 3) * 4u;
            }

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    auto compute = [&](int stage) {
#pragma unroll
        for (int rho = 0; rho < 2; ++rho) {
            f32x4_t a[TM];
            float b[TN][4];
#pragma unroll
            for (int i = 0; i < TM; ++i)      // 32 rows further = 2 row groups of 16 = 2 KB
                a[i] = *(const GE_LDS f32x4_t *)(size_t)(aAddr[rho] + (unsigned)(stage * T::A_BYTES + i * 2048));
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    b[j][e] = *(const GE_LDS float *)(size_t)(bAddr[j][rho][e] + (unsigned)(stage * T::B_BYTES));
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][e], b[j][e], acc[i][j], 0, 0, 0);
        }
    };

#define GE_F32_STEP(S, t)                                                                        \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * LOADS) : "memory");       \
    issue((t) + 3, ((S) + 3) & 3);                                                               \
    compute(S);

    issue(0, 0);
    issue(1, 1);
    issue(2, 2);
    for (int kt = 0;; kt += 4) {
        GE_F32_STEP(0, kt);
        if (kt + 1 >= nk) break;
        GE_F32_STEP(1, kt + 1);
        if (kt + 2 >= nk) break;
        GE_F32_STEP(2, kt + 2);
        if (kt + 3 >= nk) break;
        GE_F32_STEP(3, kt + 3);
        if (kt + 4 >= nk) break;
    }
#undef GE_F32_STEP
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // epilogue: accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32
    float *cBase = p.C + (long long)tc.b * p.strideC + (RAW ? (long long)tc.s * p.sliceStride : 0ll);
    const int rowLane = m0 + wm * T::WTM + 4 * g;
    const int colLane = n0 + wn * T::WTN + l32;
    float bv[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = colLane + j * 32;
        bv[j] = (!RAW && p.bias != nullptr && (!EDGE || n < p.N)) ? p.bias[n] : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = rowLane + i * 32 + 8 * (r >> 2) + (r & 3);
            float *rowPtr = cBase + (long long)m * p.ldc + colLane;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float v = RAW ? acc[i][j][r] : epilogue_value_rt(acc[i][j][r], p.alpha, bv[j], p.act);
                if (!EDGE || (m < p.M && colLane + j * 32 < p.N)) rowPtr[j * 32] = v;
            }
        }
}

}  // namespace ge
