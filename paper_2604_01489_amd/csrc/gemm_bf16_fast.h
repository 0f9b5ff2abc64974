// bf16 x bf16 -> fp32 GEMM main kernel for gfx950 (MI355X).
//
// Structure, after the optimisation list for GEMM-like kernels in the paper's
// optimisation prompt (block tiling, wave tiling, matrix instructions, bank
// conflict free staging, multi-stage asynchronous loads) and the square-GEMM
// case study (two staging buffers per operand, next K tile prefetched while the
// current one is consumed), redone for CDNA4:
//   * one workgroup owns a BM x BN tile of C and walks K in steps of 64;
//   * WM x WN wavefronts of 64 lanes, each owning a (BM/WM) x (BN/WN) sub-tile
//     as a grid of 32x32 v_mfma_f32_32x32x16_bf16 accumulators (fp32);
//   * A and B tiles go global -> LDS with buffer_load_dwordx4 ... lds (16 bytes
//     per lane, no register round trip), two stages, one barrier per K tile;
//   * A fragments are ds_read_b128, B fragments ds_read_b64_tr_b16 (B is
//     [K,N] row-major while the matrix unit wants 8 consecutive k per lane);
//   * both LDS layouts are XOR-swizzled so fragment reads spread over all banks;
//     because a direct-to-LDS load lands at base + 16*lane, the swizzle is
//     applied by choosing which global chunk each lane fetches;
//   * scale, bias and activation are applied to the accumulators in registers
//     and C is written once.
#pragma once
#include "ge_device.h"

namespace ge {

constexpr int BF16_BK = 64;
constexpr unsigned OOB_OFFSET = 0x80000000u;   // beyond num_records: the load returns 0
constexpr unsigned RSRC_RECORDS = 0x80000000u;
constexpr unsigned RSRC_FLAGS = 0x00020000u;   // raw buffer, 32-bit data format
// s_waitcnt immediate (gfx9 encoding): vmcnt = 0, expcnt and lgkmcnt left at their maxima
constexpr int WAIT_VMCNT0 = 0x0F70;

// LDS byte offset of 16-byte chunk `c` (8 bf16 along k) of row `row` in an A
// stage.  Rows r and r+8 share a 256-byte line (one in each half) and the chunk
// index is XORed with row%8, so 8 or 16 consecutive rows reading the same k
// chunk touch distinct banks.
__device__ __host__ constexpr int lds_a_offset(int row, int c)
{
    return (((row >> 4) * 8 + (row & 7)) * 256) + (((row >> 3) & 1) * 128) + ((c ^ (row & 7)) * 16);
}

// 3-bit hash of a k row used to rotate the 64-byte column segments of a B stage:
// the 8 k rows one transposing read touches (k%16 in {0..3, 8..11} or
// {4..7, 12..15}) get 8 distinct values.
__device__ __host__ constexpr int lds_b_hash(int k)
{
    return (k & 3) | ((k >> 1) & 4);
}

// LDS byte offset of 16-byte chunk `c` (8 bf16 along n) of k row `k` in a B
// stage of width BN.
template <int BN>
__device__ __host__ constexpr int lds_b_offset(int k, int c)
{
    constexpr int SEGS = BN / 32;
    return k * (BN * 2) + ((((c >> 2) ^ lds_b_hash(k)) & (SEGS - 1)) * 64) + ((c & 3) * 16);
}

template <int BM, int BN, int WM, int WN>
struct Bf16Tile {
    static constexpr int BK = BF16_BK;
    static constexpr int NW = WM * WN;
    static constexpr int THREADS = NW * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BK * BN * 2;
    static constexpr int A_LOADS = A_BYTES / 1024 / NW;  // wave-wide 1 KB loads per wave
    static constexpr int B_LOADS = B_BYTES / 1024 / NW;
    static constexpr int LDS_BYTES = 2 * (A_BYTES + B_BYTES);
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be 32x32 blocks");
    static_assert((A_BYTES / 1024) % NW == 0 && (B_BYTES / 1024) % NW == 0, "loads must divide over waves");
    static_assert(BM % 16 == 0 && BN % 32 == 0 && (BN & (BN - 1)) == 0, "tile shape");
    static_assert((TN & (TN - 1)) == 0, "TN must be a power of two");
};

// EDGE: the tile may hang over M, N or the K range (loads are zero filled
// through the buffer bounds check, stores are masked).  RAW: write alpha-less,
// bias-less fp32 partial sums for the split-K reduction instead of C.
template <int BM, int BN, int WM, int WN, bool EDGE, bool RAW, int ACT>
__global__ void __launch_bounds__(WM * WN * 64)
gemm_bf16_kernel(const GemmParams p)
{
    using T = Bf16Tile<BM, BN, WM, WN>;
    constexpr int BK = T::BK, NW = T::NW, TM = T::TM, TN = T::TN;

    __shared__ __attribute__((aligned(1024))) char sA0[T::A_BYTES];
    __shared__ __attribute__((aligned(1024))) char sA1[T::A_BYTES];
    __shared__ __attribute__((aligned(1024))) char sB0[T::B_BYTES];
    __shared__ __attribute__((aligned(1024))) char sB1[T::B_BYTES];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = w / WN, wn = w % WN;

    const TileCoord tc = map_block(p);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;
    const int kBegin = tc.s * p.kPerSlice;
    const int kLen = min(p.K - kBegin, p.kPerSlice);
    const int nk = (kLen + BK - 1) / BK;

    const char *gA = (const char *)p.A + 2 * ((long long)tc.b * p.strideA + (long long)m0 * p.lda + kBegin);
    const char *gB = (const char *)p.B + 2 * ((long long)tc.b * p.strideB + (long long)kBegin * p.ldb + n0);

    // ---- per-lane global offsets of the 16-byte chunks this lane fetches -----
    unsigned voffA[T::A_LOADS], voffB[T::B_LOADS];
    int rowA[T::A_LOADS], chA[T::A_LOADS], rowB[T::B_LOADS];
    bool okB[T::B_LOADS];
#pragma unroll
    for (int j = 0; j < T::A_LOADS; ++j) {
        const int q = (j * NW + w) * 64 + lane;      // 16-byte slot in the stage
        const int line = q >> 4, half = (q >> 3) & 1, pc = q & 7;
        const int row = (line >> 3) * 16 + half * 8 + (line & 7);
        const int c = pc ^ (row & 7);
        rowA[j] = row;
        chA[j] = c;
        voffA[j] = (unsigned)row * (unsigned)p.lda * 2u + (unsigned)c * 16u;
        if (EDGE && m0 + row >= p.M) voffA[j] = OOB_OFFSET;
    }
#pragma unroll
    for (int j = 0; j < T::B_LOADS; ++j) {
        constexpr int CPR = BN / 8;                  // chunks per k row
        const int q = (j * NW + w) * 64 + lane;
        const int k = q / CPR, pc = q % CPR;
        const int seg = ((pc >> 2) ^ lds_b_hash(k)) & (BN / 32 - 1);
        const int c = seg * 4 + (pc & 3);
        rowB[j] = k;
        voffB[j] = (unsigned)k * (unsigned)p.ldb * 2u + (unsigned)c * 16u;
        okB[j] = !EDGE || (n0 + c * 8 < p.N);
        if (!okB[j]) voffB[j] = OOB_OFFSET;
    }

    auto issue = [&](int kt, GE_LDS char *dA, GE_LDS char *dB) {
        const __amdgpu_buffer_rsrc_t rA = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(gA + (long long)kt * (BK * 2)), 0, RSRC_RECORDS, RSRC_FLAGS);
        const __amdgpu_buffer_rsrc_t rB = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(gB + (long long)kt * BK * p.ldb * 2), 0, RSRC_RECORDS, RSRC_FLAGS);
        const int kLeft = kLen - kt * BK;            // valid k in this tile (EDGE only)
#pragma unroll
        for (int j = 0; j < T::A_LOADS; ++j) {
            unsigned v = voffA[j];
            if (EDGE && chA[j] * 8 >= kLeft) v = OOB_OFFSET;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rA, (GE_LDS void *)(dA + (j * NW + w) * 1024), 16, v, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < T::B_LOADS; ++j) {
            unsigned v = voffB[j];
            if (EDGE && rowB[j] >= kLeft) v = OOB_OFFSET;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rB, (GE_LDS void *)(dB + (j * NW + w) * 1024), 16, v, 0, 0, 0);
        }
    };

    // ---- per-lane LDS read addresses ---------------------------------------
    // A fragment (tm, ks): row = wm*WTM + tm*32 + lane%32, chunk = 2*ks + lane/32.
    // The chunk bits sit alone in address bits 4..6, so stepping ks is an XOR.
    const int rowInWave = lane & 31;
    const unsigned aBase = (unsigned)lds_a_offset(wm * T::WTM + rowInWave, lane >> 5);
    // B fragment (tn, ks), read r in {0,1}: the 16-lane group g = lane/16 covers
    // n = tn*32 + (g%2)*16 .. +15 and k = ks*16 + (lane/32)*8 + r*4 .. +3; lane i
    // of the group addresses k row i/4, 4 columns starting at (i%4)*4, and
    // receives column i of the 4x16 block.
    const int i16 = lane & 15;
    const int kLane = (lane >> 5) * 8 + (i16 >> 2);
    const int cLane = ((lane >> 4) & 1) * 2 + ((i16 & 3) >> 1);
    const unsigned bBase = (unsigned)lds_b_offset<BN>(kLane, wn * TN * 4 + cLane) + (unsigned)(i16 & 1) * 8u;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    auto compute = [&](const GE_LDS char *cA, const GE_LDS char *cB) {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const GE_LDS char *ptr = cA + ((aBase ^ (unsigned)(ks * 32)) + (unsigned)(i * 32 * 128));
                a[i] = *(const GE_LDS bf16x8_t *)ptr;
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const GE_LDS char *ptr = cB + ((bBase ^ (unsigned)(j * 64)) + (unsigned)(ks * 16 * BN * 2));
                short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)ptr);
                short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GE_LDS short4_t *)(ptr + 4 * BN * 2));
                short8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                b[j] = __builtin_bit_cast(bf16x8_t, both);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };

    GE_LDS char *lA0 = (GE_LDS char *)sA0, *lA1 = (GE_LDS char *)sA1;
    GE_LDS char *lB0 = (GE_LDS char *)sB0, *lB1 = (GE_LDS char *)sB1;

    // ---- main loop: one barrier per K tile ---------------------------------
    // At the barrier every wave has (a) seen its own loads of tile kt land
    // (vmcnt 0) and (b) finished reading the other stage, so that stage can be
    // refilled with tile kt+1 while tile kt is consumed.
    issue(0, lA0, lB0);
    for (int kt = 0; kt < nk; kt += 2) {
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
        __syncthreads();
        if (kt + 1 < nk) issue(kt + 1, lA1, lB1);
        compute(lA0, lB0);
        if (kt + 1 < nk) {
            __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
            __syncthreads();
            if (kt + 2 < nk) issue(kt + 2, lA0, lB0);
            compute(lA1, lB1);
        }
    }

    // ---- epilogue: acc register r of lane l is row 8*(r/4) + 4*(l/32) + r%4,
    // column l%32 of its 32x32 block ------------------------------------------
    float *cBase;
    long long ldc;
    if (RAW) {
        ldc = p.N;
        cBase = p.C + (long long)tc.s * p.sliceStride + (long long)tc.b * p.M * p.N;
    } else {
        ldc = p.ldc;
        cBase = p.C + (long long)tc.b * p.strideC;
    }
    const int rowLane = m0 + wm * T::WTM + 4 * (lane >> 5);
    const int colLane = n0 + wn * T::WTN + (lane & 31);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = colLane + j * 32;
        const bool nOk = !EDGE || n < p.N;
        float bv = 0.0f;
        if (!RAW && p.bias != nullptr && nOk) bv = p.bias[n];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = rowLane + i * 32 + 8 * (r >> 2) + (r & 3);
                float v = acc[i][j][r];
                if (!RAW) v = epilogue_value<ACT>(v, p.alpha, bv);
                if (!EDGE || (nOk && m < p.M)) cBase[(long long)m * ldc + n] = v;
            }
        }
    }
}

}  // namespace ge
