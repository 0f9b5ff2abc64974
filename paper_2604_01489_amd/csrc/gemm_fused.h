// Kernels of the widened operator that are not the main kernel: a guarded GEMM for argument
// lists the direct-to-LDS kernel does not take (odd sizes, unaligned pointers, odd leading
// dimensions), with operands stored either way round, and the second pass of split-K with
// the run-time epilogue.  Every global access is predicated (Debugging guide, checklist "Edges").
// (The kernel that is not a template has internal linkage: this header is included by more than
// one translation unit.)
#pragma once
#include "ge_device.h"

namespace ge {

__device__ inline void store_as(void *base, long long index, int type, float v)
{
    if (type == DT_BF16) ((unsigned short *)base)[index] = (unsigned short)bf16_bits_rne(v);
    else ((float *)base)[index] = v;
}

// One output element of the widened operator from its fp32 product sum.
__device__ inline void fused_store(const GemmParams &p, long long b, int m, int n, float sum)
{
    const float rs = p.rowScale != nullptr ? p.rowScale[m] : 1.0f;
    const float bv = p.bias != nullptr ? p.bias[n] : 0.0f;
    const float res = p.R != nullptr ? load_as_f32(p.R, b * p.strideR + (long long)m * p.ldr + n, p.rType) : 0.0f;
    store_as(p.C, b * p.strideC + (long long)m * p.ldc + n, p.cType, fused_value(p, sum, rs, bv, res));
}

// bf16, any M, N, K, leading dimensions and 2-byte aligned pointers; A stored M x K or K x M,
// B stored K x N or N x K (p.transA / p.transB).  64x64 tile, K step 32, 4 waves (2x2) of one
// 32x32 accumulator each.  Both operands are staged with k innermost, padded to 40 elements, so
// the fragment reads are the same whatever the storage; the thread -> element map of the
// global reads follows the storage so that neighbouring threads read neighbouring addresses.
// RAW: fp32 partial sums for split-K instead of the epilogue.
template <bool RAW>
__global__ void __launch_bounds__(256)
gemm_bf16_fused_generic_kernel(const GemmParams p)
{
    constexpr int BM = 64, BN = 64, BK = 32, LD = BK + 8;
    __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LD];
    __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LD];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 1, wn = w & 1;
    const TileCoord tc = map_block(p);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;
    int kBegin = tc.s * p.kPerSlice;
    int kEnd = min(p.K, kBegin + p.kPerSlice);
    triangular_k_range(p, m0, BM, kBegin, kEnd);

    const uint16_t *A = (const uint16_t *)p.A + (long long)tc.b * p.strideA;
    const uint16_t *B = (const uint16_t *)p.B + (long long)tc.b * p.strideB;

    f32x16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

    for (int k0 = kBegin; k0 < kEnd; k0 += BK) {
#pragma unroll
        for (int i = 0; i < BM * BK / 256; ++i) {
            const int e = tid + i * 256;
            const int row = p.transA ? e % BM : e / BK, k = p.transA ? e / BM : e % BK;
            const int m = m0 + row, kk = k0 + k;
            uint16_t v = 0;
            if (m < p.M && kk < kEnd) {
                // a symmetric A given by one triangle: an element of the other triangle is its mirror image
                const bool mirror = (p.triA == TRI_SYM_LOWER && kk > m) || (p.triA == TRI_SYM_UPPER && kk < m);
                v = (p.transA != 0) != mirror ? A[(long long)kk * p.lda + m] : A[(long long)m * p.lda + kk];
            }
            sA[row * LD + k] = v;
        }
#pragma unroll
        for (int i = 0; i < BK * BN / 256; ++i) {
            const int e = tid + i * 256;
            const int col = p.transB ? e / BK : e % BN, k = p.transB ? e % BK : e / BN;
            const int n = n0 + col, kk = k0 + k;
            uint16_t v = 0;
            if (n < p.N && kk < kEnd) v = p.transB ? B[(long long)n * p.ldb + kk] : B[(long long)kk * p.ldb + n];
            sB[col * LD + k] = v;
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int kk = ks * 16 + (lane >> 5) * 8;
            bf16x8_t a = *(const bf16x8_t *)&sA[(wm * 32 + (lane & 31)) * LD + kk];
            bf16x8_t b = *(const bf16x8_t *)&sB[(wn * 32 + (lane & 31)) * LD + kk];
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }

    const int n = n0 + wn * 32 + (lane & 31);
    if (n >= p.N) return;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m >= p.M) continue;
        if (RAW)
            p.C[(long long)tc.s * p.sliceStride + (long long)tc.b * p.M * p.N + (long long)m * p.N + n] = acc[r];
        else
            fused_store(p, tc.b, m, n, acc[r]);
    }
}

// Convolution for argument lists the gathering main kernel does not take (channel counts that are
// not multiples of 32, unaligned pointers): the same implicit GEMM (rows = output positions,
// columns = output channels, k = (tap, channel)) with every element of the im2col tile fetched
// under its own bounds test.  64x64 tile, K step 32, 4 waves; B is the filter bank [Cout][K].
// RAW: fp32 partial sums of one K slice for split-K instead of the epilogue.
template <bool RAW>
__global__ void __launch_bounds__(256)
conv_bf16_generic_kernel(const GemmParams p)
{
    constexpr int BM = 64, BN = 64, BK = 32, LD = BK + 8;
    __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LD];
    __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LD];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 1, wn = w & 1;
    const TileCoord tc = map_block(p);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;
    const uint16_t *X = (const uint16_t *)p.A;
    const uint16_t *Wt = (const uint16_t *)p.B;
    const int kBegin = tc.s * p.kPerSlice;
    const int kEnd = min(p.K, kBegin + p.kPerSlice);

    // A thread fills the same k column (tid % 32) of 8 rows of the A tile, 8 rows apart, in every K
    // step: the output positions of its rows are decoded once, here, and the filter tap of its k
    // once per K step, so that an element costs two bounds tests and an address (the divisions by
    // run-time extents were most of the kernel's time on first-layer shapes).
    constexpr int ROWS = BM * BK / 256;
    const int kLane = tid % BK, rowLane = tid / BK;
    int ihBase[ROWS], iwBase[ROWS];
    long long imgBase[ROWS];                      // first position of the row's image; -1: row past M
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        const int m = m0 + rowLane + i * (256 / BK);
        const int pos = m % (p.convOH * p.convOW), img = m / (p.convOH * p.convOW);
        const int oh = pos / p.convOW, ow = pos % p.convOW;
        ihBase[i] = oh * p.convSh - p.convPh;
        iwBase[i] = ow * p.convSw - p.convPw;
        imgBase[i] = m < p.M ? (long long)img * p.convH * p.convW : -1;
    }

    f32x16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

    for (int k0 = kBegin; k0 < kEnd; k0 += BK) {
        const int kkA = k0 + kLane;
        const int tap = kkA / p.convCin, c = kkA - tap * p.convCin;
        const int kh = tap / p.convKW, kw = tap - kh * p.convKW;
        const int dIh = kh * p.convDh, dIw = kw * p.convDw;
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            const int ih = ihBase[i] + dIh, iw = iwBase[i] + dIw;
            uint16_t v = 0;
            if (imgBase[i] >= 0 && kkA < kEnd && ih >= 0 && ih < p.convH && iw >= 0 && iw < p.convW)
                v = X[(imgBase[i] + (long long)ih * p.convW + iw) * p.convCin + c];
            sA[(rowLane + i * (256 / BK)) * LD + kLane] = v;
        }
#pragma unroll
        for (int i = 0; i < BK * BN / 256; ++i) {
            const int e = tid + i * 256, col = e / BK, k = e % BK;
            const int n = n0 + col, kk = k0 + k;
            uint16_t v = 0;
            if (n < p.N && kk < kEnd) v = Wt[(long long)n * p.K + kk];
            sB[col * LD + k] = v;
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int kk = ks * 16 + (lane >> 5) * 8;
            bf16x8_t a = *(const bf16x8_t *)&sA[(wm * 32 + (lane & 31)) * LD + kk];
            bf16x8_t b = *(const bf16x8_t *)&sB[(wn * 32 + (lane & 31)) * LD + kk];
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }

    const int n = n0 + wn * 32 + (lane & 31);
    if (n >= p.N) return;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m >= p.M) continue;
        if (RAW) p.C[(long long)tc.s * p.sliceStride + (long long)m * p.N + n] = acc[r];
        else fused_store(p, 0, m, n, acc[r]);
    }
}

// Split-K second pass of the widened operator: slices added in ascending order by one thread
// per output (no atomics: bitwise repeatable), then the run-time epilogue.  W holds
// [slice][batch][M][N] fp32 partial sums.
static __global__ void __launch_bounds__(256)
splitk_reduce_fused_kernel(const GemmParams p, const float *__restrict__ W)
{
    const long long total = (long long)p.batch * p.M * p.N;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const int n = (int)(e % p.N);
        const long long bm = e / p.N;
        const int m = (int)(bm % p.M);
        const long long b = bm / p.M;
        // the slices in ascending order, eight loads in flight at a time (one by one, behind the loop's test,
        // a sum of 22 terms was a chain of 22 round trips to memory: 8.4 us for a 1 MB result)
        float s = 0.0f;
        for (int i0 = 0; i0 < p.splitK; i0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = i0 + u < p.splitK ? W[e + (long long)(i0 + u) * p.sliceStride] : 0.0f;
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        fused_store(p, b, m, n, s);
    }
}

}  // namespace ge
