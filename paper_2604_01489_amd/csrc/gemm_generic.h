// Guarded GEMM kernels for argument lists the fast kernels do not take (odd
// sizes, unaligned pointers, odd leading dimensions) and for fp32 operands.
// Every global access is predicated on the M/N/K remainders and stores are
// masked (Debugging guide, checklist "Edges").  Same matrix instructions and
// the same in-register epilogue as the fast path.
#pragma once
#include "ge_device.h"

namespace ge {

// ---------------------------------------------------------------------------
// bf16, any M, N, K, lda, ldb; 2-byte aligned pointers.
// 64x64 tile, K step 32, 4 waves (2x2) of one 32x32 accumulator each.
// A is staged as [m][k], B transposed as [n][k], both padded to 40 elements so
// each lane's 8 consecutive k (16 bytes) sit in distinct banks across rows.
// ---------------------------------------------------------------------------
template <bool RAW>
__global__ void __launch_bounds__(256)
gemm_bf16_generic_kernel(const GemmParams p)
{
    constexpr int BM = 64, BN = 64, BK = 32, LD = BK + 8;
    __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LD];
    __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LD];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 1, wn = w & 1;
    const TileCoord tc = map_block(p);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;
    const int kBegin = tc.s * p.kPerSlice;
    const int kEnd = min(p.K, kBegin + p.kPerSlice);

    const uint16_t *A = (const uint16_t *)p.A + (long long)tc.b * p.strideA;
    const uint16_t *B = (const uint16_t *)p.B + (long long)tc.b * p.strideB;

    f32x16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

    for (int k0 = kBegin; k0 < kEnd; k0 += BK) {
#pragma unroll
        for (int i = 0; i < BM * BK / 256; ++i) {
            const int e = tid + i * 256, row = e / BK, k = e % BK;
            const int m = m0 + row, kk = k0 + k;
            uint16_t v = 0;
            if (m < p.M && kk < kEnd) v = A[(long long)m * p.lda + kk];
            sA[row * LD + k] = v;
        }
#pragma unroll
        for (int i = 0; i < BK * BN / 256; ++i) {
            const int e = tid + i * 256, k = e / BN, col = e % BN;
            const int n = n0 + col, kk = k0 + k;
            uint16_t v = 0;
            if (n < p.N && kk < kEnd) v = B[(long long)kk * p.ldb + n];
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

    float *cBase;
    long long ldc;
    if (RAW) {
        ldc = p.N;
        cBase = p.C + (long long)tc.s * p.sliceStride + (long long)tc.b * p.M * p.N;
    } else {
        ldc = p.ldc;
        cBase = p.C + (long long)tc.b * p.strideC;
    }
    const int n = n0 + wn * 32 + (lane & 31);
    if (n < p.N) {
        const float bv = (!RAW && p.bias != nullptr) ? p.bias[n] : 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (m < p.M) {
                float v = acc[r];
                if (!RAW) v = epilogue_value_rt(v, p.alpha, bv, p.act);
                cBase[(long long)m * ldc + n] = v;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// fp32 operands, v_mfma_f32_32x32x2_f32 (true fp32 products and sums; gfx950
// has no reduced-precision fp32 matrix path, and the paper's audit forbids
// lowering operand precision anyway).  Any M, N, K, lda, ldb.
// 128x128 tile, K step 16, 4 waves (2x2), each a 2x2 grid of 32x32 blocks.
// A is staged [m][k] with an odd row pitch (17 floats) so the 32 rows a
// fragment read touches fall in 32 different banks; B is staged [k][n].
// ---------------------------------------------------------------------------
template <bool RAW>
__global__ void __launch_bounds__(256)
gemm_f32_kernel(const GemmParams p)
{
    constexpr int BM = 128, BN = 128, BK = 16, LDA_S = BK + 1, LDB_S = BN + 4;
    __shared__ float sA[BM * LDA_S];
    __shared__ __attribute__((aligned(16))) float sB[BK * LDB_S];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 1, wn = w & 1;
    const TileCoord tc = map_block(p);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;
    const int kBegin = tc.s * p.kPerSlice;
    const int kEnd = min(p.K, kBegin + p.kPerSlice);

    const float *A = (const float *)p.A + (long long)tc.b * p.strideA;
    const float *B = (const float *)p.B + (long long)tc.b * p.strideB;
    const bool vecA = ((p.lda & 3) == 0) && ((((uintptr_t)A) & 15) == 0);
    const bool vecB = ((p.ldb & 3) == 0) && ((((uintptr_t)B) & 15) == 0);

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    for (int k0 = kBegin; k0 < kEnd; k0 += BK) {
        // A tile: 128 rows x 16 k = 512 float4, two per thread.
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int e = tid + i * 256, row = e >> 2, kc = (e & 3) * 4;
            const int m = m0 + row, kk = k0 + kc;
            float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (m < p.M) {
                const float *src = A + (long long)m * p.lda + kk;
                if (vecA && kk + 4 <= kEnd) {
                    const float4 t = *(const float4 *)src;
                    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
                } else {
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        if (kk + x < kEnd) v[x] = src[x];
                }
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) sA[row * LDA_S + kc + x] = v[x];
        }
        // B tile: 16 k x 128 n = 512 float4, two per thread.
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int e = tid + i * 256, k = e >> 5, nc = (e & 31) * 4;
            const int n = n0 + nc, kk = k0 + k;
            float4 t = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (kk < kEnd) {
                const float *src = B + (long long)kk * p.ldb + n;
                if (vecB && n + 4 <= p.N) {
                    t = *(const float4 *)src;
                } else {
                    if (n + 0 < p.N) t.x = src[0];
                    if (n + 1 < p.N) t.y = src[1];
                    if (n + 2 < p.N) t.z = src[2];
                    if (n + 3 < p.N) t.w = src[3];
                }
            }
            *(float4 *)&sB[k * LDB_S + nc] = t;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            const int k = kk + (lane >> 5);
            float a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = sA[(wm * 64 + i * 32 + (lane & 31)) * LDA_S + k];
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = sB[k * LDB_S + wn * 64 + j * 32 + (lane & 31)];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    float *cBase;
    long long ldc;
    if (RAW) {
        ldc = p.N;
        cBase = p.C + (long long)tc.s * p.sliceStride + (long long)tc.b * p.M * p.N;
    } else {
        ldc = p.ldc;
        cBase = p.C + (long long)tc.b * p.strideC;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 64 + j * 32 + (lane & 31);
        if (n >= p.N) continue;
        const float bv = (!RAW && p.bias != nullptr) ? p.bias[n] : 0.0f;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m < p.M) {
                    float v = acc[i][j][r];
                    if (!RAW) v = epilogue_value_rt(v, p.alpha, bv, p.act);
                    cBase[(long long)m * ldc + n] = v;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Split-K second pass: C[b][m,n] = act(alpha * sum_{s=0}^{S-1} W[s][b][m,n] + bias[n]),
// slices added in ascending s by one thread per output: no atomics, so the
// result is bitwise repeatable (optimisation prompt, GEMM list item 7).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float *__restrict__ W, long long sliceStride, int S,
                     int M, int N, int batch, const float *__restrict__ bias,
                     float alpha, int act, float *__restrict__ C, int ldc, long long strideC)
{
    const long long total4 = (long long)batch * M * (N / 4);
    const bool vec = (N % 4 == 0) && (ldc % 4 == 0) && ((((uintptr_t)C) & 15) == 0);
    if (vec) {
        for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total4;
             e += (long long)gridDim.x * blockDim.x) {
            const int n4 = (int)(e % (N / 4));
            const long long bm = e / (N / 4);
            const int m = (int)(bm % M);
            const long long b = bm / M;
            const float *src = W + (bm * N + (long long)n4 * 4);
            float4 s = *(const float4 *)src;
            for (int i = 1; i < S; ++i) {
                const float4 t = *(const float4 *)(src + (long long)i * sliceStride);
                s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
            }
            float4 bv = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (bias != nullptr) bv = *(const float4 *)(bias + n4 * 4);
            float4 o;
            o.x = epilogue_value_rt(s.x, alpha, bv.x, act);
            o.y = epilogue_value_rt(s.y, alpha, bv.y, act);
            o.z = epilogue_value_rt(s.z, alpha, bv.z, act);
            o.w = epilogue_value_rt(s.w, alpha, bv.w, act);
            *(float4 *)(C + b * strideC + (long long)m * ldc + n4 * 4) = o;
        }
    } else {
        const long long total = (long long)batch * M * N;
        for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
             e += (long long)gridDim.x * blockDim.x) {
            const int n = (int)(e % N);
            const long long bm = e / N;
            const int m = (int)(bm % M);
            const long long b = bm / M;
            float s = W[e];
            for (int i = 1; i < S; ++i) s += W[e + (long long)i * sliceStride];
            const float bv = bias != nullptr ? bias[n] : 0.0f;
            C[b * strideC + (long long)m * ldc + n] = epilogue_value_rt(s, alpha, bv, act);
        }
    }
}

}  // namespace ge
