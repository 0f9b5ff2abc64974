// fp32 GEMM for small products (a few dozen 64 x 64 tiles at most, K below 1024): on the tiled kernel
// such a product keeps a sixteenth of the chip's SIMDs busy, each with one dependent chain of
// v_mfma_f32_32x32x2_f32 as long as K / 2 (256^3: 128 instructions of 16 passes, 3.9 us before any wait).
// Here a workgroup owns one 32 x 32 tile of C and its four waves share K: wave w multiplies
// k in [w K / 4, (w + 1) K / 4), straight from global memory (operands this small sit in the L2s:
// nothing is staged, a lane fetches 16 bytes of its row of A and four elements of its column of B per
// four matrix instructions, the loads of a 64-k chunk all in flight before its first multiply and the
// next chunk's behind it), and the four partial tiles are added through LDS in wave order (bitwise
// repeatable) by wave 0, which runs the epilogue.  Four times the blocks, a quarter of the chain.
//
// The k a lane contributes to a matrix instruction is a free choice as long as A and B agree: lane l
// (row or column l % 32, half h = l / 32) takes k = 8 rho + 4 h + e for load rho, element e.
// Needs M and N multiples of 32, K a multiple of 256, A 16-byte aligned with lda a multiple of 4.
#pragma once
#include "ge_device.h"

namespace ge {

__global__ void __launch_bounds__(256)
gemm_f32_small_kernel(const GemmParams p)
{
    constexpr int CHUNK = 64, RHO = CHUNK / 8;          // k of one batch of loads per wave
    __shared__ float red[3][16][64];                    // partial tiles of waves 1..3, register-major

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int tilesN = p.tilesN, tilesM = p.tilesM;
    const int tn = blockIdx.x % tilesN, tm = (blockIdx.x / tilesN) % tilesM, b = blockIdx.x / (tilesN * tilesM);
    const int m0 = tm * 32, n0 = tn * 32;
    const int kq = p.K / 4, kBegin = w * kq;            // a multiple of CHUNK

    const float *A = (const float *)p.A + (long long)b * p.strideA + (long long)(m0 + l32) * p.lda + kBegin + 4 * h;
    const float *B = (const float *)p.B + (long long)b * p.strideB + (long long)(kBegin + 4 * h) * p.ldb + n0 + l32;

    f32x16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

    f32x4_t a[2][RHO];
    float bq[2][RHO][4];
    auto fetch = [&](int chunk, int buf) __attribute__((always_inline)) {
        const float *ap = A + chunk * CHUNK;
        const float *bp = B + (long long)chunk * CHUNK * p.ldb;
#pragma unroll
        for (int rho = 0; rho < RHO; ++rho) {
            a[buf][rho] = *(const f32x4_t *)(ap + 8 * rho);
#pragma unroll
            for (int e = 0; e < 4; ++e) bq[buf][rho][e] = bp[(long long)(8 * rho + e) * p.ldb];
        }
    };
    auto multiply = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int rho = 0; rho < RHO; ++rho)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[buf][rho][e], bq[buf][rho][e], acc, 0, 0, 0);
    };

    const int chunks = kq / CHUNK;
    fetch(0, 0);
    for (int c = 0; c < chunks; c += 2) {
        if (c + 1 < chunks) fetch(c + 1, 1);
        multiply(0);
        if (c + 1 < chunks) {
            if (c + 2 < chunks) fetch(c + 2, 0);
            multiply(1);
        }
    }

    if (w > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) red[w - 1][r][lane] = acc[r];
    }
    __syncthreads();
    if (w == 0) {
        // accumulator register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32
        const int n = n0 + l32;
        const float bv = p.bias != nullptr ? p.bias[n] : 0.0f;
        float *cBase = p.C + (long long)b * p.strideC + n;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float v = acc[r];
            v += red[0][r][lane];
            v += red[1][r][lane];
            v += red[2][r][lane];
            const int m = m0 + 8 * (r >> 2) + 4 * h + (r & 3);
            cBase[(long long)m * p.ldc] = epilogue_value_rt(v, p.alpha, bv, p.act);
        }
    }
}

}  // namespace ge
