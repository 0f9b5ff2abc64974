// Structured operand A = diag(d): C = act(alpha * d[m] * B + bias[n]), a scaled copy of B instead
// of a GEMM whose products are almost all zero (see include/gemm_epilogue.h).  Bound by HBM.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/gemm_epilogue.h"
#include "ge_device.h"
#include "ge_host.h"

namespace {

// One lane moves 4 consecutive columns of a row: 8 bytes of B in, 16 bytes of C out, so that the
// store stream (two thirds of the traffic) is 1 KB contiguous per wave instruction.  A block owns a
// strip of 1024 columns and kDiagRows consecutive rows of the batch-by-row stack: the bias of a lane's
// columns is fetched once, the loads of all rows go out before the first is used, and no index needs a
// division per element (the earlier grid-stride loop over a flat element index spent more vector
// instructions on 64-bit divisions than the memory system could hide).  The stores carry the
// non-temporal hint: C is written once and not read back, and with whole 1 KB row pieces per
// instruction that took 8192 x 8192 from 80 to 53 us; the same hint on the loads gave the gain back.
constexpr int kDiagRows = 4;
template <int ACT>
__global__ void __launch_bounds__(256)
diag_rows_vec4_kernel(int M, int N, long long rows, int singleBatch, const float *__restrict__ d,
                      const uint16_t *__restrict__ B, int ldb, const float *__restrict__ bias, float alpha,
                      float *__restrict__ C, int ldc)
{
    const int c = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (c >= N) return;
    ge::f32x4_t bv = {0.0f, 0.0f, 0.0f, 0.0f};
    if (bias != nullptr) bv = *(const ge::f32x4_t *)(bias + c);
    const long long r0 = (long long)blockIdx.x * kDiagRows;           // row of the stack [batch][M]
    ge::u32x2_t raw[kDiagRows];
#pragma unroll
    for (int u = 0; u < kDiagRows; ++u) {
        raw[u] = ge::u32x2_t{0u, 0u};
        if (r0 + u < rows) raw[u] = *(const ge::u32x2_t *)(B + (r0 + u) * ldb + c);
    }
#pragma unroll
    for (int u = 0; u < kDiagRows; ++u) {
        const long long bm = r0 + u;
        if (bm >= rows) break;
        const int m = singleBatch ? (int)bm : (int)(bm % M);
        const float s = alpha * d[m];
        ge::f32x4_t v;
        v[0] = __uint_as_float(raw[u][0] << 16); v[1] = __uint_as_float(raw[u][0] & 0xFFFF0000u);
        v[2] = __uint_as_float(raw[u][1] << 16); v[3] = __uint_as_float(raw[u][1] & 0xFFFF0000u);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float x = __builtin_fmaf(v[r], s, bv[r]);
            if (ACT == ge::ACT_RELU) x = __builtin_fmaxf(x, 0.0f);
            if (ACT == ge::ACT_GELU_TANH) x = ge::gelu_tanh_f32(x);
            v[r] = x;
        }
        __builtin_nontemporal_store(v, (ge::f32x4_t *)(C + bm * ldc + c));
    }
}

// Any N, leading dimensions and element-aligned pointers.
__global__ void __launch_bounds__(256)
diag_rows_kernel(int M, int N, int batch, const float *__restrict__ d, const uint16_t *__restrict__ B, int ldb,
                 const float *__restrict__ bias, float alpha, int act, float *__restrict__ C, int ldc)
{
    const long long total = (long long)batch * M * N;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const int n = (int)(e % N);
        const long long bm = e / N;
        const int m = (int)(bm % M);
        const float b = __uint_as_float(((unsigned)B[bm * ldb + n]) << 16);
        C[bm * ldc + n] = ge::epilogue_value_rt(d[m] * b, alpha, bias != nullptr ? bias[n] : 0.0f, act);
    }
}

}  // namespace

extern "C" ge_status_t gemm_epilogue_diag_bf16(int M, int N, const float *d, const uint16_t *B, int ldb,
                                               const float *bias, float alpha, ge_act_t act, float *C, int ldc,
                                               int batch, void *stream)
{
    if (!d || !B || !C) return GE_ERR_NULL;
    if (M < 1 || N < 1 || batch < 1) return GE_ERR_SHAPE;
    if (ldb < N || ldc < N) return GE_ERR_LD;
    if (act != GE_ACT_NONE && act != GE_ACT_RELU && act != GE_ACT_GELU_TANH) return GE_ERR_ACT;
    if ((((uintptr_t)B) & 1u) || (((uintptr_t)C) & 3u) || (((uintptr_t)d) & 3u) || (bias && (((uintptr_t)bias) & 3u)))
        return GE_ERR_ALIGN;
    if ((long long)batch * M > (1ll << 40) / ldc || (long long)batch * M > (1ll << 40) / ldb) return GE_ERR_SHAPE;
    hipStream_t hs = (hipStream_t)stream;
    const bool vec = !((N | ldb | ldc) & 3) && !(((uintptr_t)B) & 7u) && !(((uintptr_t)C) & 15u) &&
                     !(bias && (((uintptr_t)bias) & 15u));
    if (vec) {
        const long long rows = (long long)batch * M;
        const long long rowBlocks = (rows + kDiagRows - 1) / kDiagRows, colBlocks = ((long long)N / 4 + 255) / 256;
        if (rowBlocks > 0x7fffffffll || colBlocks > 65535) return GE_ERR_SHAPE;
        const dim3 grid((unsigned)rowBlocks, (unsigned)colBlocks), block(256);
        const int single = batch == 1 ? 1 : 0;
        if (act == GE_ACT_RELU)
            GE_LAUNCH(diag_rows_vec4_kernel<ge::ACT_RELU>, grid, block, 0, hs, M, N, rows, single, d, B, ldb, bias, alpha, C, ldc);
        else if (act == GE_ACT_GELU_TANH)
            GE_LAUNCH(diag_rows_vec4_kernel<ge::ACT_GELU_TANH>, grid, block, 0, hs, M, N, rows, single, d, B, ldb, bias, alpha, C, ldc);
        else
            GE_LAUNCH(diag_rows_vec4_kernel<ge::ACT_NONE>, grid, block, 0, hs, M, N, rows, single, d, B, ldb, bias, alpha, C, ldc);
        ge_host::g_last_config = "diag_rows_vec4";
    } else {
        const long long units = (long long)batch * M * N;
        long long blocks = (units + 255) / 256;
        if (blocks > 16 * ge_host::kNumCU) blocks = 16 * ge_host::kNumCU;
        const dim3 grid((unsigned)blocks), block(256);
        GE_LAUNCH(diag_rows_kernel, grid, block, 0, hs, M, N, batch, d, B, ldb, bias, alpha, (int)act, C, ldc);
        ge_host::g_last_config = "diag_rows_generic";
    }
    return ge_host::take_launch_error() == hipSuccess ? GE_OK : GE_ERR_LAUNCH;
}
