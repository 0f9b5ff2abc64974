// Row sum of a linear layer by its collapsed form (see include/gemm_epilogue.h):
// y = alpha * A s + t with s = the sums of B over the output dimension and t = the sum of the bias.
// Three reductions over bf16 matrices with fp32 sums in a fixed order, all bound by HBM.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/gemm_epilogue.h"
#include "ge_device.h"
#include "ge_host.h"

namespace {

using namespace ge_host;

constexpr int kColChunkRows = 64;       // rows of the matrix one block of the column-sum pass adds up
constexpr int kRowWaves = 16;           // waves of a block of the row pass (one staging of v per block)
constexpr int kBlockRows = 8;           // rows a block of the wide row pass takes, all in flight at once
constexpr int kBlockCols = kRowWaves * 64 * 8;   // columns its 1024 threads cover in one sweep

// A streamed operand is read once and never again: the non-temporal hint keeps it from displacing
// anything in the caches, and on this part a read-only stream measured 7.1 TB/s with it against
// 6.3 TB/s without (sizes beyond the memory-side cache).
__device__ inline ge::i32x4_t load_stream16(const void *p) { return __builtin_nontemporal_load((const ge::i32x4_t *)p); }

__device__ inline float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(unsigned w) { return __uint_as_float(w & 0xFFFF0000u); }

// sum over the 64 lanes of a wave, the same tree every time
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// out[r] = scale * sum_c X[r,c] * v[c] + add[0]   (v == nullptr: ones; add == nullptr: 0)
// One wave per row at a time, a lane takes 8 consecutive columns per step (16 bytes of X) when
// VEC, single columns otherwise; v is staged in LDS once per block when it fits (`stage`), and a
// block of 16 waves walks rows with the stride of the grid so that the staging is paid once per many rows.
template <bool VEC>
__global__ void __launch_bounds__(kRowWaves * 64)
rows_dot_kernel(int R, int C, const uint16_t *__restrict__ X, long long ldx, const float *__restrict__ v,
                float scale, const float *__restrict__ add, float *__restrict__ out, int stage)
{
    extern __shared__ float vs[];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (stage) {
        for (int c = threadIdx.x; c < C; c += kRowWaves * 64) vs[c] = v[c];
        __syncthreads();
    }
    const float *vv = stage ? vs : v;
    const float addv = add != nullptr ? add[0] : 0.0f;
    for (long long r = (long long)blockIdx.x * kRowWaves + w; r < R; r += (long long)gridDim.x * kRowWaves) {
        const uint16_t *row = X + r * ldx;
        float acc = 0.0f;
        if (VEC) {
            const int c8 = C / 8;
#pragma unroll 4
            for (int q = lane; q < c8; q += 64) {
                const ge::i32x4_t x = *(const ge::i32x4_t *)(row + 8 * q);
                float f[8] = {bf16_lo((unsigned)x[0]), bf16_hi((unsigned)x[0]), bf16_lo((unsigned)x[1]), bf16_hi((unsigned)x[1]),
                              bf16_lo((unsigned)x[2]), bf16_hi((unsigned)x[2]), bf16_lo((unsigned)x[3]), bf16_hi((unsigned)x[3])};
                if (vv != nullptr) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(f[e], vv[8 * q + e], acc);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc += f[e];
                }
            }
            for (int c = c8 * 8 + lane; c < C; c += 64) {
                const float f = bf16_lo((unsigned)row[c]);
                acc = vv != nullptr ? __builtin_fmaf(f, vv[c], acc) : acc + f;
            }
        } else {
            for (int c = lane; c < C; c += 64) {
                const float f = bf16_lo((unsigned)row[c]);
                acc = vv != nullptr ? __builtin_fmaf(f, vv[c], acc) : acc + f;
            }
        }
        acc = wave_sum(acc);
        if (lane == 0) out[r] = __builtin_fmaf(scale, acc, addv);
    }
}

// The same for matrices whose rows can be read in 16-byte pieces (C a multiple of 8) and are at least
// 512 columns wide: a block of 1024 threads is G groups of 16/G waves, each group takes kBlockRows
// consecutive rows; a thread owns 8 consecutive columns per sweep of 8192/G columns, holds their v in
// registers and has one 16-byte load per row in flight, all issued before the first is used.  Many
// short-lived blocks that each ask for everything up front keep more of the memory system busy than few
// long-lived waves that walk their own rows: measured on an 8192 x 8192 matrix beyond the
// memory-side cache, 23 us against 33-37 us for the kernel above.  Per row: a fixed butterfly inside
// each wave, then the wave sums of its group added in wave order.
template <int G>
__global__ void __launch_bounds__(kRowWaves * 64)
rows_dot_wide_kernel(int R, int C, const uint16_t *__restrict__ X, long long ldx, const float *__restrict__ v,
                     float scale, const float *__restrict__ add, float *__restrict__ out)
{
    constexpr int WG = kRowWaves / G;               // waves of a group
    constexpr int SWEEP = WG * 64 * 8;              // columns a group covers in one sweep
    __shared__ float part[G * kBlockRows][WG];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int g = w / WG, wg = w % WG;
    const long long r0 = ((long long)blockIdx.x * G + g) * kBlockRows;
    float acc[kBlockRows];
#pragma unroll
    for (int u = 0; u < kBlockRows; ++u) acc[u] = 0.0f;
    for (int c0 = (wg * 64 + lane) * 8; c0 < C; c0 += SWEEP) {
        ge::i32x4_t x[kBlockRows];
#pragma unroll
        for (int u = 0; u < kBlockRows; ++u) {
            x[u] = ge::i32x4_t{0, 0, 0, 0};
            if (r0 + u < R) x[u] = load_stream16(X + (r0 + u) * ldx + c0);
        }
        float vv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) vv[e] = v != nullptr ? v[c0 + e] : 1.0f;
#pragma unroll
        for (int u = 0; u < kBlockRows; ++u) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[u] = __builtin_fmaf(bf16_lo((unsigned)x[u][e]), vv[2 * e], acc[u]);
                acc[u] = __builtin_fmaf(bf16_hi((unsigned)x[u][e]), vv[2 * e + 1], acc[u]);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kBlockRows; ++u) {
        const float t = wave_sum(acc[u]);
        if (lane == 0) part[g * kBlockRows + u][wg] = t;
    }
    __syncthreads();
    if (threadIdx.x < G * kBlockRows) {
        const long long r = (long long)blockIdx.x * G * kBlockRows + threadIdx.x;      // rows of a block are consecutive
        if (r < R) {
            float t = 0.0f;
#pragma unroll
            for (int k = 0; k < WG; ++k) t += part[threadIdx.x][k];
            out[r] = __builtin_fmaf(scale, t, add != nullptr ? add[0] : 0.0f);
        }
    }
}

// partial[chunk][c] = sum over the rows of chunk `chunk` (kColChunkRows rows, in row order) of X[r,c].
// A thread owns 8 consecutive columns (16 bytes per row) when VEC, one column otherwise.  The loads of
// 8 rows are issued together, ahead of their additions (left to the compiler's unrolling they went out
// one by one behind a bounds test: 50 us for 8192 x 8192 against 23 us).
template <bool VEC>
__global__ void __launch_bounds__(256)
cols_partial_kernel(int R, int C, const uint16_t *__restrict__ X, long long ldx, float *__restrict__ partial)
{
    constexpr int W = VEC ? 8 : 1, U = 8;
    const int c0 = (blockIdx.x * 256 + threadIdx.x) * W;
    if (c0 >= C) return;
    const int r0 = blockIdx.y * kColChunkRows, r1 = min(R, r0 + kColChunkRows);
    float acc[W];
#pragma unroll
    for (int e = 0; e < W; ++e) acc[e] = 0.0f;
    if (VEC && c0 + 8 <= C) {
        for (int r = r0; r < r1; r += U) {
            ge::i32x4_t x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                x[u] = ge::i32x4_t{0, 0, 0, 0};
                if (r + u < r1) x[u] = load_stream16(X + (long long)(r + u) * ldx + c0);
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[2 * e] += bf16_lo((unsigned)x[u][e]);
                    acc[2 * e + 1] += bf16_hi((unsigned)x[u][e]);
                }
        }
    } else {
        for (int r = r0; r < r1; ++r) {
            const uint16_t *row = X + (long long)r * ldx;
#pragma unroll
            for (int e = 0; e < W; ++e)
                if (c0 + e < C) acc[e] += bf16_lo((unsigned)row[c0 + e]);
        }
    }
#pragma unroll
    for (int e = 0; e < W; ++e)
        if (c0 + e < C) partial[(long long)blockIdx.y * C + c0 + e] = acc[e];
}

// sum of x[0..n) by one block: a thread adds every 256th element, then a fixed tree (x may be null: 0)
__device__ inline void block_vector_sum(int n, const float *__restrict__ x, float *__restrict__ out)
{
    __shared__ float part[4];
    float acc = 0.0f;
    if (x != nullptr)
        for (int i = threadIdx.x; i < n; i += 256) acc += x[i];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) out[0] = (part[0] + part[1]) + (part[2] + part[3]);
}

// s[c] = sum of the chunks' partial sums; the block past the last column block adds up the bias into
// s[C].  A block covers 64 columns: 16 groups of 16 threads, a thread 4 consecutive columns (16 bytes per
// load).  Group g adds chunks g, g + 16, ... in ascending order, eight loads in flight at a time, then
// the 16 sums are added in the order of g (32 groups of 8 threads: the same 5 us, a launch and a round trip).  (One thread per column over all chunks left the pass at
// the latency of a chain of dependent loads: 10 us for 2 MB; 8 groups of single columns: 6.9 us.)
constexpr int kFinishCols = 64, kFinishWays = 16;
__global__ void __launch_bounds__(256)
cols_finish_kernel(int C, int chunks, const float *__restrict__ partial, float *__restrict__ s, int nBias,
                   const float *__restrict__ bias)
{
    if (blockIdx.x == gridDim.x - 1) {
        block_vector_sum(nBias, bias, s + C);
        return;
    }
    __shared__ float part[kFinishWays][kFinishCols];
    const int g = threadIdx.x / (kFinishCols / 4), cl = (threadIdx.x % (kFinishCols / 4)) * 4;
    const int c = blockIdx.x * kFinishCols + cl;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const bool vec = (C % 4 == 0) && c + 4 <= C;          // rows of the partial sums are then 16-byte aligned
    for (int q0 = g; q0 < chunks; q0 += 8 * kFinishWays) {
        float v[8][4];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int q = q0 + u * kFinishWays;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[u][e] = 0.0f;
            if (q < chunks) {
                const float *src = partial + (long long)q * C + c;
                if (vec) {
                    const ge::f32x4_t t = *(const ge::f32x4_t *)src;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[u][e] = t[e];
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c + e < C) v[u][e] = src[e];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += v[u][e];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) part[g][cl + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < kFinishCols) {
        const int cc = blockIdx.x * kFinishCols + threadIdx.x;
        if (cc < C) {
            float t = part[0][threadIdx.x];
#pragma unroll
            for (int k = 1; k < kFinishWays; ++k) t += part[k][threadIdx.x];
            s[cc] = t;
        }
    }
}

__global__ void __launch_bounds__(256)
vector_sum_kernel(int n, const float *__restrict__ x, float *__restrict__ out)
{
    block_vector_sum(n, x, out);
}

bool vec_ok(const void *base, long long ld) { return (((uintptr_t)base) & 15u) == 0 && ld % 8 == 0; }

// The wide kernel needs rows in 16-byte pieces and enough columns to give most lanes of a wave one
// (its narrowest sweep is 512 columns); the grid's block count must fit 31 bits.
bool rows_wide(int R, int C, const void *X, long long ldx)
{
    return vec_ok(X, ldx) && C % 8 == 0 && C >= 384;
}

// rows of X times v (or ones), on `st`
void launch_rows_dot(int R, int C, const uint16_t *X, long long ldx, const float *v, float scale, const float *add,
                     float *out, hipStream_t st)
{
    if (rows_wide(R, C, X, ldx)) {
        // the narrowest sweep that covers a row, or the whole block per row
        const dim3 threads(kRowWaves * 64);
        auto blocks = [&](int G) { return dim3((unsigned)ceil_div(R, G * kBlockRows)); };
        if (C <= kBlockCols / 16)     GE_LAUNCH(rows_dot_wide_kernel<16>, blocks(16), threads, 0, st, R, C, X, ldx, v, scale, add, out);
        else if (C <= kBlockCols / 8) GE_LAUNCH(rows_dot_wide_kernel<8>, blocks(8), threads, 0, st, R, C, X, ldx, v, scale, add, out);
        else if (C <= kBlockCols / 4) GE_LAUNCH(rows_dot_wide_kernel<4>, blocks(4), threads, 0, st, R, C, X, ldx, v, scale, add, out);
        else if (C <= kBlockCols / 2) GE_LAUNCH(rows_dot_wide_kernel<2>, blocks(2), threads, 0, st, R, C, X, ldx, v, scale, add, out);
        else                          GE_LAUNCH(rows_dot_wide_kernel<1>, blocks(1), threads, 0, st, R, C, X, ldx, v, scale, add, out);
        return;
    }
    const int stage = (v != nullptr && (size_t)C * sizeof(float) <= 48 * 1024) ? 1 : 0;
    const size_t lds = stage ? (size_t)C * sizeof(float) : 0;
    long long blocks = ((long long)R + kRowWaves - 1) / kRowWaves;
    const long long cap = 2ll * kNumCU;             // two blocks of 16 waves per CU; many rows per staging of v
    if (blocks > cap) blocks = cap;
    const dim3 threads(kRowWaves * 64);
    if (vec_ok(X, ldx)) GE_LAUNCH(rows_dot_kernel<true>, dim3((unsigned)blocks), threads, lds, st, R, C, X, ldx, v, scale, add, out, stage);
    else                GE_LAUNCH(rows_dot_kernel<false>, dim3((unsigned)blocks), threads, lds, st, R, C, X, ldx, v, scale, add, out, stage);
}

}  // namespace

extern "C" size_t gemm_rowsum_params_workspace_bytes(int N, int K, int transB)
{
    if (N < 1 || K < 1 || !transB) return 0;
    return (size_t)ceil_div(N, kColChunkRows) * (size_t)K * sizeof(float);
}

extern "C" ge_status_t gemm_rowsum_params_bf16(int N, int K, const uint16_t *B, int ldb, int transB,
                                               const float *bias, float *params, void *stream)
{
    return gemm_rowsum_params_bf16_ex(N, K, B, ldb, transB, bias, params, nullptr, 0, stream);
}

extern "C" ge_status_t gemm_rowsum_params_bf16_ex(int N, int K, const uint16_t *B, int ldb, int transB,
                                                  const float *bias, float *params, void *workspace,
                                                  size_t workspace_bytes, void *stream)
{
    if (!B || !params) return GE_ERR_NULL;
    if (N < 1 || K < 1) return GE_ERR_SHAPE;
    if (ldb < (transB ? K : N)) return GE_ERR_LD;
    if (transB && ceil_div(N, kColChunkRows) > 65535) return GE_ERR_SHAPE;      // chunks ride on the grid's y axis
    if ((((uintptr_t)B) & 1u) || (((uintptr_t)params) & 3u) || (((uintptr_t)bias) & 3u)) return GE_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    if (!transB) {
        // B is K x N: s[k] is the sum of row k
        launch_rows_dot(K, N, B, ldb, nullptr, 1.0f, nullptr, params, st);
        GE_LAUNCH(vector_sum_kernel, dim3(1), dim3(256), 0, st, N, bias, params + K);
        g_last_config = "rowsum_params_rows";
    } else {
        // B is stored N x K: s[k] is the sum of column k, in two passes through the workspace
        const int chunks = ceil_div(N, kColChunkRows);
        void *ws = nullptr;
        const ge_status_t rc = acquire_workspace((size_t)chunks * (size_t)K * sizeof(float), workspace, workspace_bytes, st, &ws);
        if (rc != GE_OK) return rc;
        const bool vec = vec_ok(B, ldb);
        const dim3 grid((unsigned)ceil_div(K, 256 * (vec ? 8 : 1)), (unsigned)chunks);
        if (vec) GE_LAUNCH(cols_partial_kernel<true>, grid, dim3(256), 0, st, N, K, B, (long long)ldb, (float *)ws);
        else     GE_LAUNCH(cols_partial_kernel<false>, grid, dim3(256), 0, st, N, K, B, (long long)ldb, (float *)ws);
        GE_LAUNCH(cols_finish_kernel, dim3((unsigned)ceil_div(K, kFinishCols) + 1), dim3(256), 0, st, K, chunks, (const float *)ws,
                           params, N, bias);
        g_last_config = "rowsum_params_cols";
    }
    return ge_host::take_launch_error() == hipSuccess ? GE_OK : GE_ERR_LAUNCH;
}

extern "C" ge_status_t gemm_rowsum_bf16(int M, int K, const uint16_t *A, int lda, const float *params,
                                        float alpha, float *y, void *stream)
{
    if (!A || !params || !y) return GE_ERR_NULL;
    if (M < 1 || K < 1) return GE_ERR_SHAPE;
    if (lda < K) return GE_ERR_LD;
    if ((((uintptr_t)A) & 1u) || (((uintptr_t)params) & 3u) || (((uintptr_t)y) & 3u)) return GE_ERR_ALIGN;
    launch_rows_dot(M, K, A, lda, params, alpha, params + K, y, (hipStream_t)stream);
    g_last_config = rows_wide(M, K, A, lda) ? "rowsum_rows_wide" : vec_ok(A, lda) ? "rowsum_rows_vec8" : "rowsum_rows_generic";
    return ge_host::take_launch_error() == hipSuccess ? GE_OK : GE_ERR_LAUNCH;
}
