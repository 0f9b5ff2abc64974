// Device-side pieces shared by the gfx950 GEMM kernels: launch parameters, the
// block-id -> tile map and the in-register epilogue.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ge {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(8))) short short8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

#define GE_LDS __attribute__((address_space(3)))

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU_TANH = 2 };
enum { DT_F32 = 0, DT_BF16 = 1 };

// One launch of a GEMM kernel.  Pointers are device pointers; leading dimensions
// and strides are in elements.  When `raw` output is selected (split-K partials)
// C points at the workspace, ldc == N and sliceStride separates the K slices.
struct GemmParams {
    const void *A;
    const void *B;
    const float *bias;
    float *C;
    int M, N, K;
    int lda, ldb, ldc;
    long long strideA, strideB, strideC;  // per batch
    long long sliceStride;                // per K slice (raw output only)
    int batch;
    int splitK;      // number of K slices (1 = none)
    int kPerSlice;   // K extent of one slice, a multiple of the kernel's BK
    int tilesM, tilesN;
    int groupM;      // tile rows swept together (L2 reuse of the B panels)
    float alpha;
    int act;
    long long bytesA, bytesB;  // extent of the A and B allocations as the arguments describe them
    // The widened operator only (run-time epilogue); the plain entry points leave these zero.
    // C then points at fp32 or bf16 elements according to cType.
    const float *rowScale;     // [M] or null
    const void *R;             // residual [batch][M][ldr] of rType, or null
    long long strideR;
    int ldr, rType;
    float beta;
    float clampLo, clampHi;
    int cType;
    int transA, transB;        // operand stored transposed (read by the guarded kernel; the main
                               // kernel takes them as template arguments)
};

struct TileCoord {
    int tm, tn, b, s;
};

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Give
// every XCD a contiguous run of logical tile ids, then walk a problem's tiles
// in groups of `groupM` tile rows so that the tiles resident on one XCD at a
// time share A and B panels in that XCD's L2.  Logical order, innermost first:
// tile within problem, batch, K slice.
__device__ inline TileCoord map_block(const GemmParams &p, unsigned bid)
{
    const unsigned total = gridDim.x;
    const unsigned q = total / 8u, rem = total % 8u, xcd = bid % 8u;
    unsigned L = xcd * q + (xcd < rem ? xcd : rem) + bid / 8u;
    const unsigned tiles = (unsigned)(p.tilesM * p.tilesN);
    unsigned t = L % tiles;
    unsigned rest = L / tiles;
    TileCoord c;
    c.b = (int)(rest % (unsigned)p.batch);
    c.s = (int)(rest / (unsigned)p.batch);
    const unsigned perGroup = (unsigned)(p.groupM * p.tilesN);
    const unsigned g = t / perGroup;
    const unsigned first = g * (unsigned)p.groupM;
    unsigned rows = (unsigned)p.tilesM - first;
    if (rows > (unsigned)p.groupM) rows = (unsigned)p.groupM;
    const unsigned in = t - g * perGroup;
    c.tm = (int)(first + in % rows);
    c.tn = (int)(in / rows);
    return c;
}

__device__ inline TileCoord map_block(const GemmParams &p) { return map_block(p, blockIdx.x); }

// gelu_tanh(v) = 0.5 v (1 + tanh u) with u = sqrt(2/pi) (v + 0.044715 v^3).
// Since 0.5 (1 + tanh u) = 1 / (1 + exp(-2u)) this is v / (1 + exp(-2u)): one
// exponential and one division, finite for every finite v (exp overflow gives
// v / inf = -0 for very negative v).
__device__ inline float gelu_tanh_f32(float v)
{
    const float c2 = 2.0f * 0.7978845608028654f;
    float u2 = c2 * (v + 0.044715f * v * v * v);
    // hardware reciprocal (1 ulp) instead of an IEEE division: 1 + exp(-2u) >= 1, or +inf -> 0
    return v * __builtin_amdgcn_rcpf(1.0f + __expf(-u2));
}

// scale -> bias -> activation, fp32, in registers.
template <int ACT>
__device__ inline float epilogue_value(float acc, float alpha, float bias)
{
    float v = alpha * acc + bias;
    if (ACT == ACT_RELU) return v > 0.0f ? v : 0.0f;
    if (ACT == ACT_GELU_TANH) return gelu_tanh_f32(v);
    return v;
}

__device__ inline float epilogue_value_rt(float acc, float alpha, float bias, int act)
{
    if (act == ACT_RELU) return epilogue_value<ACT_RELU>(acc, alpha, bias);
    if (act == ACT_GELU_TANH) return epilogue_value<ACT_GELU_TANH>(acc, alpha, bias);
    return epilogue_value<ACT_NONE>(acc, alpha, bias);
}

// Nearest-even bf16 of an fp32 value, as its 16-bit pattern (the hardware conversion of gfx950).
__device__ inline unsigned bf16_bits_rne(float v)
{
    const __bf16 h = (__bf16)v;
    return (unsigned)__builtin_bit_cast(unsigned short, h);
}

__device__ inline float load_as_f32(const void *base, long long index, int type)
{
    if (type == DT_BF16) return __uint_as_float(((unsigned)((const unsigned short *)base)[index]) << 16);
    return ((const float *)base)[index];
}

// Run-time epilogue chain on one value: scale, row scale, bias, residual, activation, clamp.
__device__ inline float fused_value(const GemmParams &p, float acc, float rowScale, float bias, float res)
{
    float v = p.alpha * acc;
    v = rowScale * v;
    v = v + bias;
    v = v + p.beta * res;
    if (p.act == ACT_RELU) v = v > 0.0f ? v : 0.0f;
    else if (p.act == ACT_GELU_TANH) v = gelu_tanh_f32(v);
    v = v < p.clampLo ? p.clampLo : v;
    v = v > p.clampHi ? p.clampHi : v;
    return v;
}

// Epilogue of the widened operator for a wave tile held as TM x TN accumulators of the 16x16 MFMA
// (register r of lane l: row 4*(l/16) + r, column l%16 of its block).  rowLane / colLane are the
// global row of register 0 and the global column of this lane in block (0, 0).
// fp32 output: one dword per lane and row, 64 contiguous bytes per 16 lanes.
// bf16 output: neighbouring lanes first trade two of their four rows, so that an even lane holds
// columns (c, c+1) of rows 0 and 1 and its odd neighbour those of rows 2 and 3, and each stores
// packed pairs (4 bytes): half the store instructions, 32 contiguous bytes per 8 lanes.
template <int TM, int TN, bool EDGE>
__device__ inline void fused_epilogue_16x16(const GemmParams &p, int b, f32x4_t (&acc)[TM][TN],
                                            int rowLane, int colLane, int lane)
{
    float bv[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = colLane + j * 16;
        bv[j] = (p.bias != nullptr && (!EDGE || n < p.N)) ? p.bias[n] : 0.0f;
    }
    const bool hasR = p.R != nullptr;
    const long long rBase = (long long)b * p.strideR;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = rowLane + i * 16 + r;
            const bool rowOk = !EDGE || m < p.M;
            const float rs = (p.rowScale != nullptr && rowOk) ? p.rowScale[m] : 1.0f;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = colLane + j * 16;
                const bool ok = rowOk && (!EDGE || n < p.N);
                float res = 0.0f;
                if (hasR && ok) res = load_as_f32(p.R, rBase + (long long)m * p.ldr + n, p.rType);
                acc[i][j][r] = fused_value(p, acc[i][j][r], rs, bv[j], res);
            }
        }
    if (p.cType == DT_F32) {
        float *cBase = p.C + (long long)b * p.strideC;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = rowLane + i * 16 + r;
                float *rowPtr = cBase + (long long)m * p.ldc + colLane;
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (!EDGE || (m < p.M && colLane + j * 16 < p.N)) rowPtr[j * 16] = acc[i][j][r];
            }
    } else {
        unsigned short *cBase = (unsigned short *)p.C + (long long)b * p.strideC;
        const bool odd = lane & 1;
        const int colPair = colLane & ~1;            // first column of this lane's pair in block 0
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mPair = rowLane + i * 16 + (odd ? 2 : 0);
#pragma unroll
            for (int h = 0; h < 2; ++h) {            // the lane's two rows: mPair + h
                const int m = mPair + h;
                unsigned short *rowPtr = cBase + (long long)m * p.ldc + colPair;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    // give away row h of the other pair, receive the neighbour's value of my row
                    const float send = odd ? acc[i][j][h] : acc[i][j][2 + h];
                    const float got = __builtin_bit_cast(
                        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));
                    const float mine = odd ? acc[i][j][2 + h] : acc[i][j][h];
                    const float left = odd ? got : mine, right = odd ? mine : got;
                    const unsigned packed = bf16_bits_rne(left) | (bf16_bits_rne(right) << 16);
                    if (!EDGE || (m < p.M && colPair + j * 16 < p.N)) *(unsigned *)(rowPtr + j * 16) = packed;
                }
            }
        }
    }
}

}  // namespace ge
