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

}  // namespace ge
