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
typedef __attribute__((ext_vector_type(4))) int i32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;

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
    int rVec;                  // a lane's 4 consecutive residual elements can be read in one piece
    // convolution front-end only: geometry of the channels-last input and of the filter
    int convH, convW, convCin, convKH, convKW, convOH, convOW;
    int convSh, convSw, convPh, convPw, convDh, convDw;
    int transA, transB;        // operand stored transposed (read by the guarded kernel; the main
                               // kernel takes them as template arguments)
    int triA;                  // TRI_LOWER / TRI_UPPER: opA(A) is promised triangular (0: nothing known)
};

// TRI_SYM_*: A is symmetric and given by that triangle of the array (the guarded kernel mirrors the
// index of an element of the other one; the main kernels do not take such calls)
enum { TRI_NONE = 0, TRI_LOWER = 1, TRI_UPPER = 2, TRI_SYM_LOWER = 3, TRI_SYM_UPPER = 4 };

// The K range of a block whose tile covers rows [m0, m0 + BM) when opA(A) is promised triangular:
// a lower-triangular A is zero for k > m, so nothing beyond k = m0 + BM - 1 contributes; an
// upper-triangular one is zero for k < m, so nothing before k = m0 does.  m0 and BM are multiples
// of every kernel's K step, so the range stays aligned to it.
__device__ inline void triangular_k_range(const GemmParams &p, int m0, int BM, int &kBegin, int &kEnd)
{
    if (p.triA == TRI_LOWER) kEnd = min(kEnd, m0 + BM);
    if (p.triA == TRI_UPPER) kBegin = max(kBegin, m0);
    if (kEnd < kBegin) kEnd = kBegin;
}

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
    if (p.triA == TRI_LOWER || p.triA == TRI_UPPER) {
        // Tiles of a triangular A differ in work by their tile row (the K range grows or shrinks
        // with it).  Walk the tiles in groups of four tile columns, every tile row of a group from
        // the longest K range to the shortest: each XCD's run of logical ids then holds the same mix
        // of long and short tiles, the long ones start first, and the tiles resident on an XCD at a
        // time still form a block of tile rows x 4 tile columns that shares panels in its L2.
        const unsigned groupN = 4u;
        const unsigned perColGroup = groupN * (unsigned)p.tilesM;
        const unsigned gc = t / perColGroup;
        const unsigned firstN = gc * groupN;
        unsigned cols = (unsigned)p.tilesN - firstN;
        if (cols > groupN) cols = groupN;
        const unsigned inc = t - gc * perColGroup;
        const unsigned r = inc / cols;
        c.tn = (int)(firstN + inc % cols);
        c.tm = p.triA == TRI_LOWER ? (int)((unsigned)p.tilesM - 1u - r) : (int)r;
        return c;
    }
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

// The coordinates of the calling block.  The divisions above run on the vector unit; the results
// are block-uniform, and pinning them to scalar registers here keeps everything derived from them
// (tile origins, operand bases, buffer resources handed to inline assembly) scalar as well.
__device__ inline TileCoord map_block(const GemmParams &p)
{
    TileCoord c = map_block(p, blockIdx.x);
    c.tm = __builtin_amdgcn_readfirstlane(c.tm);
    c.tn = __builtin_amdgcn_readfirstlane(c.tn);
    c.b = __builtin_amdgcn_readfirstlane(c.b);
    c.s = __builtin_amdgcn_readfirstlane(c.s);
    return c;
}

// gelu_tanh(v) = 0.5 v (1 + tanh u) with u = sqrt(2/pi) (v + 0.044715 v^3).
// Since 0.5 (1 + tanh u) = 1 / (1 + exp(-2u)) this is v / (1 + exp(-2u)): one
// exponential and one division, finite for every finite v (exp overflow gives
// v / inf = -0 for very negative v).  Written on the hardware's base-2 exponential with the
// constants folded, -2u log2(e) = v (K0 + K1 v^2): seven vector instructions a value (the
// epilogue of a tile is a single wave per SIMD issuing them one after the other).
__device__ inline float gelu_tanh_f32(float v)
{
    constexpr float K0 = -2.0f * 0.7978845608028654f * 1.4426950408889634f, K1 = K0 * 0.044715f;
    const float p = __builtin_fmaf(v * v, K1, K0);
    // hardware reciprocal (1 ulp) instead of an IEEE division: 1 + 2^x >= 1, or +inf -> 0
    return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * p));
}

// The same for N values, stage by stage: the hardware wants a wait state between a transcendental
// instruction and the use of its result, and one wave per SIMD has nobody else to fill it; with the N
// chains advancing together each stage's instructions follow one another and no wait state is left.
template <int N>
__device__ __forceinline__ void gelu_tanh_f32_n(float (&v)[N])
{
    constexpr float K0 = -2.0f * 0.7978845608028654f * 1.4426950408889634f, K1 = K0 * 0.044715f;
    float x[N];
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] = v[i] * v[i];
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] = __builtin_fmaf(x[i], K1, K0);
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] = v[i] * x[i];
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] = __builtin_amdgcn_exp2f(x[i]);
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] = 1.0f + x[i];
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] = __builtin_amdgcn_rcpf(x[i]);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = v[i] * x[i];
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

// scale -> bias -> activation for the N values of one row piece (acc in, result out)
template <int ACT, int N>
__device__ __forceinline__ void epilogue_values(float (&v)[N], float alpha, const float (&bias)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = alpha * v[i] + bias[i];
    if (ACT == ACT_RELU) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = v[i] > 0.0f ? v[i] : 0.0f;
    } else if (ACT == ACT_GELU_TANH) {
        gelu_tanh_f32_n<N>(v);
    }
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

__device__ inline unsigned pack_bf16_pair(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    const f32x2_t f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2_t));
}

// How a fused epilogue reads its residual.  The mode is block-uniform; the epilogues branch on it
// once, around the whole walk over the row blocks, so that inside a walk the fetches of row block
// i + 1 (row scale, residual) can be issued ahead of the arithmetic of row block i: with a fetch
// right before each use, a tile pays one round trip to L2 or HBM per row block, which a short-K
// (store-bound) shape notices and a residual doubles.
enum { RES_NONE = 0, RES_BF16 = 1, RES_F32 = 2, RES_BF16_SCALAR = 3, RES_F32_SCALAR = 4,
       RES_BF16_LDS = 5 };   // the caller has staged the tile's bf16 residual in the LDS image, where the results are parked

__device__ inline float bf16_bits_as_f32(unsigned bits16) { return __uint_as_float(bits16 << 16); }

// Activation and clamp of one row block, the activation by a uniform branch around the loops.
// relu needs no instruction of its own: clamp(max(v, 0), lo, hi) with lo <= hi is the clamp of v to
// [max(lo, 0), hi], or the constant hi where that interval is empty (hi < 0), so the bounds are
// adjusted once, on the scalar unit, and each value costs one median-of-three either way (on a
// store-bound shape the epilogue's vector instructions are time nothing else overlaps).
//
// Non-finite values follow the compare-and-select chain of fused_value (and of the CPU reference):
// relu maps NaN to 0, which is then clamped; without relu a NaN stays a NaN through the clamp.  The
// median-of-three instruction returns the smaller bound for a NaN, which is the right answer after
// relu and the wrong one otherwise: there the clamp is skipped altogether when both sides are off
// (a uniform branch), and a NaN is put back by one compare and select per value when they are not.
__device__ __forceinline__ float clamp_keep_nan(float v, float lo, float hi)
{
    const float c = __builtin_amdgcn_fmed3f(v, lo, hi);
    return v != v ? v : c;
}

// The activation and clamp of a call as a compile-time case, chosen once per tile around the whole walk
// over its row blocks.  With the choice taken inside every row block, the code of the cases not taken
// (the gelu's, most of it) lies between the row blocks: the walk jumps across more code than the
// instruction cache holds and waits for a fetch from L2 in every row block (measured on the 3 x 3
// convolution with relu: 0.6 us per row block of 16 x 64 values, 9 us per tile, against 2 us of arithmetic).
enum { CHAIN_ANY = 0, CHAIN_RELU = 1, CHAIN_LINEAR = 2, CHAIN_GELU = 3 };

__device__ __forceinline__ int chain_mode(const GemmParams &p)
{
    const bool clampOn = p.clampLo != -__builtin_inff() || p.clampHi != __builtin_inff();
    if (p.act == ACT_RELU) return CHAIN_RELU;
    if (!clampOn && p.act == ACT_NONE) return CHAIN_LINEAR;
    if (!clampOn && p.act == ACT_GELU_TANH) return CHAIN_GELU;
    return CHAIN_ANY;
}

template <int TN, int MODE = CHAIN_ANY>
__device__ __forceinline__ void act_clamp_row_block(const GemmParams &p, f32x4_t (&v)[TN])
{
    if constexpr (MODE == CHAIN_LINEAR) {
        return;
    } else if constexpr (MODE == CHAIN_GELU) {
        float t[TN * 4];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) t[j * 4 + r] = v[j][r];
        gelu_tanh_f32_n<TN * 4>(t);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) v[j][r] = t[j * 4 + r];
        return;
    } else if constexpr (MODE == CHAIN_RELU) {
        float lo = p.clampLo, hi = p.clampHi;
        lo = lo > 0.0f ? lo : 0.0f;
        lo = hi < lo ? hi : lo;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) v[j][r] = __builtin_amdgcn_fmed3f(v[j][r], lo, hi);
        return;
    }
    const bool clampOn = p.clampLo != -__builtin_inff() || p.clampHi != __builtin_inff();
    if (p.act == ACT_GELU_TANH) {
        if (clampOn) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) v[j][r] = clamp_keep_nan(gelu_tanh_f32(v[j][r]), p.clampLo, p.clampHi);
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) v[j][r] = gelu_tanh_f32(v[j][r]);
        }
    } else if (p.act == ACT_RELU) {
        float lo = p.clampLo, hi = p.clampHi;
        lo = lo > 0.0f ? lo : 0.0f;
        lo = hi < lo ? hi : lo;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) v[j][r] = __builtin_amdgcn_fmed3f(v[j][r], lo, hi);
    } else if (clampOn) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) v[j][r] = clamp_keep_nan(v[j][r], p.clampLo, p.clampHi);
    }
}

// ---- bf16 output: accumulators of the swapped product (lane: one row, 4 consecutive columns per block)

// What row block (row m of this lane) needs from memory: its row scale and, per column block, the
// lane's 4 residual elements as raw words (RES_BF16: two words of packed pairs; RES_F32: four).
template <int RES, int TN, bool EDGE>
__device__ __forceinline__ void fetch_row_block_t(const GemmParams &p, int b, int m, int colLane, float &rs, unsigned (&raw)[TN][4])
{
    const bool rowOk = !EDGE || m < p.M;
    rs = (p.rowScale != nullptr && rowOk) ? p.rowScale[m] : 1.0f;
    if constexpr (RES == RES_BF16 || RES == RES_F32) {
        const long long rowAt = (long long)b * p.strideR + (long long)m * p.ldr;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = colLane + j * 16;
            const bool inside = !EDGE || (rowOk && n < p.N);
            if constexpr (RES == RES_BF16) {
                u32x2_t t = {0u, 0u};
                if (inside) t = *(const u32x2_t *)((const unsigned short *)p.R + rowAt + n);
                raw[j][0] = t[0];
                raw[j][1] = t[1];
            } else {
                i32x4_t t = {0, 0, 0, 0};
                if (inside) t = *(const i32x4_t *)((const float *)p.R + rowAt + n);
#pragma unroll
                for (int r = 0; r < 4; ++r) raw[j][r] = (unsigned)t[r];
            }
        }
    }
}

template <int RES, int TN, bool EDGE, int MODE = CHAIN_ANY>
__device__ __forceinline__ void apply_row_block_t(const GemmParams &p, int b, f32x4_t (&v)[TN], const float (&bv)[TN][4],
                                         float rs, const unsigned (&raw)[TN][4], int m, int colLane)
{
    const float scale = p.alpha * rs;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) v[j][r] = __builtin_fmaf(v[j][r], scale, bv[j][r]);
    if constexpr (RES == RES_BF16) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            v[j][0] = __builtin_fmaf(p.beta, __uint_as_float(raw[j][0] << 16), v[j][0]);
            v[j][1] = __builtin_fmaf(p.beta, __uint_as_float(raw[j][0] & 0xFFFF0000u), v[j][1]);
            v[j][2] = __builtin_fmaf(p.beta, __uint_as_float(raw[j][1] << 16), v[j][2]);
            v[j][3] = __builtin_fmaf(p.beta, __uint_as_float(raw[j][1] & 0xFFFF0000u), v[j][3]);
        }
    } else if constexpr (RES == RES_F32) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) v[j][r] = __builtin_fmaf(p.beta, __uint_as_float(raw[j][r]), v[j][r]);
    } else if constexpr (RES == RES_BF16_SCALAR || RES == RES_F32_SCALAR) {
        // a residual whose rows cannot be read in 8- or 16-byte pieces: element by element, at the use
        const long long rowAt = (long long)b * p.strideR + (long long)m * p.ldr;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = colLane + j * 16;
            if (EDGE && (m >= p.M || n >= p.N)) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float res = RES == RES_BF16_SCALAR ? bf16_bits_as_f32(((const unsigned short *)p.R)[rowAt + n + r])
                                                         : ((const float *)p.R)[rowAt + n + r];
                v[j][r] = __builtin_fmaf(p.beta, res, v[j][r]);
            }
        }
    }
    act_clamp_row_block<TN, MODE>(p, v);
}

// The lane's bias values for the swapped product: 4 consecutive columns from colLane + 16 j per
// column block (colLane is a multiple of 4), in one piece where the pointer allows.
template <int TN, bool EDGE>
__device__ __forceinline__ void fetch_bias_t(const GemmParams &p, int colLane, float (&bv)[TN][4])
{
    const bool biasVec = (((unsigned long long)p.bias) & 15ull) == 0ull;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = colLane + j * 16;
        const bool ok = p.bias != nullptr && (!EDGE || n < p.N);
        if (biasVec) {
            f32x4_t t = {0.0f, 0.0f, 0.0f, 0.0f};
            if (ok) t = *(const f32x4_t *)(p.bias + n);
#pragma unroll
            for (int r = 0; r < 4; ++r) bv[j][r] = t[r];
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) bv[j][r] = ok ? p.bias[n + r] : 0.0f;
        }
    }
}

// The chain over all row blocks of a wave tile and the parking of the results, as bf16, in the
// row-major LDS image of the block tile.
template <int RES, int BN, int TM, int TN, bool EDGE, int MODE = CHAIN_ANY>
__device__ __forceinline__ void chain_and_park_t(const GemmParams &p, int b, f32x4_t (&acc)[TM][TN], const float (&bv)[TN][4],
                                        GE_LDS char *lds, int m0, int colLane, int tileRow, int tileCol)
{
    constexpr int PITCH = BN * 2, CHUNKS = PITCH / 16;
    // Row scale and residual of row block i + PF - 1 are fetched before the arithmetic of block i.  A block's
    // arithmetic takes a fraction of a round trip to memory, so with one block ahead every block waits for
    // its fetch (the 3 x 3 convolution with a bf16 residual: 0.4 us per row block, 5.7 us per tile).  Packed
    // bf16 pieces are two registers per column block: all of them are fetched up front where that takes at
    // most 128 registers (the fragments' registers are free by now), so that a tile pays one round trip.
    constexpr int PF = RES == RES_BF16 ? (TM * TN * 2 <= 128 ? TM + 1 : 4) : 2;
    // RES_BF16_LDS: the residual's pieces are read from the image (each by the lane that parks its result
    // there); memory is asked for the row scale only
    constexpr int RESF = RES == RES_BF16_LDS ? RES_NONE : RES, RESA = RES == RES_BF16_LDS ? RES_BF16 : RES;
    float rs[PF];
    unsigned raw[PF][TN][4];
#pragma unroll
    for (int d = 0; d < PF - 1; ++d)
        if (d < TM) fetch_row_block_t<RESF, TN, EDGE>(p, b, m0 + tileRow + d * 16, colLane, rs[d], raw[d]);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = tileRow + i * 16;
        if (i + PF - 1 < TM)
            fetch_row_block_t<RESF, TN, EDGE>(p, b, m0 + row + (PF - 1) * 16, colLane, rs[(i + PF - 1) % PF], raw[(i + PF - 1) % PF]);
        if constexpr (RES == RES_BF16_LDS) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int cb = (tileCol + j * 16) * 2;
                const u32x2_t t = *(const GE_LDS u32x2_t *)(lds + row * PITCH + (((cb >> 4) ^ (row & (CHUNKS - 1))) << 4) + (cb & 15));
                raw[i % PF][j][0] = t[0];
                raw[i % PF][j][1] = t[1];
            }
        }
        apply_row_block_t<RESA, TN, EDGE, MODE>(p, b, acc[i], bv, rs[i % PF], raw[i % PF], m0 + row, colLane);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int cb = (tileCol + j * 16) * 2;
            u32x2_t v;
            v[0] = pack_bf16_pair(acc[i][j][0], acc[i][j][1]);
            v[1] = pack_bf16_pair(acc[i][j][2], acc[i][j][3]);
            *(GE_LDS u32x2_t *)(lds + row * PITCH + (((cb >> 4) ^ (row & (CHUNKS - 1))) << 4) + (cb & 15)) = v;
        }
    }
}

// Epilogue of the widened operator with bf16 output, for a block tile whose accumulators were
// produced with the operands of the 16x16 MFMA swapped, i.e. transposed blocks: lane l of a block
// holds row l%16, register r column 4*(l/16) + r.  A lane then owns 4 consecutive columns of one
// row, which is what the chain wants (one row scale per lane, bias and residual in pieces, bf16
// conversions that pack pairs), and the tile goes to C through LDS: the waves park their values
// in a row-major image of the tile (16-byte chunks XOR-swizzled by the row, so that the 16 rows a
// write instruction touches fall in different banks), then every wave instruction moves 1 KB of
// whole rows to C with 16 bytes per lane.  Each row block runs the whole chain and is parked
// before the next one starts.  C must be able to take 16-byte row pieces (the host checks).
// `lds` must hold BM*BN*2 bytes nobody reads any more; all NW waves of the block call this.
// resInLds: the caller has copied the tile's bf16 residual into the image (same rows, same chunk swizzle) and
// waited for its own copies; the barrier below makes them visible, and each lane reads the pieces it replaces.
// (tileRow, tileCol): row of this lane and first of its 4 columns in block (0, 0) of the wave
// tile, relative to the block tile.
// NT: the row pieces leave with the non-temporal hint (C is not read back).  Measured at 8192^3 on the
// four-wave kernel: 0.826 -> 0.811 ms; on the eight-wave kernel no gain (short-K batched shape, 8192^3
// with A stored K x M) or a loss (3 x 3 convolution, 0.132 -> 0.135 ms), so only the former asks for it.
template <int BM, int BN, int NW, int LDS_BYTES, int TM, int TN, bool EDGE, bool NT = false>
__device__ __forceinline__ void fused_epilogue_bf16_through_lds(const GemmParams &p, int b, f32x4_t (&acc)[TM][TN], GE_LDS char *lds,
                                                       int m0, int n0, int tileRow, int tileCol, int w, int lane,
                                                       bool resInLds = false)
{
    constexpr int PITCH = BN * 2, CHUNKS = PITCH / 16, ROWS_PER_INSTR = 1024 / PITCH;
    static_assert(BM * PITCH <= LDS_BYTES, "bf16 image of the tile fits the stages");
    const int colLane = n0 + tileCol;
    float bv[TN][4];
    fetch_bias_t<TN, EDGE>(p, colLane, bv);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // every wave is done with the stages
    // the case of activation and clamp, then the way the residual is read, each a uniform branch around the whole walk
#define GE_PARK(RES_, MODE_) chain_and_park_t<RES_, BN, TM, TN, EDGE, MODE_>(p, b, acc, bv, lds, m0, colLane, tileRow, tileCol)
#define GE_PARK_BY_MODE(RES_)                                              \
    do {                                                                   \
        if (mode == CHAIN_RELU) GE_PARK(RES_, CHAIN_RELU);                 \
        else if (mode == CHAIN_GELU) GE_PARK(RES_, CHAIN_GELU);            \
        else if (mode == CHAIN_LINEAR) GE_PARK(RES_, CHAIN_LINEAR);        \
        else GE_PARK(RES_, CHAIN_ANY);                                     \
    } while (0)
    const int mode = chain_mode(p);
    if (p.R == nullptr) GE_PARK_BY_MODE(RES_NONE);
    else if (resInLds) GE_PARK_BY_MODE(RES_BF16_LDS);
    else if (p.rVec && p.rType == DT_BF16) GE_PARK_BY_MODE(RES_BF16);
    else if (p.rVec) GE_PARK_BY_MODE(RES_F32);
    else if (p.rType == DT_BF16) GE_PARK(RES_BF16_SCALAR, CHAIN_ANY);
    else GE_PARK(RES_F32_SCALAR, CHAIN_ANY);
#undef GE_PARK_BY_MODE
#undef GE_PARK
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    unsigned short *cBase = (unsigned short *)p.C + (long long)b * p.strideC;
    const int rowInGroup = lane / CHUNKS, chunk = lane % CHUNKS;
#pragma unroll
    for (int it = 0; it < BM / ROWS_PER_INSTR / NW; ++it) {
        const int row = (it * NW + w) * ROWS_PER_INSTR + rowInGroup;
        const i32x4_t v = *(const GE_LDS i32x4_t *)(lds + row * PITCH + ((chunk ^ (row & (CHUNKS - 1))) << 4));
        const int m = m0 + row, n = n0 + chunk * 8;
        if (!EDGE || (m < p.M && n < p.N)) {
            if (NT) __builtin_nontemporal_store(v, (i32x4_t *)(cBase + (long long)m * p.ldc + n));
            else *(i32x4_t *)(cBase + (long long)m * p.ldc + n) = v;
        }
    }
}

// ---- fp32 output: accumulators of the plain product (register r of lane l: row 4*(l/16) + r,
// column l%16 of its block)

// Row scales of the lane's 4 rows and, per row and column block, its residual element as a raw fp32 word.
template <int RES, int TN, bool EDGE>
__device__ __forceinline__ void fetch_row_block_n(const GemmParams &p, int b, int mFirst, int colLane, float (&rs)[4],
                                         unsigned (&raw)[4][TN])
{
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int m = mFirst + r;
        rs[r] = (p.rowScale != nullptr && (!EDGE || m < p.M)) ? p.rowScale[m] : 1.0f;
    }
    if constexpr (RES != RES_NONE) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = mFirst + r;
            const long long rowAt = (long long)b * p.strideR + (long long)m * p.ldr + colLane;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const bool inside = !EDGE || (m < p.M && colLane + j * 16 < p.N);
                unsigned t = 0u;
                if constexpr (RES == RES_BF16) {
                    if (inside) t = (unsigned)((const unsigned short *)p.R)[rowAt + j * 16];
                    raw[r][j] = t << 16;
                } else {
                    if (inside) t = ((const unsigned *)p.R)[rowAt + j * 16];
                    raw[r][j] = t;
                }
            }
        }
    }
}

// One row block at a time: chain, then stores, with the fetches of row block i + 1 issued ahead of
// the arithmetic of block i.  (Loads and stores share one completion counter on this hardware and
// complete out of order with respect to each other, so a fetch issued among stores is waited for
// together with them; a pass of fetches over the whole tile ahead of a pass of stores avoids that
// but made the register allocator spill the accumulators, and fetching all row scales up front
// measured slower.)
template <int RES, int TM, int TN, bool EDGE, int MODE = CHAIN_ANY>
__device__ __forceinline__ void chain_and_store_n(const GemmParams &p, int b, f32x4_t (&acc)[TM][TN], const float (&bv)[TN],
                                         int rowLane, int colLane)
{
    float *cBase = p.C + (long long)b * p.strideC;
    float rs[2][4];
    unsigned raw[2][4][TN];
    fetch_row_block_n<RES, TN, EDGE>(p, b, rowLane, colLane, rs[0], raw[0]);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        f32x4_t (&v)[TN] = acc[i];
        if (i + 1 < TM) fetch_row_block_n<RES, TN, EDGE>(p, b, rowLane + (i + 1) * 16, colLane, rs[(i + 1) & 1], raw[(i + 1) & 1]);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float scale = p.alpha * rs[i & 1][r];
#pragma unroll
            for (int j = 0; j < TN; ++j) v[j][r] = __builtin_fmaf(v[j][r], scale, bv[j]);
        }
        if constexpr (RES != RES_NONE) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int j = 0; j < TN; ++j) v[j][r] = __builtin_fmaf(p.beta, __uint_as_float(raw[i & 1][r][j]), v[j][r]);
        }
        act_clamp_row_block<TN, MODE>(p, v);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = rowLane + i * 16 + r;
            float *rowPtr = cBase + (long long)m * p.ldc + colLane;
#pragma unroll
            for (int j = 0; j < TN; ++j)
                if (!EDGE || (m < p.M && colLane + j * 16 < p.N)) rowPtr[j * 16] = v[j][r];
        }
    }
}

// Epilogue of the widened operator with fp32 output, straight from the accumulators: the chain in
// registers, then one dword per lane and row, 64 contiguous bytes per 16 lanes, as in the plain
// kernel.
template <int TM, int TN, bool EDGE>
__device__ __forceinline__ void fused_epilogue_f32_direct(const GemmParams &p, int b, f32x4_t (&acc)[TM][TN],
                                                 int rowLane, int colLane)
{
    float bv[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = colLane + j * 16;
        bv[j] = (p.bias != nullptr && (!EDGE || n < p.N)) ? p.bias[n] : 0.0f;
    }
#define GE_STORE_BY_MODE(RES_)                                                                                          \
    do {                                                                                                               \
        if (mode == CHAIN_RELU) chain_and_store_n<RES_, TM, TN, EDGE, CHAIN_RELU>(p, b, acc, bv, rowLane, colLane);     \
        else if (mode == CHAIN_GELU) chain_and_store_n<RES_, TM, TN, EDGE, CHAIN_GELU>(p, b, acc, bv, rowLane, colLane); \
        else if (mode == CHAIN_LINEAR) chain_and_store_n<RES_, TM, TN, EDGE, CHAIN_LINEAR>(p, b, acc, bv, rowLane, colLane); \
        else chain_and_store_n<RES_, TM, TN, EDGE, CHAIN_ANY>(p, b, acc, bv, rowLane, colLane);                        \
    } while (0)
    const int mode = chain_mode(p);
    if (p.R == nullptr) GE_STORE_BY_MODE(RES_NONE);
    else if (p.rType == DT_BF16) GE_STORE_BY_MODE(RES_BF16);
    else GE_STORE_BY_MODE(RES_F32);
#undef GE_STORE_BY_MODE
}

}  // namespace ge
