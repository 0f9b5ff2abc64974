// Measured ceilings for the report (see include/ge_probes.h): an MFMA-only loop and a streaming store.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ge_probes.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) int i32x4_t;

// 4 A and 4 B fragments per lane from the caller's values, 16 accumulators: the register
// footprint and operand reuse of one K step of a 64 x 64 wave tile, with no memory traffic.
__global__ void __launch_bounds__(512) mfma_loop_kernel(const i32x4_t *operands, float *sink, int iters)
{
    bf16x8_t a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = __builtin_bit_cast(bf16x8_t, operands[threadIdx.x * 8 + i]);
        b[i] = __builtin_bit_cast(bf16x8_t, operands[threadIdx.x * 8 + 4 + i]);
    }
    f32x4_t acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[j][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) s += acc[j][r];
    sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

__global__ void __launch_bounds__(256) store_kernel(f32x4_t *dst, size_t n4, float value)
{
    const f32x4_t v = {value, value, value, value};
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += step) dst[i] = v;
}

}  // namespace

extern "C" ge_status_t ge_probe_mfma_bf16(const void *operands, float *sink, int blocks, int iters, void *stream)
{
    if (!operands || !sink) return GE_ERR_NULL;
    if ((((uintptr_t)operands) & 15u) || (((uintptr_t)sink) & 3u)) return GE_ERR_ALIGN;
    if (blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 24)) return GE_ERR_SHAPE;
    hipLaunchKernelGGL(mfma_loop_kernel, dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream,
                       (const i32x4_t *)operands, sink, iters);
    return hipGetLastError() == hipSuccess ? GE_OK : GE_ERR_LAUNCH;
}

extern "C" ge_status_t ge_probe_store_f32(float *dst, size_t count, float value, void *stream)
{
    if (!dst) return GE_ERR_NULL;
    if (((uintptr_t)dst) & 15u) return GE_ERR_ALIGN;
    if (count == 0 || (count & 3u)) return GE_ERR_SHAPE;
    const size_t n4 = count / 4;
    size_t blocks = (n4 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(store_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (f32x4_t *)dst, n4, value);
    return hipGetLastError() == hipSuccess ? GE_OK : GE_ERR_LAUNCH;
}
