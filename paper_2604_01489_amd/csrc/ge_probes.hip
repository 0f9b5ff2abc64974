// Measured ceilings for the report (see include/ge_probes.h): an MFMA-only loop, a streaming store and a
// stream with a chosen mix of reads and writes.  Built into a library of its own (libge_probes.so):
// measurement aids are not part of the operator's library.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ge_probes.h"
#include "ge_host.h"

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

// Each thread and trip reads R and writes W pieces of 16 bytes; consecutive lanes touch consecutive
// pieces.  What is written depends on what was read, and with W == 0 a value that never occurs is
// tested for at the end, so the reads cannot be dropped.
template <int R, int W>
__global__ void __launch_bounds__(256) stream_mix_kernel(const i32x4_t *__restrict__ src, i32x4_t *__restrict__ dst, size_t trips,
                                                         int *sink)
{
    const size_t step = (size_t)gridDim.x * blockDim.x;
    i32x4_t keep = {0, 0, 0, 0};
    for (size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x; t < trips; t += step) {
        i32x4_t v = {1, 2, 3, 4};
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const i32x4_t x = src[(size_t)j * trips + t];
            v[0] ^= x[0]; v[1] ^= x[1]; v[2] ^= x[2]; v[3] ^= x[3];
        }
#pragma unroll
        for (int j = 0; j < W; ++j) dst[(size_t)j * trips + t] = v;
        keep[0] |= v[0] & v[1] & v[2] & v[3];
    }
    if (W == 0 && keep[0] == 0x7fffffff) sink[0] = 1;
}

template <int R, int W>
void launch_mix(const void *src, void *dst, size_t trips, int *sink, hipStream_t st)
{
    size_t blocks = (trips + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    GE_LAUNCH((stream_mix_kernel<R, W>), dim3((unsigned)blocks), dim3(256), 0, st, (const i32x4_t *)src, (i32x4_t *)dst, trips, sink);
}

}  // namespace

namespace ge_host {
thread_local hipError_t g_launch_error = hipSuccess;     // this library's own copy of the launch status
}

extern "C" ge_status_t ge_probe_stream_mix(const void *src, void *dst, size_t trips, int reads, int writes, void *stream)
{
    if ((reads > 0 && !src) || !dst) return GE_ERR_NULL;
    if ((((uintptr_t)src) & 15u) || (((uintptr_t)dst) & 15u)) return GE_ERR_ALIGN;
    if (trips == 0 || trips > ((size_t)1 << 36)) return GE_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    int *sink = (int *)dst;
    const int key = reads * 16 + writes;
    switch (key) {
    case 1 * 16 + 0: launch_mix<1, 0>(src, dst, trips, sink, st); break;
    case 2 * 16 + 0: launch_mix<2, 0>(src, dst, trips, sink, st); break;
    case 1 * 16 + 1: launch_mix<1, 1>(src, dst, trips, sink, st); break;
    case 1 * 16 + 2: launch_mix<1, 2>(src, dst, trips, sink, st); break;
    case 1 * 16 + 4: launch_mix<1, 4>(src, dst, trips, sink, st); break;
    case 1 * 16 + 8: launch_mix<1, 8>(src, dst, trips, sink, st); break;
    case 0 * 16 + 1: launch_mix<0, 1>(src, dst, trips, sink, st); break;
    default: return GE_ERR_CONFIG;
    }
    return ge_host::take_launch_error() == hipSuccess ? GE_OK : GE_ERR_LAUNCH;
}

extern "C" ge_status_t ge_probe_mfma_bf16(const void *operands, float *sink, int blocks, int iters, void *stream)
{
    if (!operands || !sink) return GE_ERR_NULL;
    if ((((uintptr_t)operands) & 15u) || (((uintptr_t)sink) & 3u)) return GE_ERR_ALIGN;
    if (blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 24)) return GE_ERR_SHAPE;
    GE_LAUNCH(mfma_loop_kernel, dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream,
                       (const i32x4_t *)operands, sink, iters);
    return ge_host::take_launch_error() == hipSuccess ? GE_OK : GE_ERR_LAUNCH;
}

extern "C" ge_status_t ge_probe_store_f32(float *dst, size_t count, float value, void *stream)
{
    if (!dst) return GE_ERR_NULL;
    if (((uintptr_t)dst) & 15u) return GE_ERR_ALIGN;
    if (count == 0 || (count & 3u)) return GE_ERR_SHAPE;
    const size_t n4 = count / 4;
    size_t blocks = (n4 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    GE_LAUNCH(store_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (f32x4_t *)dst, n4, value);
    return ge_host::take_launch_error() == hipSuccess ? GE_OK : GE_ERR_LAUNCH;
}
