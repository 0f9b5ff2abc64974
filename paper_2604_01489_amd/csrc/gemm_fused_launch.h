// Launchers of the widened operator's tiled kernels, one translation unit per group of kernel variants
// (gemm_fused_t256.hip, gemm_fused_t256_edge.hip, gemm_fused_t128.hip, gemm_fused_t128_edge.hip,
// gemm_fused_w4_e0.hip, _e1.hip, _e2.hip) so that the variants compile side by side: in one unit the
// 87 kernels took a quarter of an hour.  gemm_fused_api.hip picks the group.
#pragma once
#include <hip/hip_runtime.h>

#include "ge_device.h"

namespace ge_host {

// 256 x 256 (eight waves) and 128 x 128 (four waves) block tiles; full tiles only or tiles that may hang
// over M, N or the K range; k64: 64 k per load phase (both operands along k).  raw: fp32 partial tiles.
void fused_tile_256_full(const ge::GemmParams &p, bool k64, bool raw, dim3 grid, hipStream_t st);
void fused_tile_256_edge(const ge::GemmParams &p, bool k64, bool raw, dim3 grid, hipStream_t st);
void fused_tile_128_full(const ge::GemmParams &p, bool k64, bool raw, dim3 grid, hipStream_t st);
void fused_tile_128_edge(const ge::GemmParams &p, bool k64, bool raw, dim3 grid, hipStream_t st);
// the four-wave kernel by edge handling: 0 full tiles, 1 tiles hanging over M or N, 2 also any K range
void fused_four_wave_e0(const ge::GemmParams &p, bool raw, dim3 grid, hipStream_t st);
void fused_four_wave_e1(const ge::GemmParams &p, bool raw, dim3 grid, hipStream_t st);
void fused_four_wave_e2(const ge::GemmParams &p, bool raw, dim3 grid, hipStream_t st);

}  // namespace ge_host
