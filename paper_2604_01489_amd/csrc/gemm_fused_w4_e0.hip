// One group of kernel variants of the widened operator: the four-wave kernel, edge handling 0 (gemm_fused_launch.h).
#include "gemm_fused_w4_launch.h"

namespace ge_host {

void fused_four_wave_e0(const ge::GemmParams &p, bool raw, dim3 grid, hipStream_t st) { launch_four_wave<0>(p, raw, grid, st); }

}  // namespace ge_host
