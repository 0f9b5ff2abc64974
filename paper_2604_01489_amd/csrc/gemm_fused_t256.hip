// One group of kernel variants of the widened operator: 256 x 256 block tiles, full tiles (gemm_fused_launch.h).
#include "gemm_fused_tiles.h"

namespace ge_host {

void fused_tile_256_full(const ge::GemmParams &p, bool k64, bool raw, dim3 grid, hipStream_t st)
{
    launch_tile_mode<256, 256, 2, 4, false>(p, k64, raw, grid, st);
}

}  // namespace ge_host
