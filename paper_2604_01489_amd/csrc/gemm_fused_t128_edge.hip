// One group of kernel variants of the widened operator: 128 x 128 block tiles, tiles that may hang over M, N or the K range (gemm_fused_launch.h).
#include "gemm_fused_tiles.h"

namespace ge_host {

void fused_tile_128_edge(const ge::GemmParams &p, bool k64, bool raw, dim3 grid, hipStream_t st)
{
    launch_tile_mode<128, 128, 2, 2, true>(p, k64, raw, grid, st);
}

}  // namespace ge_host
