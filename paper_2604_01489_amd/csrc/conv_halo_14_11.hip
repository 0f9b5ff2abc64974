// One variant of the halo-staged 3 x 3 convolution kernel: 14 and 11 row blocks per tile (conv_halo_launch.h).
#include "conv_halo.h"
#include "ge_host.h"

namespace ge_host {

void launch_conv_halo_14_11(const ge::GemmParams &p, const ge::HaloTiles &ht, hipStream_t st)
{
    const dim3 grid((unsigned)(ht.tiles1 + ht.tiles2));
    if (p.cType == ge::DT_BF16) GE_LAUNCH((ge::conv_halo_bf16_kernel<14, 11, true>), grid, dim3(256), 0, st, p, ht);
    else GE_LAUNCH((ge::conv_halo_bf16_kernel<14, 11, false>), grid, dim3(256), 0, st, p, ht);
}

}  // namespace ge_host
