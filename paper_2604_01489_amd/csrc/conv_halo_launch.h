// Launchers of the halo-staged 3 x 3 convolution kernel, one translation unit per variant (conv_halo_14_11.hip,
// conv_halo_12_12.hip) so that the variants compile side by side; conv_api.hip plans the launch and picks one.
#pragma once
#include <hip/hip_runtime.h>

#include "conv_halo_layout.h"
#include "ge_device.h"

namespace ge {

struct HaloTiles {
    int R1, g1, R2, g2;
    int tiles1;       // blocks of the first kind: images * g1 * tilesN; the rest are of the second
    int tiles2;
    int tilesN;       // Cout / 256
    int posMul;       // floor(65536 / OW) + 1: pos / OW == (pos * posMul) >> 16 for pos < 256
};

}  // namespace ge

namespace ge_host {

// row blocks of 16 positions multiplied for a tile of the first and of the second kind: 14 and 11, 12 and 12;
// fp32 or bf16 output by p.cType
void launch_conv_halo_14_11(const ge::GemmParams &p, const ge::HaloTiles &ht, hipStream_t st);
void launch_conv_halo_12_12(const ge::GemmParams &p, const ge::HaloTiles &ht, hipStream_t st);

}  // namespace ge_host
