// The four-wave kernel of the widened operator by output mode and operand storage: the templates that
// the gemm_fused_w4_e*.hip units instantiate for one edge handling each.
#pragma once
#include "gemm_bf16_w4.h"
#include "gemm_fused_launch.h"
#include "ge_host.h"

namespace ge_host {

template <int EDGE, int MODE>
void launch_four_wave_layout(const GemmParams &p, dim3 grid, hipStream_t st)
{
    constexpr bool R = MODE == 0, F = MODE != 0, H = MODE == 2;
    if (p.transA) {         // with B along k; the caller keeps the other storage of B on the eight-wave kernel
        GE_LAUNCH((ge::gemm_bf16_w4_kernel<EDGE, R, ge::ACT_NONE, true, true, F, H>), grid, dim3(256), 0, st, p);
    } else {
        if (p.transB) GE_LAUNCH((ge::gemm_bf16_w4_kernel<EDGE, R, ge::ACT_NONE, false, true, F, H>), grid, dim3(256), 0, st, p);
        else          GE_LAUNCH((ge::gemm_bf16_w4_kernel<EDGE, R, ge::ACT_NONE, false, false, F, H>), grid, dim3(256), 0, st, p);
    }
}

template <int EDGE>
void launch_four_wave(const GemmParams &p, bool raw, dim3 grid, hipStream_t st)
{
    if (raw) launch_four_wave_layout<EDGE, 0>(p, grid, st);
    else if (p.cType == ge::DT_BF16) launch_four_wave_layout<EDGE, 2>(p, grid, st);
    else launch_four_wave_layout<EDGE, 1>(p, grid, st);
}


}  // namespace ge_host
