// The eight-wave / 128 x 128 kernels of the widened operator by output mode and operand storage: the
// templates that the gemm_fused_t*.hip units instantiate for one block tile and one edge handling each.
#pragma once
#include "gemm_bf16_fast.h"
#include "gemm_fused_launch.h"
#include "ge_host.h"

namespace ge_host {

// MODE: 0 = fp32 partial tiles (split-K), 1 = fused epilogue with fp32 output, 2 = with bf16 output
template <int BM, int BN, int WM, int WN, bool EDGE, int MODE, bool K64>
void launch_layout(const GemmParams &p, dim3 grid, hipStream_t st)
{
    constexpr int threads = WM * WN * 64;
    constexpr bool R = MODE == 0, F = MODE != 0, H = MODE == 2;
    if constexpr (K64) {        // only the layout stage_k64 names
        GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, EDGE, R, ge::ACT_NONE, false, true, F, H, false, true>), grid, dim3(threads), 0, st, p);
    } else if (p.transA) {
        if (p.transB) GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, EDGE, R, ge::ACT_NONE, true, true, F, H>), grid, dim3(threads), 0, st, p);
        else          GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, EDGE, R, ge::ACT_NONE, true, false, F, H>), grid, dim3(threads), 0, st, p);
    } else {
        if (p.transB) GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, EDGE, R, ge::ACT_NONE, false, true, F, H>), grid, dim3(threads), 0, st, p);
        else          GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, EDGE, R, ge::ACT_NONE, false, false, F, H>), grid, dim3(threads), 0, st, p);
    }
}

template <int BM, int BN, int WM, int WN, bool EDGE>
void launch_tile_mode(const GemmParams &p, bool k64, bool raw, dim3 grid, hipStream_t st)
{
    const int mode = raw ? 0 : p.cType == ge::DT_BF16 ? 2 : 1;
    if (k64) {
        if (mode == 0)      launch_layout<BM, BN, WM, WN, EDGE, 0, true>(p, grid, st);
        else if (mode == 1) launch_layout<BM, BN, WM, WN, EDGE, 1, true>(p, grid, st);
        else                launch_layout<BM, BN, WM, WN, EDGE, 2, true>(p, grid, st);
    } else {
        if (mode == 0)      launch_layout<BM, BN, WM, WN, EDGE, 0, false>(p, grid, st);
        else if (mode == 1) launch_layout<BM, BN, WM, WN, EDGE, 1, false>(p, grid, st);
        else                launch_layout<BM, BN, WM, WN, EDGE, 2, false>(p, grid, st);
    }
}


}  // namespace ge_host
