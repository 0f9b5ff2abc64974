// Host-side pieces shared by the translation units of the library: plan selection, the
// library-owned split-K workspace and the last-configuration string.  Defined in
// gemm_epilogue_api.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

#include <tuple>
#include <utility>

#include "../../include/gemm_epilogue.h"
#include "ge_device.h"

namespace ge_host {

using ge::GemmParams;

constexpr int kNumCU = 256;          // MI355X

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

// ---- shape -> plan -------------------------------------------------------
enum TileKind { TILE_256 = 0, TILE_128 = 1, TILE_GENERIC = 2, TILE_SKINNY = 3 };

struct Plan {
    TileKind tile;
    int bm, bn, bk;
    int tilesM, tilesN;
    int splitK;      // >= 1
    int kPerSlice;
    bool edge;
};

extern thread_local const char *g_last_config;

// ---- launches ------------------------------------------------------------
// A launch whose result is the launch's own: hipLaunchKernel returns it directly, so neither a
// stale error somebody else left in the runtime's per-thread slot is reported as ours, nor is it
// cleared on their behalf.  GE_LAUNCH(kernel, grid, block, ldsBytes, stream, args...) records the
// first failure of the calling thread; take_launch_error() returns and clears it.
extern thread_local hipError_t g_launch_error;

template <typename... KArgs, typename Tuple, size_t... I>
inline hipError_t launch_packed(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st, Tuple &vals,
                                std::index_sequence<I...>)
{
    void *ptrs[] = {(void *)&std::get<I>(vals)...};
    return hipLaunchKernel((const void *)kernel, grid, block, ptrs, lds, st);
}

template <typename... KArgs, typename... Args>
inline void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<KArgs...> vals{static_cast<KArgs>(args)...};
    const hipError_t err = launch_packed(kernel, grid, block, lds, st, vals, std::index_sequence_for<KArgs...>{});
    if (g_launch_error == hipSuccess) g_launch_error = err;
}

inline hipError_t take_launch_error()
{
    const hipError_t err = g_launch_error;
    g_launch_error = hipSuccess;
    return err;
}

#define GE_LAUNCH(...) ::ge_host::launch(__VA_ARGS__)

// ---- switches for timing runs and tests (ge_set_option in the header) ------
enum { FORCE_NONE = 0, FORCE_256 = 1, FORCE_128 = 2, FORCE_GENERIC = 3 };
int opt_force_config();   // FORCE_*
bool opt_eight_waves();   // keep full 256 x 256 tiles on the eight-wave kernel
bool opt_stage_k32();     // no 64-k load phases in the eight-wave kernel
// the halo-staged 3 x 3 convolution kernel: by the plan's rule, never, whenever the shape allows it, or
// one of its variants whenever the shape allows that one (HALO_VARIANT0 + index)
enum { HALO_AUTO = 0, HALO_OFF = 1, HALO_ON = 2, HALO_VARIANT0 = 3 };
int opt_conv_halo();

int choose_split(long long tiles, int K, int minSlice);
// skinny: the caller can launch the tall-skinny kernel (the plain operator only), so the plan may name it
ge_status_t make_plan_bf16(int M, int N, int K, int batch, bool fast, ge_plan_t plan, int split_k, Plan *out,
                           bool skinny = false);
size_t partial_bytes(int M, int N, int batch, int splitK);
int choose_group_m(int tilesM, int tilesN);
// The four-wave kernel (gemm_bf16_w4.h) takes launches of 256 x 256 tiles whose blocks walk a K range
// long enough for its deeper pipeline to pay; four_wave_edge names the variant: 0 full tiles, 1 tiles
// hanging over M or N, 2 also K ranges that are not multiples of 128.  The option "waves" = "8" keeps the eight-wave
// kernel, for timing and for its tests.
int four_wave_edge(const Plan &pl, int K);
bool four_wave_ok(const Plan &pl, int K);
// The buffer for `need` bytes of partial results of a call on `stream`: the caller's, if it gave one
// (checked for size and alignment), else the library's buffer for (current device, stream), grown by
// hipMalloc when a larger one is first needed -- never while the stream is capturing (GE_ERR_WORKSPACE)
// and never by freeing what an earlier call was handed (outgrown buffers are kept until
// ge_release_workspace).
ge_status_t acquire_workspace(size_t need, void *user, size_t user_bytes, hipStream_t stream, void **out);

// A symmetric A given by one triangle with few output columns (gemm_symm_api.hip): whether the kernel
// that fetches every stored element once takes the call, with which super-tile width, and the bytes
// of its partial results; run_symm launches it and the second pass (p: the call's launch parameters).
struct SymmPlan {
    bool fast;
    int st, np, terms;
    size_t bytes;
};
SymmPlan plan_symm(const ge_fused_args_t &a);
ge_status_t run_symm(const ge_fused_args_t &a, const SymmPlan &plan, GemmParams p, hipStream_t hs);

// The plain operator C = act(alpha A B + bias) (row-major operands, fp32 out): what the plain
// entry points call, and what the widened one calls when none of its extras is in use.
ge_status_t run_bf16(int M, int N, int K, const uint16_t *A, int lda, const uint16_t *B, int ldb,
                     const float *bias, float alpha, ge_act_t act, float *C, int ldc, int batch,
                     ge_plan_t plan, int split_k, void *workspace, size_t workspace_bytes, void *stream);

}  // namespace ge_host
