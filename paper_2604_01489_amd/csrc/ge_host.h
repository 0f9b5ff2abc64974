// Host-side pieces shared by the translation units of the library: plan selection, the
// library-owned split-K workspace and the last-configuration string.  Defined in
// gemm_epilogue_api.hip.
#pragma once
#include <stddef.h>

#include "../../include/gemm_epilogue.h"
#include "ge_device.h"

namespace ge_host {

using ge::GemmParams;

constexpr int kNumCU = 256;          // MI355X

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

// ---- shape -> plan -------------------------------------------------------
enum TileKind { TILE_256 = 0, TILE_128 = 1, TILE_GENERIC = 2 };

struct Plan {
    TileKind tile;
    int bm, bn, bk;
    int tilesM, tilesN;
    int splitK;      // >= 1
    int kPerSlice;
    bool edge;
};

extern thread_local const char *g_last_config;

int choose_split(long long tiles, int K, int minSlice);
ge_status_t make_plan_bf16(int M, int N, int K, int batch, bool fast, ge_plan_t plan, int split_k, Plan *out);
size_t partial_bytes(int M, int N, int batch, int splitK);
int choose_group_m(int tilesM, int tilesN);
// The four-wave kernel (gemm_bf16_w4.h) takes launches of 256 x 256 tiles whose blocks walk a K range
// long enough for its deeper pipeline to pay; four_wave_edge names the variant: 0 full tiles, 1 tiles
// hanging over M or N, 2 also K ranges that are not multiples of 128.  GE_WAVES=8 in the environment keeps the eight-wave
// kernel, for timing and for its tests.
int four_wave_edge(const Plan &pl, int K);
bool four_wave_ok(const Plan &pl, int K);
ge_status_t acquire_workspace(size_t need, void *user, size_t user_bytes, void **out);

// The plain operator C = act(alpha A B + bias) (row-major operands, fp32 out): what the plain
// entry points call, and what the widened one calls when none of its extras is in use.
ge_status_t run_bf16(int M, int N, int K, const uint16_t *A, int lda, const uint16_t *B, int ldb,
                     const float *bias, float alpha, ge_act_t act, float *C, int ldc, int batch,
                     ge_plan_t plan, int split_k, void *workspace, size_t workspace_bytes, void *stream);

}  // namespace ge_host
