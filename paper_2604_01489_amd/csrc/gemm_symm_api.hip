// Host side of the symmetric-operand kernel (gemm_symm.h): plan (super-tile width, workspace) and
// launches.  Called by gemm_epilogue_bf16_fused for a_structure = GE_A_SYM_LOWER / GE_A_SYM_UPPER; a
// translation unit of its own because the kernel's instantiations take minutes to compile.
#include <hip/hip_runtime.h>

#include <cstdio>

#include "../../include/gemm_epilogue.h"
#include "gemm_fused.h"
#include "gemm_symm.h"
#include "ge_host.h"

namespace ge_host {

namespace {
thread_local char g_symm_config[64];
}

// ---- symmetric A given by one triangle, few output columns: every stored element fetched once -------
SymmPlan plan_symm(const ge_fused_args_t &a)
{
    SymmPlan sp{};
    sp.fast = a.N <= 32 && a.M >= 512 && (a.M % 8) == 0 && (a.lda % 8) == 0 && !(((uintptr_t)a.A) & 15u) &&
              (long long)a.lda * 2 * ge_symm::SUB + 4096 < (1ll << 31) && opt_force_config() != FORCE_GENERIC;
    if (!sp.fast) return sp;
    sp.np = a.N <= 16 ? 16 : 32;
    // The side of the super-tiles: wider ones write fewer partial results (8 N / ST bytes per byte of A) but
    // make fewer workgroups, and what counts is the number of rounds those take on the CUs times the
    // sub-tiles of one.  Estimated cost in sub-tile loads per CU, partial results included; ties go to the
    // wider tile.  (768 with 32 columns does not fit the LDS.)
    double best = 0.0;
    for (int st : {768, 512, 256}) {
        if (st == 768 && sp.np == 32) continue;
        const long long t = ceil_div(a.M, st), blocks = t * (t + 1) / 2 * a.batch;
        const long long rounds = (blocks + kNumCU - 1) / kNumCU;
        const double ns = st / 128.0;
        const double cost = (double)rounds * ns * ns * (1.0 + 8.0 * a.N / st);
        if (best == 0.0 || cost < best) { best = cost; sp.st = st; }
    }
    sp.terms = ceil_div(a.M, sp.st);
    sp.bytes = (size_t)sp.terms * (size_t)a.batch * (size_t)a.M * (size_t)a.N * sizeof(float);
    const long long blocks = (long long)sp.terms * (sp.terms + 1) / 2;
    if (blocks > 0x7fffffffll || a.batch > 65535) sp.fast = false;
    return sp;
}

namespace {
template <int ST, int NP>
void launch_symm(const ge::SymmParams &sp, bool upper, dim3 grid, hipStream_t st)
{
    if (upper) GE_LAUNCH((ge::gemm_symm_bf16_kernel<ST, NP, true>), grid, dim3(256), 0, st, sp);
    else       GE_LAUNCH((ge::gemm_symm_bf16_kernel<ST, NP, false>), grid, dim3(256), 0, st, sp);
}

}  // namespace

// p: the launch parameters of the call as the second pass needs them (epilogue, C, sizes)
ge_status_t run_symm(const ge_fused_args_t &a, const SymmPlan &plan, GemmParams p, hipStream_t hs)
{
    void *ws = nullptr;
    ge_status_t st = acquire_workspace(plan.bytes, a.workspace, a.workspace_bytes, hs, &ws);
    if (st != GE_OK) return st;
    ge::SymmParams sp{};
    sp.A = a.A; sp.B = a.B; sp.W = (float *)ws;
    sp.M = a.M; sp.N = a.N; sp.lda = a.lda; sp.ldb = a.ldb;
    sp.transB = a.transB ? 1 : 0;
    sp.upper = a.a_structure == GE_A_SYM_UPPER ? 1 : 0;
    sp.batch = a.batch;
    sp.tiles = plan.terms;
    sp.bVec = (!a.transB && (a.N % 8) == 0 && (a.ldb % 8) == 0 && !(((uintptr_t)a.B) & 15u)) ? 1 : 0;
    sp.bytesA = 2 * (((long long)a.M - 1) * a.lda + a.M);
    const dim3 grid((unsigned)((long long)plan.terms * (plan.terms + 1) / 2), (unsigned)a.batch);
    const bool upper = sp.upper != 0;
    if (plan.st == 768) {
        launch_symm<768, 16>(sp, upper, grid, hs);
    } else if (plan.st == 512) {
        if (plan.np == 16) launch_symm<512, 16>(sp, upper, grid, hs);
        else               launch_symm<512, 32>(sp, upper, grid, hs);
    } else {
        if (plan.np == 16) launch_symm<256, 16>(sp, upper, grid, hs);
        else               launch_symm<256, 32>(sp, upper, grid, hs);
    }
    if (ge_host::take_launch_error() != hipSuccess) return GE_ERR_LAUNCH;
    // the terms are the slices of the second pass: added in their order, then the consumer chain
    p.splitK = plan.terms;
    p.sliceStride = (long long)a.batch * a.M * a.N;
    const long long total = (long long)a.batch * a.M * a.N;
    long long blocks = (total + 255) / 256;
    if (blocks > 16 * kNumCU) blocks = 16 * kNumCU;
    GE_LAUNCH(ge::splitk_reduce_fused_kernel, dim3((unsigned)blocks), dim3(256), 0, hs, p, (const float *)ws);
    if (ge_host::take_launch_error() != hipSuccess) return GE_ERR_LAUNCH;
    std::snprintf(g_symm_config, sizeof g_symm_config, "bf16_symm_%s_%dx%d_n%d", upper ? "upper" : "lower", plan.st, plan.st, plan.np);
    g_last_config = g_symm_config;
    return GE_OK;
}

}  // namespace ge_host
