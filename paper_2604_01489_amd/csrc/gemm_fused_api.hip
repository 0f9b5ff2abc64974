// C-ABI of the widened operator (operands stored either way round, row scale, residual, clamp,
// fp32 or bf16 output): validation, plan selection and kernel launches.  See
// include/gemm_epilogue.h for the contract.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>

#include "../../include/gemm_epilogue.h"
#include "gemm_fused.h"
#include "gemm_fused_launch.h"
#include "ge_host.h"

namespace {

using ge::GemmParams;
using namespace ge_host;

const char *kLayoutName[4] = {"nn", "nt", "tn", "tt"};
thread_local char g_config_buf[96];

void set_config(const char *kernel, int transA, int transB, bool splitk)
{
    std::snprintf(g_config_buf, sizeof g_config_buf, "bf16_fused_%s_%s%s", kernel,
                  kLayoutName[(transA ? 2 : 0) + (transB ? 1 : 0)], splitk ? "_splitk" : "");
    g_last_config = g_config_buf;
}

bool is_symmetric(const ge_fused_args_t &a) { return a.a_structure == GE_A_SYM_LOWER || a.a_structure == GE_A_SYM_UPPER; }

ge_status_t validate(const ge_fused_args_t &a)
{
    if (!a.A || !a.B || !a.C) return GE_ERR_NULL;
    if (a.M < 1 || a.N < 1 || a.K < 1 || a.batch < 1) return GE_ERR_SHAPE;
    if (a.lda < (a.transA ? a.M : a.K) || a.ldb < (a.transB ? a.K : a.N) || a.ldc < a.N) return GE_ERR_LD;
    if (a.R && a.ldr < a.N) return GE_ERR_LD;
    if (a.act != GE_ACT_NONE && a.act != GE_ACT_RELU && a.act != GE_ACT_GELU_TANH) return GE_ERR_ACT;
    if (a.c_type != GE_DTYPE_F32 && a.c_type != GE_DTYPE_BF16) return GE_ERR_EPILOGUE;
    if (a.a_structure < GE_A_GENERAL || a.a_structure > GE_A_SYM_UPPER) return GE_ERR_CONFIG;
    if ((a.a_structure == GE_A_LOWER || a.a_structure == GE_A_UPPER) && a.plan == GE_PLAN_SPLITK) return GE_ERR_CONFIG;
    if (is_symmetric(a) && a.transA) return GE_ERR_CONFIG;
    if (is_symmetric(a) && a.M != a.K) return GE_ERR_SHAPE;
    if (a.R && a.r_type != GE_DTYPE_F32 && a.r_type != GE_DTYPE_BF16) return GE_ERR_EPILOGUE;
    if (!(a.clamp_lo <= a.clamp_hi)) return GE_ERR_EPILOGUE;
    const uintptr_t cMask = a.c_type == GE_DTYPE_F32 ? 3u : 1u, rMask = a.r_type == GE_DTYPE_F32 ? 3u : 1u;
    if ((((uintptr_t)a.A) & 1u) || (((uintptr_t)a.B) & 1u) || (((uintptr_t)a.C) & cMask)) return GE_ERR_ALIGN;
    if (a.R && (((uintptr_t)a.R) & rMask)) return GE_ERR_ALIGN;
    if ((a.bias && (((uintptr_t)a.bias) & 3u)) || (a.row_scale && (((uintptr_t)a.row_scale) & 3u))) return GE_ERR_ALIGN;
    // element counts of one operand / result must fit 63 bits with room to spare
    const long long big = 1ll << 40;
    if ((long long)a.batch * a.M > big / a.ldc || (long long)a.batch * (a.transA ? a.K : a.M) > big / a.lda ||
        (long long)a.batch * (a.transB ? a.N : a.K) > big / a.ldb)
        return GE_ERR_SHAPE;
    return GE_OK;
}

// The direct-to-LDS kernel moves 16-byte chunks along an operand's rows: they must be aligned
// and must not straddle the end of a row's payload.
bool fast_ok(const ge_fused_args_t &a)
{
    if ((((uintptr_t)a.A) | ((uintptr_t)a.B)) & 15u) return false;
    if ((a.lda | a.ldb) & 7) return false;
    if ((a.transA ? a.M : a.K) & 7) return false;
    if ((a.K | a.N) & 7) return false;            // B's row payload; N also for the 16-byte pieces of a bf16 C
    // bf16 output leaves the kernel in 16-byte row pieces
    if (a.c_type == GE_DTYPE_BF16 && ((((uintptr_t)a.C) & 15u) || (a.ldc & 7))) return false;
    // per-lane byte offsets inside one tile panel must stay below 2^31
    const long long rowsA = a.transA ? 32 : 256, rowsB = a.transB ? 256 : 32;
    if ((long long)a.lda * 2 * rowsA + 1024 >= (1ll << 31)) return false;
    if ((long long)a.ldb * 2 * rowsB + 1024 >= (1ll << 31)) return false;
    return true;
}

// 64 k per load phase (see the kernel) where both operands' rows run along k: measured at 8192^3
// with bf16 output, 0.85 -> 0.81 ms for that layout and 0.75 -> 0.81 ms for each of the other three,
// whose k-strided operands are fetched in whole lines anyway and only lose the deeper ring.
// The option "stage_k" = "32" switches it off, for timing.
bool stage_k64(bool transA, bool transB)
{
    if (opt_stage_k32()) return false;
    return !transA && transB;
}

// A 64-k stage needs the K range of every block to be a multiple of 64, or the edge variant.
template <int BM>
bool launch_tile(const GemmParams &p, bool edge, bool raw, dim3 grid, hipStream_t st)
{
    // 128 x 128 blocks: only where more than one block shares a CU (measured with both operands along
    // k, bf16 out: 4096x2048x2048, 512 blocks, 33 us with 64 k per load phase against 44 us with 32;
    // 2048^3, 256 blocks, 27 against 22 us; 2048x2048x8192 81 against 66 us)
    const bool k64 = stage_k64(p.transA != 0, p.transB != 0) && (BM == 256 || grid.x > (unsigned)kNumCU);
    if (k64) edge = edge || (p.K % 64) || (p.kPerSlice % 64);
    if (BM == 256) { if (edge) fused_tile_256_edge(p, k64, raw, grid, st); else fused_tile_256_full(p, k64, raw, grid, st); }
    else           { if (edge) fused_tile_128_edge(p, k64, raw, grid, st); else fused_tile_128_full(p, k64, raw, grid, st); }
    return k64;
}

}  // namespace

extern "C" size_t gemm_epilogue_fused_workspace_bytes(const ge_fused_args_t *args)
{
    if (!args || validate(*args) != GE_OK) return 0;
    const ge_fused_args_t &a = *args;
    if (is_symmetric(a)) {
        const SymmPlan sp = plan_symm(a);
        if (sp.fast) return sp.bytes;
    }
    Plan pl;
    const bool triangular = a.a_structure == GE_A_LOWER || a.a_structure == GE_A_UPPER;
    const bool fast = fast_ok(a) && !is_symmetric(a);
    if (make_plan_bf16(a.M, a.N, a.K, a.batch, fast, triangular ? GE_PLAN_DIRECT : a.plan, a.split_k, &pl) != GE_OK) return 0;
    return partial_bytes(a.M, a.N, a.batch, pl.splitK);
}

extern "C" ge_status_t gemm_epilogue_bf16_fused(const ge_fused_args_t *args, void *stream)
{
    if (!args) return GE_ERR_NULL;
    const ge_fused_args_t &a = *args;
    ge_status_t st = validate(a);
    if (st != GE_OK) return st;
    // nothing but scale, bias and activation on row-major operands with fp32 output: the plain
    // operator, whose kernels carry the activation as a compile-time choice
    if (!a.transA && !a.transB && !a.row_scale && !a.R && a.c_type == GE_DTYPE_F32 && std::isinf(a.clamp_lo) &&
        a.clamp_lo < 0 && std::isinf(a.clamp_hi) && a.clamp_hi > 0 && a.a_structure == GE_A_GENERAL)
        return run_bf16(a.M, a.N, a.K, a.A, a.lda, a.B, a.ldb, a.bias, a.alpha, a.act, (float *)a.C, a.ldc, a.batch, a.plan,
                        a.split_k, a.workspace, a.workspace_bytes, stream);
    Plan pl;
    // a triangular A: every tile walks its own K range, in one pass (K slices would cut across them);
    // a symmetric A given by one triangle: the guarded kernel (it mirrors indices element by element),
    // unless the kernel for few output columns takes the call (below)
    const bool triangular = a.a_structure == GE_A_LOWER || a.a_structure == GE_A_UPPER;
    const ge_plan_t plan = triangular ? GE_PLAN_DIRECT : a.plan;
    st = make_plan_bf16(a.M, a.N, a.K, a.batch, fast_ok(a) && !is_symmetric(a), plan, a.split_k, &pl);
    if (st != GE_OK) return st;

    GemmParams p{};
    p.A = a.A; p.B = a.B; p.bias = a.bias; p.C = (float *)a.C;
    p.M = a.M; p.N = a.N; p.K = a.K;
    p.lda = a.lda; p.ldb = a.ldb; p.ldc = a.ldc;
    const long long rowsA = a.transA ? a.K : a.M, colsA = a.transA ? a.M : a.K;
    const long long rowsB = a.transB ? a.N : a.K, colsB = a.transB ? a.K : a.N;
    p.strideA = rowsA * a.lda;
    p.strideB = rowsB * a.ldb;
    p.strideC = (long long)a.M * a.ldc;
    p.sliceStride = (long long)a.batch * a.M * a.N;
    p.batch = a.batch;
    p.splitK = pl.splitK;
    p.kPerSlice = pl.kPerSlice;
    p.tilesM = pl.tilesM;
    p.tilesN = pl.tilesN;
    p.groupM = choose_group_m(pl.tilesM, pl.tilesN);
    p.alpha = a.alpha;
    p.act = (int)a.act;
    // extent of the operands as the arguments describe them (last row ends at its last element)
    p.bytesA = 2 * (((long long)a.batch * rowsA - 1) * a.lda + colsA);
    p.bytesB = 2 * (((long long)a.batch * rowsB - 1) * a.ldb + colsB);
    p.rowScale = a.row_scale;
    p.R = a.R;
    p.strideR = (long long)a.M * a.ldr;
    p.ldr = a.ldr;
    p.rType = (int)a.r_type;
    p.beta = a.R ? a.beta : 0.0f;
    p.clampLo = a.clamp_lo;
    p.clampHi = a.clamp_hi;
    p.cType = (int)a.c_type;
    const int rElem = a.r_type == GE_DTYPE_BF16 ? 2 : 4;
    p.rVec = (a.R && !(((uintptr_t)a.R) & 15u) && ((long long)a.ldr * rElem) % 16 == 0) ? 1 : 0;
    p.transA = a.transA ? 1 : 0;
    p.transB = a.transB ? 1 : 0;
    p.triA = (int)a.a_structure;

    if (is_symmetric(a)) {
        const SymmPlan sp = plan_symm(a);
        if (sp.fast) return run_symm(a, sp, p, (hipStream_t)stream);
    }

    const bool raw = pl.splitK > 1;
    void *ws = nullptr;
    GemmParams pg = p;                      // the GEMM pass: partial tiles go to the workspace
    if (raw) {
        st = acquire_workspace(partial_bytes(a.M, a.N, a.batch, pl.splitK), a.workspace, a.workspace_bytes, (hipStream_t)stream, &ws);
        if (st != GE_OK) return st;
        pg.C = (float *)ws;
    }
    const dim3 grid((unsigned)((long long)pl.tilesM * pl.tilesN * a.batch * pl.splitK));
    hipStream_t hs = (hipStream_t)stream;
    switch (pl.tile) {
    case TILE_256:
        // both operands k-strided: every request is a whole line already and the four-wave
        // kernel has nothing to gain (measured at 8192^3: 0.812 against 0.806 ms)
        if (four_wave_ok(pl, a.K) && !(a.transA && !a.transB)) {
            const int mode = four_wave_edge(pl, a.K);
            if (mode == 2) fused_four_wave_e2(pg, raw, grid, hs);
            else if (mode == 1) fused_four_wave_e1(pg, raw, grid, hs);
            else fused_four_wave_e0(pg, raw, grid, hs);
            set_config("256x256x64_w4", a.transA, a.transB, raw);
        } else if (launch_tile<256>(pg, pl.edge, raw, grid, hs)) set_config("256x256x64_w8", a.transA, a.transB, raw);
        else set_config("256x256x32_w8", a.transA, a.transB, raw);
        break;
    case TILE_128:
        if (launch_tile<128>(pg, pl.edge, raw, grid, hs)) set_config("128x128x64_w4", a.transA, a.transB, raw);
        else set_config("128x128x32_w4", a.transA, a.transB, raw);
        break;
    default:
        if (raw) GE_LAUNCH(ge::gemm_bf16_fused_generic_kernel<true>, grid, dim3(256), 0, hs, pg);
        else     GE_LAUNCH(ge::gemm_bf16_fused_generic_kernel<false>, grid, dim3(256), 0, hs, pg);
        set_config("generic_64x64x32", a.transA, a.transB, raw);
        break;
    }
    if (ge_host::take_launch_error() != hipSuccess) return GE_ERR_LAUNCH;
    if (raw) {
        const long long total = (long long)a.batch * a.M * a.N;
        long long blocks = (total + 255) / 256;
        if (blocks > 16 * kNumCU) blocks = 16 * kNumCU;
        GE_LAUNCH(ge::splitk_reduce_fused_kernel, dim3((unsigned)blocks), dim3(256), 0, hs, p, (const float *)ws);
        if (ge_host::take_launch_error() != hipSuccess) return GE_ERR_LAUNCH;
    }
    return GE_OK;
}
