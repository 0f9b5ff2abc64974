// C-ABI of the convolution front-end: a channels-last convolution evaluated as an implicit GEMM
// on the main bf16 kernel (rows = output positions gathered on the fly, columns = output
// channels, k = filter tap x input channel) with the fused consumer chain.  See
// include/gemm_epilogue.h for the contract.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>

#include "../../include/gemm_epilogue.h"
#include "conv_halo_launch.h"
#include "conv_rows.h"
#include "gemm_bf16_fast.h"
#include "gemm_fused.h"
#include "ge_host.h"

namespace {

using ge::GemmParams;
using namespace ge_host;

int out_size(int in, int k, int stride, int pad, int dil)
{
    const long long span = (long long)in + 2ll * pad - (long long)dil * (k - 1) - 1;
    return span < 0 ? 0 : (int)(span / stride + 1);
}

template <int BM, int BN, int WM, int WN>
void launch_conv(const GemmParams &p, bool edge, bool raw, dim3 grid, hipStream_t st)
{
    constexpr int threads = WM * WN * 64;
    const bool h = p.cType == ge::DT_BF16;
    if (raw) {
        if (edge) GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, true, true, ge::ACT_NONE, false, true, false, false, true>), grid, dim3(threads), 0, st, p);
        else      GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, false, true, ge::ACT_NONE, false, true, false, false, true>), grid, dim3(threads), 0, st, p);
    } else if (edge) {
        if (h) GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, true, false, ge::ACT_NONE, false, true, true, true, true>), grid, dim3(threads), 0, st, p);
        else   GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, true, false, ge::ACT_NONE, false, true, true, false, true>), grid, dim3(threads), 0, st, p);
    } else {
        if (h) GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, false, false, ge::ACT_NONE, false, true, true, true, true>), grid, dim3(threads), 0, st, p);
        else   GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, false, false, ge::ACT_NONE, false, true, true, false, true>), grid, dim3(threads), 0, st, p);
    }
}

// Validation and plan of one call: everything that depends on the sizes and on the alignment of the
// pointers only, shared by the call itself and by the workspace query.
struct ConvPlan {
    int OH, OW;
    long long M, K, xElems;
    bool rows;          // the few-channel kernel: a K step is one filter row
    bool rowsPairs;     //   ... whose input rows are 4-byte aligned and even in length
    int halo;           // the halo-staged 3 x 3 kernel: 0 no, else 1 + index into kHaloVariants
    ge_halo::HaloPlan haloPlan;
    Plan pl;
};

// The variants of the halo-staged kernel that are built: row blocks of 16 positions multiplied for a tile
// of the first and of the second kind.  14 and 11 serve rows of 49 to 56 positions cut 4 + 3 (residual
// networks' 56 x 56 images), 12 and 12 any cut of at most 192 positions.
constexpr int kHaloVariants[2][2] = {{14, 11}, {12, 12}};     // launch_conv_halo_14_11, launch_conv_halo_12_12
constexpr int kHaloTileOverhead = 2;      // prologue and epilogue of a tile, in row blocks of its main loop

// Workgroups of the few-channel kernel that the device holds at once (they walk over the output rows);
// a host-side computation of the runtime, nothing is enqueued.
template <int NT, bool OUTBF16, bool PAIRS, int KHT>
int rows_resident_blocks(size_t ldsBytes)
{
    // the answer depends on the variant and on its LDS bytes only: kept per thread for the last size asked
    static thread_local size_t knownFor = ~(size_t)0;
    static thread_local int known = 0;
    if (knownFor == ldsBytes) return known;
    int perCU = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&perCU, ge::conv_rows_bf16_kernel<NT, OUTBF16, PAIRS, KHT>, 256, ldsBytes) != hipSuccess ||
        perCU < 1)
        perCU = 1;
    knownFor = ldsBytes;
    known = perCU * kNumCU;
    return known;
}

template <int NT, bool OUTBF16, bool PAIRS, int KHT>
void launch_rows_kh(const GemmParams &p, int items, size_t ldsBytes, hipStream_t st)
{
    const int resident = rows_resident_blocks<NT, OUTBF16, PAIRS, KHT>(ldsBytes);
    const int blocks = items < resident ? items : resident;
    GE_LAUNCH((ge::conv_rows_bf16_kernel<NT, OUTBF16, PAIRS, KHT>), dim3((unsigned)blocks), dim3(256), ldsBytes, st, p, items);
}

// 7 and 3 filter rows (first layers) have kernels of their own, any other count one with a run-time count
template <int NT, bool OUTBF16, bool PAIRS>
void launch_rows(const GemmParams &p, int items, size_t ldsBytes, hipStream_t st)
{
    if (p.convKH == 7) launch_rows_kh<NT, OUTBF16, PAIRS, 7>(p, items, ldsBytes, st);
    else if (p.convKH == 3) launch_rows_kh<NT, OUTBF16, PAIRS, 3>(p, items, ldsBytes, st);
    else launch_rows_kh<NT, OUTBF16, PAIRS, 0>(p, items, ldsBytes, st);
}

ge_status_t plan_conv(const ge_conv_args_t &a, ConvPlan *out)
{
    if (!a.X || !a.Wt || !a.Y) return GE_ERR_NULL;
    if (a.N < 1 || a.H < 1 || a.W < 1 || a.Cin < 1 || a.Cout < 1 || a.KH < 1 || a.KW < 1) return GE_ERR_SHAPE;
    if (a.stride_h < 1 || a.stride_w < 1 || a.pad_h < 0 || a.pad_w < 0 || a.dil_h < 1 || a.dil_w < 1) return GE_ERR_SHAPE;
    const int OH = out_size(a.H, a.KH, a.stride_h, a.pad_h, a.dil_h), OW = out_size(a.W, a.KW, a.stride_w, a.pad_w, a.dil_w);
    if (OH < 1 || OW < 1) return GE_ERR_SHAPE;
    const long long M = (long long)a.N * OH * OW, K = (long long)a.KH * a.KW * a.Cin;
    const long long xElems = (long long)a.N * a.H * a.W * a.Cin;
    // the kernels index positions and k with 32-bit integers
    if (M > 0x7fffffffll / 2 || K > 0x7fffffffll / 2 || xElems > (1ll << 40) || M * a.Cout > (1ll << 40)) return GE_ERR_SHAPE;
    if (a.pad_h > (1 << 20) || a.pad_w > (1 << 20) || (long long)a.dil_h * a.KH > (1 << 20) || (long long)a.dil_w * a.KW > (1 << 20))
        return GE_ERR_SHAPE;
    if (a.act != GE_ACT_NONE && a.act != GE_ACT_RELU && a.act != GE_ACT_GELU_TANH) return GE_ERR_ACT;
    if (a.y_type != GE_DTYPE_F32 && a.y_type != GE_DTYPE_BF16) return GE_ERR_EPILOGUE;
    if (a.R && a.r_type != GE_DTYPE_F32 && a.r_type != GE_DTYPE_BF16) return GE_ERR_EPILOGUE;
    if (!(a.clamp_lo <= a.clamp_hi)) return GE_ERR_EPILOGUE;
    const uintptr_t yMask = a.y_type == GE_DTYPE_F32 ? 3u : 1u, rMask = a.r_type == GE_DTYPE_F32 ? 3u : 1u;
    if ((((uintptr_t)a.X) & 1u) || (((uintptr_t)a.Wt) & 1u) || (((uintptr_t)a.Y) & yMask)) return GE_ERR_ALIGN;
    if (a.R && (((uintptr_t)a.R) & rMask)) return GE_ERR_ALIGN;
    if (a.bias && (((uintptr_t)a.bias) & 3u)) return GE_ERR_ALIGN;

    // gathering kernel: a K step is 32 channels of one tap, chunks of 8 channels are 16 aligned
    // bytes, byte offsets into the input fit 31 bits; bf16 output leaves in 16-byte row pieces
    bool fast = !((((uintptr_t)a.X) | ((uintptr_t)a.Wt)) & 15u) && (a.Cin % 32 == 0) && (a.Cout % 8 == 0) &&
                xElems * 2 < (1ll << 31) - (1 << 20) && K * 2 * 256 + 1024 < (1ll << 31);
    if (a.y_type == GE_DTYPE_BF16 && (((uintptr_t)a.Y) & 15u)) fast = false;
    out->OH = OH; out->OW = OW; out->M = M; out->K = K; out->xElems = xElems;
    // few input channels: one filter row per K step (conv_rows.h) where a row of the filter fits the
    // 32 elements of a step, its image of an input row fits 512 dwords, a lane's 8 channels of Y (and
    // of R) are 16 aligned bytes or two such pieces, and the filter bank can be copied dword by dword
    out->rows = false; out->rowsPairs = false;
    if (!fast && opt_force_config() != FORCE_GENERIC && a.dil_w == 1 && (long long)a.KW * a.Cin <= ge_conv_rows::KSTEP &&
        a.KH <= ge_conv_rows::KH_MAX && (a.Cout == 32 || a.Cout == 64) && (long long)a.W * a.Cin < (1 << 20) && a.pad_w < 4096 &&
        a.stride_w < 4096 && (long long)OW * a.stride_w * a.Cin < (1 << 20) && !(((uintptr_t)a.Y) & 15u) &&
        !(a.R && (((uintptr_t)a.R) & 15u)) && !(((uintptr_t)a.Wt) & 3u)) {
        const int pitch = ge_conv_rows::pitch_dwords(a.W, a.Cin, OW, a.stride_w, a.pad_w);
        if (pitch <= 512) {
            out->rows = true;
            out->rowsPairs = ((a.W * a.Cin) % 2 == 0) && !(((uintptr_t)a.X) & 3u);
        }
    }
    // 3 x 3, unit stride and dilation, whole 256-channel tiles, 64-channel pairs of slabs, an output row
    // with its two halo columns within the 64 positions of a staged row: the halo-staged kernel
    out->halo = 0;
    const int haloOpt = opt_conv_halo();
    if (fast && opt_force_config() == FORCE_NONE && haloOpt != HALO_OFF && a.KH == 3 && a.KW == 3 && a.stride_h == 1 &&
        a.stride_w == 1 && a.dil_h == 1 && a.dil_w == 1 && a.Cin % 64 == 0 && a.Cout % 256 == 0 && OW <= ge_halo::MAX_OW &&
        a.pad_w <= 2 && a.pad_h <= 2) {
        for (int v = 0; v < 2; ++v) {
            if (haloOpt >= HALO_VARIANT0 && haloOpt != HALO_VARIANT0 + v) continue;
            const ge_halo::HaloPlan hp = ge_halo::halo_plan(a.N, OH, OW, a.Cout / 256, kNumCU, kHaloTileOverhead,
                                                             kHaloVariants[v][0], kHaloVariants[v][1]);
            if (hp.cost < 0) continue;
            // left to itself: tiles for at least half of the CUs (fewer: the gathering kernel has K slices), and
            // at least 0.7 of the positions its loops multiply are output positions
            const long long n1 = (long long)a.N * hp.g1 * (a.Cout / 256), n2 = (long long)a.N * hp.g2 * (a.Cout / 256);
            const long long multiplied = 16 * (n1 * hp.blocks16a + n2 * hp.blocks16b);
            if (haloOpt == HALO_AUTO && (n1 + n2 < kNumCU / 2 || 10 * M * (a.Cout / 256) < 7 * multiplied)) continue;
            if (!out->halo || hp.cost < out->haloPlan.cost) { out->halo = 1 + v; out->haloPlan = hp; }
        }
    }
    ge_status_t st = make_plan_bf16((int)M, a.Cout, (int)K, 1, fast, GE_PLAN_AUTO, 0, &out->pl);
    if (st == GE_OK && out->halo) { out->pl.splitK = 1; out->pl.kPerSlice = (int)K; }
    if (st == GE_OK && out->rows) { out->pl.splitK = 1; out->pl.kPerSlice = (int)K; }
    return st;
}

}  // namespace

extern "C" size_t conv2d_epilogue_workspace_bytes(const ge_conv_args_t *args)
{
    ConvPlan cp;
    if (!args || plan_conv(*args, &cp) != GE_OK) return 0;
    return partial_bytes((int)cp.M, args->Cout, 1, cp.pl.splitK);
}

extern "C" ge_status_t conv2d_epilogue_bf16(const ge_conv_args_t *args, void *stream)
{
    if (!args) return GE_ERR_NULL;
    const ge_conv_args_t &a = *args;
    ConvPlan cp;
    ge_status_t st = plan_conv(a, &cp);
    if (st != GE_OK) return st;
    const int OH = cp.OH, OW = cp.OW;
    const long long M = cp.M, K = cp.K, xElems = cp.xElems;
    const Plan &pl = cp.pl;

    GemmParams p{};
    p.A = a.X; p.B = a.Wt; p.bias = a.bias; p.C = (float *)a.Y;
    p.M = (int)M; p.N = a.Cout; p.K = (int)K;
    p.lda = (int)K; p.ldb = (int)K; p.ldc = a.Cout;
    p.strideA = 0; p.strideB = 0; p.strideC = 0;
    p.batch = 1;
    p.splitK = pl.splitK;
    p.kPerSlice = pl.kPerSlice;
    p.sliceStride = M * a.Cout;
    p.tilesM = pl.tilesM;
    p.tilesN = pl.tilesN;
    p.groupM = choose_group_m(pl.tilesM, pl.tilesN);
    p.alpha = a.alpha;
    p.act = (int)a.act;
    p.bytesA = xElems * 2;
    p.bytesB = (long long)a.Cout * K * 2;
    p.R = a.R;
    p.strideR = 0;
    p.ldr = a.Cout;
    p.rType = (int)a.r_type;
    p.beta = a.R ? a.beta : 0.0f;
    const int rElem = a.r_type == GE_DTYPE_BF16 ? 2 : 4;
    p.rVec = (a.R && !(((uintptr_t)a.R) & 15u) && ((long long)a.Cout * rElem) % 16 == 0) ? 1 : 0;
    p.clampLo = a.clamp_lo;
    p.clampHi = a.clamp_hi;
    p.cType = (int)a.y_type;
    p.transA = 0;
    p.transB = 1;
    p.convH = a.H; p.convW = a.W; p.convCin = a.Cin; p.convKH = a.KH; p.convKW = a.KW;
    p.convOH = OH; p.convOW = OW;
    p.convSh = a.stride_h; p.convSw = a.stride_w; p.convPh = a.pad_h; p.convPw = a.pad_w;
    p.convDh = a.dil_h; p.convDw = a.dil_w;

    if (cp.rows) {
        const int pitch = ge_conv_rows::pitch_dwords(a.W, a.Cin, OW, a.stride_w, a.pad_w);
        const size_t ldsBytes = (size_t)ge_conv_rows::lds_dwords(a.KH, pitch, a.Cout, a.KW * a.Cin) * 4;
        const int items = a.N * OH;                      // N * OH * OW fits 30 bits (checked by the plan)
        hipStream_t hs = (hipStream_t)stream;
        const bool h = a.y_type == GE_DTYPE_BF16;
        if (a.Cout == 64) {
            if (cp.rowsPairs) { if (h) launch_rows<4, true, true>(p, items, ldsBytes, hs); else launch_rows<4, false, true>(p, items, ldsBytes, hs); }
            else              { if (h) launch_rows<4, true, false>(p, items, ldsBytes, hs); else launch_rows<4, false, false>(p, items, ldsBytes, hs); }
        } else {
            if (cp.rowsPairs) { if (h) launch_rows<2, true, true>(p, items, ldsBytes, hs); else launch_rows<2, false, true>(p, items, ldsBytes, hs); }
            else              { if (h) launch_rows<2, true, false>(p, items, ldsBytes, hs); else launch_rows<2, false, false>(p, items, ldsBytes, hs); }
        }
        g_last_config = "conv_bf16_rows_k32";
        return ge_host::take_launch_error() != hipSuccess ? GE_ERR_LAUNCH : GE_OK;
    }

    if (cp.halo) {
        const ge_halo::HaloPlan &hp = cp.haloPlan;
        ge::HaloTiles ht{};
        ht.R1 = hp.R1; ht.g1 = hp.g1; ht.R2 = hp.R2; ht.g2 = hp.g2;
        ht.tilesN = a.Cout / 256;
        ht.tiles1 = a.N * hp.g1 * ht.tilesN;
        ht.tiles2 = a.N * hp.g2 * ht.tilesN;
        ht.posMul = 65536 / OW + 1;
        hipStream_t hs = (hipStream_t)stream;
        if (cp.halo == 1) { launch_conv_halo_14_11(p, ht, hs); g_last_config = "conv_bf16_halo_3x3_w4_14_11"; }
        else              { launch_conv_halo_12_12(p, ht, hs); g_last_config = "conv_bf16_halo_3x3_w4_12_12"; }
        return ge_host::take_launch_error() != hipSuccess ? GE_ERR_LAUNCH : GE_OK;
    }

    // few output tiles and a long K (late layers: small images, many channels): K slices into the
    // library's workspace, summed in slice order by the second pass, which also runs the chain
    const bool raw = pl.splitK > 1;
    void *ws = nullptr;
    GemmParams pg = p;
    if (raw) {
        st = acquire_workspace(partial_bytes((int)M, a.Cout, 1, pl.splitK), a.workspace, a.workspace_bytes, (hipStream_t)stream, &ws);
        if (st != GE_OK) return st;
        pg.C = (float *)ws;
    }
    const dim3 grid((unsigned)((long long)pl.tilesM * pl.tilesN * pl.splitK));
    hipStream_t hs = (hipStream_t)stream;
    switch (pl.tile) {
    case TILE_256:
        launch_conv<256, 256, 2, 4>(pg, pl.edge, raw, grid, hs);
        g_last_config = raw ? "conv_bf16_256x256x32_w8_splitk" : "conv_bf16_256x256x32_w8";
        break;
    case TILE_128:
        launch_conv<128, 128, 2, 2>(pg, pl.edge, raw, grid, hs);
        g_last_config = raw ? "conv_bf16_128x128x32_w4_splitk" : "conv_bf16_128x128x32_w4";
        break;
    default:
        if (raw) GE_LAUNCH(ge::conv_bf16_generic_kernel<true>, grid, dim3(256), 0, hs, pg);
        else     GE_LAUNCH(ge::conv_bf16_generic_kernel<false>, grid, dim3(256), 0, hs, pg);
        g_last_config = raw ? "conv_bf16_generic_64x64x32_splitk" : "conv_bf16_generic_64x64x32";
        break;
    }
    if (ge_host::take_launch_error() != hipSuccess) return GE_ERR_LAUNCH;
    if (raw) {
        const long long total = M * a.Cout;
        long long blocks = (total + 255) / 256;
        if (blocks > 16 * kNumCU) blocks = 16 * kNumCU;
        GE_LAUNCH(ge::splitk_reduce_fused_kernel, dim3((unsigned)blocks), dim3(256), 0, hs, p, (const float *)ws);
        if (ge_host::take_launch_error() != hipSuccess) return GE_ERR_LAUNCH;
    }
    return GE_OK;
}
