// C-ABI of the gfx950 fused GEMM library: argument validation, plan selection
// (direct / batched / split-K, tile shape) and kernel launches.  See
// include/gemm_epilogue.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/gemm_epilogue.h"
#include "gemm_bf16_fast.h"
#include "gemm_bf16_w4.h"
#include "gemm_f32_fast.h"
#include "gemm_generic.h"
#include "ge_host.h"

namespace ge_host {

thread_local const char *g_last_config = "none";

thread_local hipError_t g_launch_error = hipSuccess;

// Library-owned buffers for partial results, one per (device, stream) that has needed one: calls on
// different streams never share a buffer, calls on one stream are ordered by it.
struct Workspace {
    int dev;
    hipStream_t stream;
    void *ptr;
    size_t bytes;
};
std::vector<Workspace> g_ws, g_ws_retired;
std::mutex g_ws_mutex;

// Switches for timing runs and tests: set by ge_set_option, initial values from the environment,
// read once when the library is loaded.
std::atomic<int> g_opt_force{FORCE_NONE};
std::atomic<int> g_opt_waves8{0}, g_opt_stage32{0};

int parse_force(const char *v)
{
    if (!v) return FORCE_NONE;
    if (std::strcmp(v, "256x256") == 0) return FORCE_256;
    if (std::strcmp(v, "128x128") == 0) return FORCE_128;
    if (std::strcmp(v, "generic") == 0) return FORCE_GENERIC;
    return -1;
}

const bool g_env_read = [] {
    const int f = parse_force(std::getenv("GE_FORCE_CONFIG"));
    g_opt_force = f < 0 ? FORCE_NONE : f;
    const char *w = std::getenv("GE_WAVES"), *k = std::getenv("GE_STAGE_K");
    g_opt_waves8 = (w && std::strcmp(w, "8") == 0) ? 1 : 0;
    g_opt_stage32 = (k && std::strcmp(k, "32") == 0) ? 1 : 0;
    return true;
}();

int opt_force_config() { return g_opt_force.load(std::memory_order_relaxed); }
bool opt_eight_waves() { return g_opt_waves8.load(std::memory_order_relaxed) != 0; }
bool opt_stage_k32() { return g_opt_stage32.load(std::memory_order_relaxed) != 0; }

bool fast_path_ok(int N, int K, const void *A, int lda, const void *B, int ldb)
{
    if ((((uintptr_t)A) | ((uintptr_t)B)) & 15u) return false;
    if ((lda | ldb | N | K) & 7) return false;
    // per-lane byte offsets inside one tile panel must stay below 2^31
    if ((long long)lda * 2 * 256 + 256 >= (1ll << 31)) return false;
    if ((long long)ldb * 2 * 64 + 1024 >= (1ll << 31)) return false;
    return true;
}

// K slices so that a launch with few output tiles still covers the chip (the guarded kernels; the
// direct-to-LDS kernels choose tile and slices together, see plan_cost_us).
int choose_split(long long tiles, int K, int minSlice)
{
    const int kMinSlice = minSlice;            // K extent below which a slice is not worth its partial tile
    if (tiles * 2 > kNumCU || K < 2 * kMinSlice) return 1;
    long long s = kNumCU / tiles;
    const long long maxS = K / kMinSlice;
    if (s > maxS) s = maxS;
    if (s > 64) s = 64;
    return s < 2 ? 1 : (int)s;
}

void slice_k(int K, int bk, int want, int *splitK, int *kPerSlice)
{
    int per = ceil_div(ceil_div(K, want), bk) * bk;
    if (per < bk) per = bk;
    *kPerSlice = per;
    *splitK = ceil_div(K, per);
}

// Estimated time in microseconds of one structure -- block tile (256 or 128) and number of K slices --
// from a few measured rates: a 256 x 256 block takes 0.80 us per 32-wide K step and about 8 us to fill
// its pipeline and store its tile, one to a CU; a 128 x 128 block takes 0.30 us per step alone on a CU
// and 0.54 us when two share it (about 5 and 6 us fixed); K slices add the second pass (a launch and
// the partial tiles written and read at about 4 TB/s).  Per output element the large tile is the
// cheaper one (0.20 against 0.27-0.30 us per 128 x 128 x 32 of work); the small one wins where the
// large one would leave CUs idle or need many slices.  Calibrated on, and checked against, the timed
// search over both choices (tune.py): the rule is for ranking structures, not for predicting times.
double plan_cost_us(int M, int N, int K, int batch, int tile, int slices)
{
    const long long tiles = (long long)ceil_div(M, tile) * ceil_div(N, tile) * batch;
    const long long blocks = tiles * slices;
    const double steps = (double)ceil_div(ceil_div(K, slices), 32);
    double t;
    if (tile == 256) t = (double)((blocks + kNumCU - 1) / kNumCU) * (steps * 0.80 + 8.0);
    else if (blocks <= kNumCU) t = steps * 0.30 + 5.0;
    else t = (double)((blocks + 2 * kNumCU - 1) / (2 * kNumCU)) * (steps * 0.54 + 6.0);
    if (slices > 1) t += 3.0 + (double)(slices + 1) * (double)batch * (double)M * (double)N * 4.0 / 4.0e6;
    return t;
}

// The slice count of lowest estimated cost for a tile (1 = none); slices keep at least minSlice of K.
int best_slices(int M, int N, int K, int batch, int tile, int minSlice, double *cost)
{
    int best = 1;
    double bestCost = plan_cost_us(M, N, K, batch, tile, 1);
    const int maxS = K / minSlice < 64 ? K / minSlice : 64;
    for (int s2 = 2; s2 <= maxS; ++s2) {
        const double c = plan_cost_us(M, N, K, batch, tile, s2);
        if (c < bestCost) { bestCost = c; best = s2; }
    }
    if (cost) *cost = bestCost;
    return best;
}

ge_status_t make_plan_bf16(int M, int N, int K, int batch, bool fast, ge_plan_t plan, int split_k, Plan *out)
{
    Plan pl{};
    if (plan != GE_PLAN_AUTO && plan != GE_PLAN_DIRECT && plan != GE_PLAN_SPLITK) return GE_ERR_CONFIG;
    if (split_k < 0) return GE_ERR_CONFIG;
    const int force = opt_force_config();
    int want = 1;
    if (!fast || force == FORCE_GENERIC) {
        pl.tile = TILE_GENERIC; pl.bm = 64; pl.bn = 64; pl.bk = 32;
        const long long tiles = (long long)ceil_div(M, 64) * ceil_div(N, 64) * batch;
        if (plan == GE_PLAN_SPLITK) want = split_k > 0 ? split_k : choose_split(tiles, K, 512);
        else if (plan == GE_PLAN_AUTO) want = choose_split(tiles, K, 512);
        if (plan == GE_PLAN_SPLITK && want < 2) want = 2;
    } else {
        // both tiles are candidates when the problem has 256 rows and columns; each with the slice
        // count the plan asks for (none, the caller's, or its own best), the cheaper structure wins
        constexpr int kMinSlice = 512;
        int tileOf[2] = {256, 128}, slicesOf[2] = {1, 1};
        double costOf[2] = {0.0, 0.0};
        for (int c = 0; c < 2; ++c) {
            if (plan == GE_PLAN_DIRECT) slicesOf[c] = 1;
            else if (plan == GE_PLAN_SPLITK && split_k > 0) slicesOf[c] = split_k < 2 ? 2 : split_k;
            else {
                slicesOf[c] = best_slices(M, N, K, batch, tileOf[c], kMinSlice, nullptr);
                if (plan == GE_PLAN_SPLITK && slicesOf[c] < 2) slicesOf[c] = 2;
            }
            costOf[c] = plan_cost_us(M, N, K, batch, tileOf[c], slicesOf[c]);
        }
        bool big = (M >= 256 && N >= 256) && costOf[0] <= costOf[1];
        if (force == FORCE_256) big = true;
        if (force == FORCE_128) big = false;
        if (big) { pl.tile = TILE_256; pl.bm = 256; pl.bn = 256; pl.bk = ge::BF16_BK; want = slicesOf[0]; }
        else     { pl.tile = TILE_128; pl.bm = 128; pl.bn = 128; pl.bk = ge::BF16_BK; want = slicesOf[1]; }
    }
    pl.tilesM = ceil_div(M, pl.bm);
    pl.tilesN = ceil_div(N, pl.bn);
    const long long tiles = (long long)pl.tilesM * pl.tilesN * batch;
    if (tiles > 0x7fffffffll / 64) return GE_ERR_SHAPE;
    slice_k(K, pl.bk, want, &pl.splitK, &pl.kPerSlice);
    if (pl.splitK == 1) pl.kPerSlice = ceil_div(K, pl.bk) * pl.bk;
    if (tiles * pl.splitK > 0x7fffffffll) return GE_ERR_SHAPE;
    pl.edge = (M % pl.bm) || (N % pl.bn) || (K % pl.bk) || (pl.kPerSlice % pl.bk);
    *out = pl;
    return GE_OK;
}

size_t partial_bytes(int M, int N, int batch, int splitK)
{
    return splitK <= 1 ? 0 : (size_t)splitK * (size_t)batch * (size_t)M * (size_t)N * sizeof(float);
}

ge_status_t validate(int M, int N, int K, const void *A, int lda, const void *B, int ldb,
                     const void *bias, int act, const void *C, int ldc, int batch, size_t elem)
{
    if (!A || !B || !C) return GE_ERR_NULL;
    if (M < 1 || N < 1 || K < 1 || batch < 1) return GE_ERR_SHAPE;
    if (lda < K || ldb < N || ldc < N) return GE_ERR_LD;
    if (act != GE_ACT_NONE && act != GE_ACT_RELU && act != GE_ACT_GELU_TANH) return GE_ERR_ACT;
    if (((uintptr_t)A % elem) || ((uintptr_t)B % elem) || ((uintptr_t)C % 4) || ((uintptr_t)bias % 4))
        return GE_ERR_ALIGN;
    // element counts of one operand must fit 63 bits comfortably
    const long double big = 9.0e18L;
    if ((long double)batch * M * lda > big || (long double)batch * K * ldb > big ||
        (long double)batch * M * ldc > big)
        return GE_ERR_SHAPE;
    return GE_OK;
}

GemmParams base_params(int M, int N, int K, const void *A, int lda, const void *B, int ldb,
                       const float *bias, float alpha, int act, float *C, int ldc, int batch)
{
    GemmParams p{};
    p.A = A; p.B = B; p.bias = bias; p.C = C;
    p.M = M; p.N = N; p.K = K;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.strideA = (long long)M * lda;
    p.strideB = (long long)K * ldb;
    p.strideC = (long long)M * ldc;
    p.sliceStride = (long long)batch * M * N;
    p.batch = batch;
    p.splitK = 1;
    p.alpha = alpha;
    p.act = act;
    p.bytesA = 0;
    p.bytesB = 0;
    return p;
}

// Tile rows swept together: enough that the ~32 tiles resident on one XCD form
// a compact block (A panels and B panels both reused from that XCD's L2).
int choose_group_m(int tilesM, int tilesN)
{
    int g = 8;
    if (tilesN < 4) g = 32 / (tilesN < 1 ? 1 : tilesN);
    if (g > tilesM) g = tilesM;
    return g < 1 ? 1 : g;
}

ge_status_t acquire_workspace(size_t need, void *user, size_t user_bytes, hipStream_t stream, void **out)
{
    if (user) {
        if (user_bytes < need || ((uintptr_t)user & 255u)) return GE_ERR_WORKSPACE;
        *out = user;
        return GE_OK;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return GE_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    Workspace *ws = nullptr;
    for (Workspace &w : g_ws)
        if (w.dev == dev && w.stream == stream) { ws = &w; break; }
    if (ws && ws->bytes >= need) {
        *out = ws->ptr;
        return GE_OK;
    }
    // A larger buffer is needed.  hipMalloc is not a capturable operation, and a graph captured
    // now would keep replaying into whatever address it recorded: refuse instead.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return GE_ERR_WORKSPACE;
    void *ptr = nullptr;
    if (hipMalloc(&ptr, need) != hipSuccess) return GE_ERR_WORKSPACE;
    if (ws) {
        // work enqueued earlier (or a graph captured earlier) may still use the outgrown buffer
        g_ws_retired.push_back(Workspace{dev, nullptr, ws->ptr, 0});
        ws->ptr = ptr;
        ws->bytes = need;
    } else {
        g_ws.push_back(Workspace{dev, stream, ptr, need});
    }
    *out = ptr;
    return GE_OK;
}

template <int EDGE>
hipError_t launch_four_wave(const GemmParams &p, bool raw, int act, dim3 grid, hipStream_t st)
{
    if (raw) {
        GE_LAUNCH((ge::gemm_bf16_w4_kernel<EDGE, true, ge::ACT_NONE, false, false, false, false>), grid, dim3(256), 0, st, p);
    } else if (act == GE_ACT_RELU) {
        GE_LAUNCH((ge::gemm_bf16_w4_kernel<EDGE, false, ge::ACT_RELU, false, false, false, false>), grid, dim3(256), 0, st, p);
    } else if (act == GE_ACT_GELU_TANH) {
        GE_LAUNCH((ge::gemm_bf16_w4_kernel<EDGE, false, ge::ACT_GELU_TANH, false, false, false, false>), grid, dim3(256), 0, st, p);
    } else {
        GE_LAUNCH((ge::gemm_bf16_w4_kernel<EDGE, false, ge::ACT_NONE, false, false, false, false>), grid, dim3(256), 0, st, p);
    }
    return ge_host::take_launch_error();
}

template <int BM, int BN, int WM, int WN, bool EDGE>
hipError_t launch_fast_sel(const GemmParams &p, bool raw, int act, dim3 grid, hipStream_t st)
{
    constexpr int threads = WM * WN * 64;
    if (raw) {
        GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, EDGE, true, ge::ACT_NONE>), grid, dim3(threads), 0, st, p);
    } else if (act == GE_ACT_RELU) {
        GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, EDGE, false, ge::ACT_RELU>), grid, dim3(threads), 0, st, p);
    } else if (act == GE_ACT_GELU_TANH) {
        GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, EDGE, false, ge::ACT_GELU_TANH>), grid, dim3(threads), 0, st, p);
    } else {
        GE_LAUNCH((ge::gemm_bf16_kernel<BM, BN, WM, WN, EDGE, false, ge::ACT_NONE>), grid, dim3(threads), 0, st, p);
    }
    return ge_host::take_launch_error();
}

hipError_t launch_reduce(const GemmParams &p, const float *W, float *C, int ldc, int act,
                         const float *bias, float alpha, hipStream_t st)
{
    const long long total = (long long)p.batch * p.M * p.N;
    long long blocks = (total / 4 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 16 * kNumCU) blocks = 16 * kNumCU;
    GE_LAUNCH(ge::splitk_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       W, p.sliceStride, p.splitK, p.M, p.N, p.batch, bias, alpha, act, C, ldc,
                       (long long)p.M * ldc);
    return ge_host::take_launch_error();
}

bool four_wave_ok(const Plan &pl, int K)
{
    if (opt_eight_waves()) return false;
    const int range = pl.splitK > 1 ? pl.kPerSlice : K;
    return pl.tile == TILE_256 && range >= 256;
}

int four_wave_edge(const Plan &pl, int K)
{
    if (K % 128 != 0 || (pl.splitK > 1 && pl.kPerSlice % 128 != 0)) return 2;
    return pl.edge ? 1 : 0;
}

ge_status_t run_bf16(int M, int N, int K, const uint16_t *A, int lda, const uint16_t *B, int ldb,
                     const float *bias, float alpha, ge_act_t act, float *C, int ldc, int batch,
                     ge_plan_t plan, int split_k, void *workspace, size_t workspace_bytes, void *stream)
{
    ge_status_t st = validate(M, N, K, A, lda, B, ldb, bias, (int)act, C, ldc, batch, 2);
    if (st != GE_OK) return st;
    Plan pl;
    st = make_plan_bf16(M, N, K, batch, fast_path_ok(N, K, A, lda, B, ldb), plan, split_k, &pl);
    if (st != GE_OK) return st;

    GemmParams p = base_params(M, N, K, A, lda, B, ldb, bias, alpha, (int)act, C, ldc, batch);
    p.tilesM = pl.tilesM;
    p.tilesN = pl.tilesN;
    p.groupM = choose_group_m(pl.tilesM, pl.tilesN);
    p.splitK = pl.splitK;
    p.kPerSlice = pl.kPerSlice;

    // extent of the operands as the arguments describe them (last row ends at its last element)
    p.bytesA = 2 * (((long long)batch * M - 1) * lda + K);
    p.bytesB = 2 * (((long long)batch * K - 1) * ldb + N);

    const bool raw = pl.splitK > 1;
    void *ws = nullptr;
    if (raw) {
        st = acquire_workspace(partial_bytes(M, N, batch, pl.splitK), workspace, workspace_bytes, (hipStream_t)stream, &ws);
        if (st != GE_OK) return st;
        p.C = (float *)ws;
    }
    const dim3 grid((unsigned)((long long)pl.tilesM * pl.tilesN * batch * pl.splitK));
    hipStream_t hs = (hipStream_t)stream;
    hipError_t err;
    switch (pl.tile) {
    case TILE_256:
        if (four_wave_ok(pl, K)) {
            const int mode = four_wave_edge(pl, K);
            err = mode == 2 ? launch_four_wave<2>(p, raw, (int)act, grid, hs)
                : mode == 1 ? launch_four_wave<1>(p, raw, (int)act, grid, hs) : launch_four_wave<0>(p, raw, (int)act, grid, hs);
            g_last_config = raw ? "bf16_256x256x64_w4_splitk" : "bf16_256x256x64_w4";
            break;
        }
        err = pl.edge ? launch_fast_sel<256, 256, 2, 4, true>(p, raw, (int)act, grid, hs)
                      : launch_fast_sel<256, 256, 2, 4, false>(p, raw, (int)act, grid, hs);
        g_last_config = raw ? "bf16_256x256x32_w8_splitk" : "bf16_256x256x32_w8";
        break;
    case TILE_128:
        err = pl.edge ? launch_fast_sel<128, 128, 2, 2, true>(p, raw, (int)act, grid, hs)
                      : launch_fast_sel<128, 128, 2, 2, false>(p, raw, (int)act, grid, hs);
        g_last_config = raw ? "bf16_128x128x32_w4_splitk" : "bf16_128x128x32_w4";
        break;
    default:
        if (raw) GE_LAUNCH(ge::gemm_bf16_generic_kernel<true>, grid, dim3(256), 0, hs, p);
        else     GE_LAUNCH(ge::gemm_bf16_generic_kernel<false>, grid, dim3(256), 0, hs, p);
        err = ge_host::take_launch_error();
        g_last_config = raw ? "bf16_generic_64x64x32_splitk" : "bf16_generic_64x64x32";
        break;
    }
    if (err != hipSuccess) return GE_ERR_LAUNCH;
    if (raw) {
        err = launch_reduce(p, (const float *)ws, C, ldc, (int)act, bias, alpha, hs);
        if (err != hipSuccess) return GE_ERR_LAUNCH;
    }
    return GE_OK;
}

// ---- scratch for the entry point that allocates nothing -----------------------------------------
// Partial tiles of gemm_epilogue_bf16_static live in this array, which every GPU the library runs
// on holds, at its own address, until the process ends.  In host code the array's name is not a
// device address: the address is asked for once per device (with that device current) and kept.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
constexpr int kMaxDevices = 64;
void *g_static_scratch_ptr[kMaxDevices] = {};
std::mutex g_static_scratch_mutex;

}  // namespace ge_host

static __device__ __align__(256) unsigned char scratch[ge_host::kStaticScratchBytes];

namespace ge_host {

ge_status_t static_scratch(void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GE_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return GE_ERR_WORKSPACE;
        g_static_scratch_ptr[dev] = ptr;
    }
    *out = g_static_scratch_ptr[dev];
    return GE_OK;
}

}  // namespace ge_host

using namespace ge_host;

extern "C" {

ge_status_t gemm_epilogue_bf16(int M, int N, int K, const uint16_t *A, int lda, const uint16_t *B, int ldb,
                               const float *bias, float alpha, ge_act_t act, float *C, int ldc,
                               int batch, void *stream)
{
    return run_bf16(M, N, K, A, lda, B, ldb, bias, alpha, act, C, ldc, batch, GE_PLAN_AUTO, 0, nullptr, 0, stream);
}

ge_status_t gemm_epilogue_bf16_ex(int M, int N, int K, const uint16_t *A, int lda, const uint16_t *B, int ldb,
                                  const float *bias, float alpha, ge_act_t act, float *C, int ldc,
                                  int batch, ge_plan_t plan, int split_k, void *workspace,
                                  size_t workspace_bytes, void *stream)
{
    return run_bf16(M, N, K, A, lda, B, ldb, bias, alpha, act, C, ldc, batch, plan, split_k, workspace,
                    workspace_bytes, stream);
}

ge_status_t gemm_epilogue_bf16_static(int M, int N, int K, const uint16_t *A, int lda, const uint16_t *B, int ldb,
                                      const float *bias, float alpha, ge_act_t act, float *C, int ldc,
                                      int batch, ge_plan_t plan, int split_k, void *stream)
{
    ge_status_t st = validate(M, N, K, A, lda, B, ldb, bias, (int)act, C, ldc, batch, 2);
    if (st != GE_OK) return st;
    Plan pl;
    st = make_plan_bf16(M, N, K, batch, fast_path_ok(N, K, A, lda, B, ldb), plan, split_k, &pl);
    if (st != GE_OK) return st;
    void *ws = nullptr;
    if (pl.splitK > 1) {
        if (partial_bytes(M, N, batch, pl.splitK) > kStaticScratchBytes) return GE_ERR_WORKSPACE;
        st = static_scratch(&ws);
        if (st != GE_OK) return st;
    }
    // with a workspace in hand the common path neither allocates nor frees; every partial tile is
    // written before the second pass reads it, so what an earlier call left in the array is never seen
    return run_bf16(M, N, K, A, lda, B, ldb, bias, alpha, act, C, ldc, batch, plan, split_k, ws,
                    ws ? kStaticScratchBytes : 0, stream);
}

size_t gemm_epilogue_static_scratch_bytes(void) { return kStaticScratchBytes; }

ge_status_t gemm_epilogue_f32(int M, int N, int K, const float *A, int lda, const float *B, int ldb,
                              const float *bias, float alpha, ge_act_t act, float *C, int ldc,
                              int batch, void *stream)
{
    ge_status_t st = validate(M, N, K, A, lda, B, ldb, bias, (int)act, C, ldc, batch, 4);
    if (st != GE_OK) return st;
    GemmParams p = base_params(M, N, K, A, lda, B, ldb, bias, alpha, (int)act, C, ldc, batch);
    p.bytesA = 4 * (((long long)batch * M - 1) * lda + K);
    p.bytesB = 4 * (((long long)batch * K - 1) * ldb + N);
    p.splitK = 1;
    p.kPerSlice = ceil_div(K, 16) * 16;
    hipStream_t hs = (hipStream_t)stream;
    // direct-to-LDS kernel: 16-byte chunks of 4 floats must not straddle rows or the K / N edge
    const bool fast = !((((uintptr_t)A) | ((uintptr_t)B)) & 15u) && !((lda | ldb | N | K) & 3) &&
                      (long long)lda * 4 * 128 + 256 < (1ll << 31) && (long long)ldb * 4 * 16 + 1024 < (1ll << 31) &&
                      opt_force_config() != FORCE_GENERIC;
    if (fast) {
        // 128x128 tiles once they give every other CU a block, else 64x64 (more blocks, less padding)
        const long long t128 = (long long)ceil_div(M, 128) * ceil_div(N, 128) * batch;
        const bool big = t128 * 2 >= kNumCU && M >= 128 && N >= 128;
        const int bm = big ? 128 : 64;
        p.tilesM = ceil_div(M, bm);
        p.tilesN = ceil_div(N, bm);
        p.groupM = choose_group_m(p.tilesM, p.tilesN);
        const long long blocks = (long long)p.tilesM * p.tilesN * batch;
        if (blocks > 0x7fffffffll) return GE_ERR_SHAPE;
        const bool edge = (M % bm) || (N % bm) || (K % 16);
        const dim3 grid((unsigned)blocks), block(256);
        if (big) {
            if (edge) GE_LAUNCH((ge::gemm_f32_fast_kernel<128, 128, true>), grid, block, 0, hs, p);
            else      GE_LAUNCH((ge::gemm_f32_fast_kernel<128, 128, false>), grid, block, 0, hs, p);
            g_last_config = "f32_128x128x16_w4";
        } else {
            if (edge) GE_LAUNCH((ge::gemm_f32_fast_kernel<64, 64, true>), grid, block, 0, hs, p);
            else      GE_LAUNCH((ge::gemm_f32_fast_kernel<64, 64, false>), grid, block, 0, hs, p);
            g_last_config = "f32_64x64x16_w4";
        }
        if (ge_host::take_launch_error() != hipSuccess) return GE_ERR_LAUNCH;
        return GE_OK;
    }
    p.tilesM = ceil_div(M, 128);
    p.tilesN = ceil_div(N, 128);
    p.groupM = choose_group_m(p.tilesM, p.tilesN);
    const long long blocks = (long long)p.tilesM * p.tilesN * batch;
    if (blocks > 0x7fffffffll) return GE_ERR_SHAPE;
    GE_LAUNCH(ge::gemm_f32_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, hs, p);
    if (ge_host::take_launch_error() != hipSuccess) return GE_ERR_LAUNCH;
    g_last_config = "f32_generic_128x128x16";
    return GE_OK;
}

size_t gemm_epilogue_workspace_bytes(int M, int N, int K, int batch, ge_plan_t plan, int split_k)
{
    if (M < 1 || N < 1 || K < 1 || batch < 1) return 0;
    Plan pl;
    // the tile choice (hence the slice count) depends on whether the fast
    // kernels apply; report the larger of the two answers
    size_t need = 0;
    for (int fast = 0; fast < 2; ++fast) {
        if (make_plan_bf16(M, N, K, batch, fast != 0, plan, split_k, &pl) != GE_OK) continue;
        const size_t b = partial_bytes(M, N, batch, pl.splitK);
        if (b > need) need = b;
    }
    return need;
}

int gemm_epilogue_auto_split_k(int M, int N, int K, int batch)
{
    if (M < 1 || N < 1 || K < 1 || batch < 1) return 0;
    Plan pl;
    if (make_plan_bf16(M, N, K, batch, true, GE_PLAN_AUTO, 0, &pl) != GE_OK) return 0;
    return pl.splitK;
}

ge_status_t ge_release_workspace(void)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return GE_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    for (std::vector<Workspace> *list : {&g_ws, &g_ws_retired}) {
        size_t kept = 0;
        for (Workspace &w : *list) {
            if (w.dev == dev) (void)hipFree(w.ptr);
            else (*list)[kept++] = w;
        }
        list->resize(kept);
    }
    return GE_OK;
}

ge_status_t ge_set_option(const char *name, const char *value)
{
    if (!name) return GE_ERR_NULL;
    if (std::strcmp(name, "force_config") == 0) {
        const int f = parse_force(value);
        if (f < 0) return GE_ERR_CONFIG;
        g_opt_force = f;
    } else if (std::strcmp(name, "waves") == 0) {
        if (value && std::strcmp(value, "8") != 0 && std::strcmp(value, "4") != 0) return GE_ERR_CONFIG;
        g_opt_waves8 = (value && std::strcmp(value, "8") == 0) ? 1 : 0;
    } else if (std::strcmp(name, "stage_k") == 0) {
        if (value && std::strcmp(value, "32") != 0 && std::strcmp(value, "64") != 0) return GE_ERR_CONFIG;
        g_opt_stage32 = (value && std::strcmp(value, "32") == 0) ? 1 : 0;
    } else {
        return GE_ERR_CONFIG;
    }
    return GE_OK;
}

const char *ge_status_string(ge_status_t status)
{
    switch (status) {
    case GE_OK: return "ok";
    case GE_ERR_NULL: return "A, B or C is NULL";
    case GE_ERR_SHAPE: return "M, N, K and batch must be >= 1 and fit the index range";
    case GE_ERR_LD: return "leading dimension smaller than the row length";
    case GE_ERR_ACT: return "unknown activation";
    case GE_ERR_ALIGN: return "pointer not aligned to its element size";
    case GE_ERR_WORKSPACE: return "split-K workspace missing, too small, misaligned or not allocatable";
    case GE_ERR_LAUNCH: return "kernel launch failed";
    case GE_ERR_CONFIG: return "unknown plan or split count";
    case GE_ERR_EPILOGUE: return "clamp bounds out of order or unknown element type";
    }
    return "unknown status";
}

const char *ge_last_config(void) { return g_last_config; }

}  // extern "C"
