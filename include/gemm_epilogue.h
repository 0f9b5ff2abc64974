/*
 * gemm_epilogue -- fused dense matrix multiply for AMD MI355X (CDNA4, gfx950).
 *
 *     C[b][m,n] = act( alpha * sum_{k<K} A[b][m,k] * B[b][k,n] + bias[n] )
 *
 * The contraction is the plain row-major matmul of the paper's naive baseline
 * (appendix "Comparison of CuTe and CUDA Representations for Square GEMM",
 * Fig. simp_cuda): A is [M,K] row-major, B is [K,N] row-major, C is [M,N]
 * row-major, the operand convention of the optimisation prompt's GEMM section.
 * The writeback adds no previous C (beta = 0, as in the epilogue of the initial
 * CuTe kernel, Fig. simple_cute) and applies scale, bias and activation in
 * registers before the single store (Level-2 optimisation prompt, "Fusion":
 * bias/add/scale/activation fused into the producer writeback).  Operand
 * precision is never lowered (Experiments, "Manual Correctness Audit"): bf16
 * operands are multiplied exactly and accumulated in fp32; fp32 operands use
 * true fp32 matrix instructions.
 *
 * Layout.  All matrices are row-major with a leading dimension in ELEMENTS:
 *     A[m,k] = A[m*lda + k],  B[k,n] = B[k*ldb + n],  C[m,n] = C[m*ldc + n].
 * Batch b starts at A + b*M*lda, B + b*K*ldb, C + b*M*ldc (packed strides);
 * bias (length N) is shared by every batch.
 *
 * Ownership.  Every pointer is a DEVICE pointer owned by the caller and must
 * stay valid until the work enqueued on `stream` has finished.  The calls
 * enqueue kernels on `stream` (a hipStream_t passed as void*, NULL = the
 * default stream) and return without synchronising.  C must not overlap A, B
 * or bias.  bf16 values are passed as their 16-bit patterns so this header
 * needs no HIP types.
 *
 * Partial results.  Plans that slice K (and the column-sum pass of
 * gemm_rowsum_params_bf16) park fp32 partial results in a workspace.  A call
 * that takes a `workspace` argument and is given one allocates nothing.
 * Otherwise the library keeps one buffer per (device, stream): the first call
 * on a stream that needs a larger one than that stream has had calls hipMalloc
 * (which may take time but does not wait for the device); a buffer that was
 * handed out is never freed or moved before ge_release_workspace, so work
 * already enqueued, and graphs already captured, keep a valid address.  A
 * stream that is being captured is refused such a first allocation
 * (GE_ERR_WORKSPACE): run the call once on that stream before capturing, or
 * pass a workspace.  Calls on different streams use different buffers; calls
 * on one stream are ordered by it.
 *
 * Errors.  Every call validates its arguments first and returns a status; on
 * any status other than GE_OK nothing was enqueued and C is untouched.
 *
 * Determinism.  For a fixed library build, device and argument list the result
 * is bitwise repeatable, including the split-K path (partials are summed in
 * slice order by a second kernel; no atomics).
 */
#ifndef GEMM_EPILOGUE_H
#define GEMM_EPILOGUE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GE_ACT_NONE = 0,      /* v                                                      */
    GE_ACT_RELU = 1,      /* v > 0 ? v : 0                                          */
    GE_ACT_GELU_TANH = 2  /* 0.5 v (1 + tanh( sqrt(2/pi) (v + 0.044715 v^3) ))      */
} ge_act_t;

typedef enum {
    GE_OK = 0,
    GE_ERR_NULL = 1,       /* A, B or C is NULL                                     */
    GE_ERR_SHAPE = 2,      /* M, N, K or batch < 1, or a product overflows          */
    GE_ERR_LD = 3,         /* lda < K, ldb < N or ldc < N                           */
    GE_ERR_ACT = 4,        /* act is not a ge_act_t value                           */
    GE_ERR_ALIGN = 5,      /* a pointer is not aligned to its element size          */
    GE_ERR_WORKSPACE = 6,  /* split-K workspace missing, too small or not allocatable */
    GE_ERR_LAUNCH = 7,     /* the HIP runtime refused a launch                      */
    GE_ERR_CONFIG = 8,     /* unknown plan / forced configuration does not fit      */
    GE_ERR_EPILOGUE = 9    /* clamp_lo > clamp_hi (or NaN), or an unknown element type */
} ge_status_t;

/* How the work is decomposed (the paper's design choice "work decomposition and
 * tiling across thread blocks and warps", Introduction; split-K and the skinny
 * rule are items 7 and 9 of the optimisation prompt's GEMM list).            */
typedef enum {
    GE_PLAN_AUTO = 0,      /* choose from the shape                                 */
    GE_PLAN_DIRECT = 1,    /* one pass, epilogue in the GEMM kernel                 */
    GE_PLAN_SPLITK = 2     /* K sliced over blocks, partials reduced in slice order */
} ge_plan_t;

/*
 * bf16 operands, fp32 accumulation, fp32 output.
 *   M, N, K >= 1      problem size per batch
 *   A, lda            device, bf16 bits, lda >= K
 *   B, ldb            device, bf16 bits, ldb >= N
 *   bias              device, fp32[N], or NULL for no bias
 *   alpha             scale applied to the accumulated product
 *   act               activation
 *   C, ldc            device, fp32, ldc >= N; only C[m, 0..N) is written
 *   batch >= 1        number of independent problems (packed strides)
 *   stream            hipStream_t
 * Fast kernels (direct-to-LDS loads) need A and B 16-byte aligned, lda, ldb, N
 * and K multiples of 8; any other legal argument list takes a guarded generic
 * kernel with the same result contract (the coding and debugging guide's rule
 * for vectorised copies: gated by alignment, with a correct fallback).  Large-K
 * small-MN shapes use split-K with the library's workspace of the stream (see
 * "Partial results" above).
 */
ge_status_t gemm_epilogue_bf16(int M, int N, int K,
                               const uint16_t *A, int lda,
                               const uint16_t *B, int ldb,
                               const float *bias, float alpha, ge_act_t act,
                               float *C, int ldc, int batch, void *stream);

/* fp32 operands, fp32 matrix instructions, fp32 output.  Same contract.  A product whose tiles
 * would leave more than half of the CUs idle and whose K is long is sliced over K and summed in slice
 * order (bitwise repeatable); this call has no workspace argument, so its partial sums always go to
 * the library's buffer of the stream (see "Partial results" above: inside a stream capture such a
 * call needs one earlier call of the same size on that stream, else GE_ERR_WORKSPACE). */
ge_status_t gemm_epilogue_f32(int M, int N, int K,
                              const float *A, int lda,
                              const float *B, int ldb,
                              const float *bias, float alpha, ge_act_t act,
                              float *C, int ldc, int batch, void *stream);

/*
 * Same operator with explicit control:
 *   plan, split_k     GE_PLAN_AUTO picks both; GE_PLAN_SPLITK uses `split_k`
 *                     slices (>= 2, or 0 to let the library choose)
 *   workspace         device buffer for split-K partials, 256-byte aligned, of
 *                     at least gemm_epilogue_workspace_bytes(...) bytes; NULL
 *                     selects the library-owned buffer
 * Never allocates when `workspace` is given.
 */
ge_status_t gemm_epilogue_bf16_ex(int M, int N, int K,
                                  const uint16_t *A, int lda,
                                  const uint16_t *B, int ldb,
                                  const float *bias, float alpha, ge_act_t act,
                                  float *C, int ldc, int batch,
                                  ge_plan_t plan, int split_k,
                                  void *workspace, size_t workspace_bytes,
                                  void *stream);

/*
 * gemm_epilogue_bf16_ex for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same operator, same kernels and the same bits as gemm_epilogue_bf16_ex; split-K
 * partials go to a fixed array of gemm_epilogue_static_scratch_bytes() = 64 MiB of device
 * memory that is part of the library's code object (every GPU the library runs on holds
 * its own copy until the process ends).  The call allocates and frees nothing, on the host
 * side of the HIP runtime or on the device; the first call on a device only asks the
 * runtime for the array's address.
 *   A plan whose partial tiles (split_k * batch * M * N * 4 bytes) exceed the array
 *   returns GE_ERR_WORKSPACE and enqueues nothing.
 *   Every partial tile is written before it is read, so nothing has to be cleared between
 *   calls; but all calls on one GPU share the one array: calls that overlap in time on
 *   the same GPU (different streams, or replays of graphs in flight together) race.
 * Errors: as gemm_epilogue_bf16_ex.
 */
ge_status_t gemm_epilogue_bf16_static(int M, int N, int K,
                                      const uint16_t *A, int lda,
                                      const uint16_t *B, int ldb,
                                      const float *bias, float alpha, ge_act_t act,
                                      float *C, int ldc, int batch,
                                      ge_plan_t plan, int split_k, void *stream);
size_t gemm_epilogue_static_scratch_bytes(void);

/*
 * The widened operator (bf16 operands, fp32 accumulation):
 *
 *     P[b][m,n] = sum_{k<K} opA(A[b])[m,k] * opB(B[b])[k,n]
 *     v         = alpha * row_scale[m] * P[b][m,n] + bias[n] + beta * R[b][m,n]
 *     C[b][m,n] = round( min(max(act(v), clamp_lo), clamp_hi) )
 *
 * The consumer chain after the product is what the Level-2 optimisation prompt
 * asks to fold into the producer's writeback ("Fusion": bias / add / scale /
 * activation; "clamp" in its list of consumer operations): computed on the
 * accumulator in registers, C written once.  opA / opB choose how an operand is
 * STORED, not what is computed (the strided, transposed operand views of the
 * initial CuTe kernel, Fig. simple_cute): the matrix instruction sees the same
 * fragments either way.  With A = I and row_scale = d the operator is
 * diag(d) * B, the paper's diagonal-matrix multiply.  The order of the chain,
 * the broadcast axes and beta are this library's reading; the paper names the
 * operations only.
 *
 *   M, N, K, batch >= 1
 *   A, lda, transA    device, bf16 bits.  transA = 0: A[m,k] = A[m*lda + k], lda >= K;
 *                     transA != 0: A[m,k] = A[k*lda + m], lda >= M
 *   B, ldb, transB    device, bf16 bits.  transB = 0: B[k,n] = B[k*ldb + n], ldb >= N;
 *                     transB != 0: B[k,n] = B[n*ldb + k], ldb >= K
 *   alpha             scale of the product
 *   row_scale         device, fp32[M], or NULL (= 1); multiplies the scaled product of
 *                     row m, not the bias; shared by every batch
 *   bias              device, fp32[N], or NULL; shared by every batch
 *   R, ldr, r_type    device residual [M, ldr >= N] per batch of r_type elements, or NULL;
 *   beta              scale of the residual (ignored when R is NULL)
 *   act               activation, applied after the residual
 *   clamp_lo/hi       clamp_lo <= clamp_hi, applied after the activation;
 *                     -INFINITY / +INFINITY switch a side off
 *   C, ldc, c_type    device result [M, ldc >= N] per batch; GE_DTYPE_BF16 rounds the fp32
 *                     value to nearest-even.  Only C[m, 0..N) is written
 *   plan, split_k, workspace, workspace_bytes   as for gemm_epilogue_bf16_ex
 *   a_structure       what the caller knows about opA(A) (optimisation prompt, "Rules for GEMM":
 *                     use a stated characteristic of an operand, never an assumed one):
 *                     GE_A_GENERAL nothing; GE_A_LOWER: opA(A)[m,k] == 0 for k > m;
 *                     GE_A_UPPER: opA(A)[m,k] == 0 for k < m.  A promise about the VALUES, in
 *                     every batch: the operand is still a full M x K array holding those zeros,
 *                     the result is that of the general call bit for bit, and the library skips
 *                     the K ranges in which a whole tile row of A is zero (about half the
 *                     multiply-adds of a square product).  With a false promise the skipped
 *                     terms are missing from the result.  Not with GE_PLAN_SPLITK.
 *                     GE_A_SYM_LOWER / GE_A_SYM_UPPER (same prompt: a symmetric operand's reads can be
 *                     reduced): A is a symmetric K x K matrix (M == K, transA == 0) GIVEN BY ONE
 *                     TRIANGLE of the array: S[m,k] = A[m*lda + k] for k <= m (lower; k >= m for upper)
 *                     and S[m,k] = S[k,m] otherwise; the operator is computed with S in place of
 *                     opA(A).  No element of the other triangle enters the result, whatever it holds
 *                     (the array must still be allocated in full: M rows of lda).  With N <= 32, M >= 512 a
 *                     multiple of 8, A 16-byte aligned and lda a multiple of 8 every element of the
 *                     stored triangle is fetched from memory once (the product is a stream of A there, so
 *                     that halves its time: a kernel of its own, whose partial results go to the
 *                     workspace, gemm_epilogue_fused_workspace_bytes of it); any other legal argument list
 *                     takes the guarded kernel with the same result contract.  plan and split_k are
 *                     honoured by the guarded kernel only.
 * Batches are packed: A advances by (transA ? K : M)*lda elements, B by
 * (transB ? N : K)*ldb, R by M*ldr, C by M*ldc.  C must not overlap any input.
 *
 * `args` is a HOST pointer, read before the call returns.  The direct-to-LDS
 * kernels need A and B 16-byte aligned, lda and ldb multiples of 8 and the row
 * payloads (K or M for A, N or K for B) multiples of 8, plus for bf16 output an
 * even N and ldc and a 4-byte aligned C; any other legal argument list takes a
 * guarded kernel with the same result contract.
 * Errors: as gemm_epilogue_bf16, plus GE_ERR_EPILOGUE.
 */
typedef enum { GE_DTYPE_F32 = 0, GE_DTYPE_BF16 = 1 } ge_dtype_t;
typedef enum { GE_A_GENERAL = 0, GE_A_LOWER = 1, GE_A_UPPER = 2, GE_A_SYM_LOWER = 3, GE_A_SYM_UPPER = 4 } ge_structure_t;

typedef struct ge_fused_args {
    int M, N, K, batch;
    const uint16_t *A; int lda; int transA;
    const uint16_t *B; int ldb; int transB;
    float alpha;
    const float *row_scale;
    const float *bias;
    const void *R; int ldr; ge_dtype_t r_type; float beta;
    ge_act_t act;
    float clamp_lo, clamp_hi;
    void *C; int ldc; ge_dtype_t c_type;
    ge_plan_t plan; int split_k;
    void *workspace; size_t workspace_bytes;
    ge_structure_t a_structure;
} ge_fused_args_t;

ge_status_t gemm_epilogue_bf16_fused(const ge_fused_args_t *args, void *stream);

/* Bytes of workspace gemm_epilogue_bf16_fused needs for these arguments (0 when it runs in one
 * pass, or when the arguments are not valid).  Reads sizes, flags and the alignment of the pointers
 * only.  Host only. */
size_t gemm_epilogue_fused_workspace_bytes(const ge_fused_args_t *args);

/*
 * Convolution front-end of the fused operator (bf16 operands, fp32 accumulation), channels-last:
 *
 *     S[n,oh,ow,co] = sum_{kh,kw,c} X[n, oh*stride_h - pad_h + kh*dil_h,
 *                                        ow*stride_w - pad_w + kw*dil_w, c] * Wt[co,kh,kw,c]
 *     Y[n,oh,ow,co] = round( min(max(act(alpha*S + bias[co] + beta*R[n,oh,ow,co]), clamp_lo), clamp_hi) )
 *
 * X is read as zero outside [0,H) x [0,W); OH = (H + 2 pad_h - dil_h (KH-1) - 1) / stride_h + 1,
 * OW likewise.  This is the cross-correlation deep-learning frameworks call convolution,
 * evaluated as the implicit GEMM of the paper's convolution guidance (optimisation prompt,
 * convolution section: output positions x output channels, K = KH*KW*Cin, the im2col tile
 * gathered on the fly) on the same matrix-instruction core and with the same fused consumer
 * chain as gemm_epilogue_bf16_fused.  Channels-last storage is this library's reading: 8
 * consecutive channels of one tap are then 16 contiguous bytes.
 *
 *   X                 device, bf16 bits, [N, H, W, Cin] packed
 *   Wt                device, bf16 bits, [Cout, KH, KW, Cin] packed
 *   bias              device, fp32[Cout] or NULL
 *   R, r_type, beta   device residual [N, OH, OW, Cout] packed, or NULL
 *   Y, y_type         device result [N, OH, OW, Cout] packed; GE_DTYPE_BF16 rounds to nearest-even
 *   the other fields  as in ge_fused_args_t
 * `args` is a HOST pointer, read before the call returns.  The gathering kernel needs X and
 * Wt 16-byte aligned, Cin a multiple of 32, Cout a multiple of 8, an input smaller than
 * 2 GiB and (for bf16 output) Y 16-byte aligned; any other legal argument list takes a guarded
 * kernel with the same result contract.  Shapes with few output tiles and a long K are split
 * over K and summed in slice order (bitwise repeatable); the partial results go to `workspace`
 * (256-byte aligned, at least conv2d_epilogue_workspace_bytes(args) bytes) or, when it is NULL,
 * to the library's buffer of the stream (see "Partial results" above).
 * Errors: GE_ERR_NULL, GE_ERR_SHAPE (a size < 1, an empty output, index ranges), GE_ERR_ACT,
 * GE_ERR_EPILOGUE, GE_ERR_ALIGN, GE_ERR_WORKSPACE, GE_ERR_LAUNCH.
 */
typedef struct ge_conv_args {
    int N, H, W, Cin, Cout, KH, KW;
    int stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
    const uint16_t *X;
    const uint16_t *Wt;
    float alpha;
    const float *bias;
    const void *R; ge_dtype_t r_type; float beta;
    ge_act_t act;
    float clamp_lo, clamp_hi;
    void *Y; ge_dtype_t y_type;
    void *workspace; size_t workspace_bytes;
} ge_conv_args_t;

ge_status_t conv2d_epilogue_bf16(const ge_conv_args_t *args, void *stream);

/* Bytes of workspace the convolution needs for these sizes (0 when it runs in one pass, or
 * when the sizes are not valid).  Host only; reads the sizes and pointers' alignment only. */
size_t conv2d_epilogue_workspace_bytes(const ge_conv_args_t *args);

/*
 * Structured operand: A = diag(d), an M x M matrix given by its diagonal.
 *
 *     C[b][m,n] = act( alpha * d[m] * B[b][m,n] + bias[n] )
 *
 * This is gemm_epilogue_bf16 with A = diag(d) (equally: the widened operator with
 * A = I and row_scale = d) computed without the M*M*N products that are zero.
 * The paper's optimisation prompt asks to exploit a known operand structure
 * ("Rules for GEMM": use specific characteristics of the input matrices), and
 * its largest matmul speedup is this diagonal-matrix multiply (Experiments,
 * "Variance of Speedup Results").  The work left is one scaled copy of B:
 * bound by HBM, 2 bytes read and 4 written per output.
 *   M, N, batch >= 1
 *   d                 device, fp32[M], shared by every batch
 *   B, ldb            device, bf16 bits, [M, ldb >= N] per batch (packed: M*ldb)
 *   bias              device, fp32[N] or NULL
 *   C, ldc            device, fp32 [M, ldc >= N] per batch; only C[m, 0..N) is written
 * Errors: GE_ERR_NULL (d, B or C), GE_ERR_SHAPE, GE_ERR_LD, GE_ERR_ACT, GE_ERR_ALIGN,
 * GE_ERR_LAUNCH.  Any alignment of B and C that their element types allow is
 * accepted (16-byte row pieces when N, ldb, ldc are multiples of 4 and the
 * pointers allow it, element-wise otherwise).
 */
ge_status_t gemm_epilogue_diag_bf16(int M, int N, const float *d,
                                    const uint16_t *B, int ldb,
                                    const float *bias, float alpha, ge_act_t act,
                                    float *C, int ldc, int batch, void *stream);

/*
 * Row sum of a linear layer, without the layer's output:
 *
 *     y[m] = sum_{n<N} ( alpha * sum_{k<K} A[m,k] * opB(B)[k,n] + bias[n] )
 *          = alpha * sum_{k<K} A[m,k] * s[k] + t,     s[k] = sum_n opB(B)[k,n],  t = sum_n bias[n]
 *
 * The second line is the algebraic simplification the Level-2 optimisation prompt puts before
 * any tuning ("First priority: algebraic simplification": the sum over the output dimension of a
 * linear layer becomes x @ sum(weight) + sum(bias)); it is exact in real arithmetic and needs
 * 2 K (M + N) operations instead of 2 M N K.  s and t depend on the layer's parameters only and
 * are computed by a call of their own, to be kept for every later input (same prompt,
 * "Parameter-only reduction rule").  Both calls are bound by HBM: B is read once, then A once.
 * Sums are fp32, in a fixed order: results are repeatable bit for bit.
 *
 * gemm_rowsum_params_bf16:
 *   N, K >= 1
 *   B, ldb, transB    device, bf16 bits.  transB = 0: B[k,n] = B[k*ldb + n], ldb >= N;
 *                     transB != 0 (a weight matrix as frameworks store it): B[k,n] = B[n*ldb + k], ldb >= K
 *   bias              device, fp32[N], or NULL (t = 0)
 *   params            device, fp32[K + 1], written: s[0..K), then t
 * gemm_rowsum_bf16:
 *   M, K >= 1
 *   A, lda            device, bf16 bits, A[m,k] = A[m*lda + k], lda >= K
 *   params            device, fp32[K + 1] as written by gemm_rowsum_params_bf16
 *   y                 device, fp32[M], written
 * 16-byte row pieces are used when the pointer and leading dimension allow it, single elements
 * otherwise.  gemm_rowsum_params_bf16 with transB != 0 parks partial column sums in the library's
 * workspace of the stream (see "Partial results" at the top).
 * Errors: GE_ERR_NULL, GE_ERR_SHAPE, GE_ERR_LD, GE_ERR_ALIGN (a pointer not aligned to its
 * element), GE_ERR_WORKSPACE, GE_ERR_LAUNCH.
 */
ge_status_t gemm_rowsum_params_bf16(int N, int K, const uint16_t *B, int ldb, int transB,
                                    const float *bias, float *params, void *stream);
/* The same with a caller's workspace (256-byte aligned, at least gemm_rowsum_params_workspace_bytes(N, K,
 * transB) bytes, which is 0 for transB == 0): never allocates.  workspace == NULL selects the library's. */
ge_status_t gemm_rowsum_params_bf16_ex(int N, int K, const uint16_t *B, int ldb, int transB,
                                       const float *bias, float *params,
                                       void *workspace, size_t workspace_bytes, void *stream);
size_t gemm_rowsum_params_workspace_bytes(int N, int K, int transB);
ge_status_t gemm_rowsum_bf16(int M, int K, const uint16_t *A, int lda, const float *params,
                             float alpha, float *y, void *stream);

/* Bytes of split-K workspace the bf16 call needs for this shape with `plan` and
 * `split_k` as above (0 when the chosen plan is direct): the size depends on the
 * plan the caller is going to ask for, so the query takes the same two arguments
 * as the call.  Host only. */
size_t gemm_epilogue_workspace_bytes(int M, int N, int K, int batch,
                                     ge_plan_t plan, int split_k);

/* Number of K slices GE_PLAN_AUTO would use for the bf16 call (1 = direct).
 * Host only; needs no device. */
int gemm_epilogue_auto_split_k(int M, int N, int K, int batch);

/* Frees every library-owned workspace of the current device, outgrown ones included.
 * The caller has synchronised the streams that used them and replays no graph that
 * was captured over them.  Calls hipFree (which waits for the device). */
ge_status_t ge_release_workspace(void);

/*
 * Switches for timing runs and tests; none changes a result contract.
 *   "force_config"  "256x256" | "128x128" | "generic": block tile of the bf16 kernels
 *                   ("generic" also for fp32), whatever the planner would pick
 *   "waves"         "8": full 256 x 256 tiles stay on the eight-wave kernel ("4": default)
 *   "stage_k"       "32": no 64-k load phases in the eight-wave kernel ("64": default)
 *   "conv_halo"     "off": 3 x 3 convolutions stay on the gathering kernel; "on": the
 *                   halo-staged kernel for every shape it can take, however few tiles;
 *                   "14_11" | "12_12": that variant of it for every shape it can take
 * value == NULL restores the default.  Process-wide, effective from the next call.  The
 * initial values come from the environment variables GE_FORCE_CONFIG, GE_WAVES,
 * GE_STAGE_K and GE_CONV_HALO, read once when the library is loaded; no entry point reads the
 * environment afterwards.
 * Errors: GE_ERR_NULL (name), GE_ERR_CONFIG (unknown name or value).
 */
ge_status_t ge_set_option(const char *name, const char *value);

/* Static, never NULL. */
const char *ge_status_string(ge_status_t status);

/* Name of the kernel configuration the last successful call on this thread
 * launched ("bf16_256x256x64_w4", "bf16_256x256x32_w8", "f32_128x128x16", ...); for reports. */
const char *ge_last_config(void);

#ifdef __cplusplus
}
#endif
#endif /* GEMM_EPILOGUE_H */
