"""ctypes binding of the C-ABI library (``include/gemm_epilogue.h``).

Argument marshalling only: every step of the operator runs in the HIP kernels
of ``libgemm_epilogue.so``.  Tensors are torch device tensors used purely as
device memory; the stream is torch's current HIP stream unless one is given.
There is no CPU fallback: if the library is missing or no GPU is present the
calls raise.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgemm_epilogue.so")
PROBES_LIB_PATH = os.path.join(_HERE, "libge_probes.so")

ACT = {"none": 0, "relu": 1, "gelu_tanh": 2}
PLAN = {"auto": 0, "direct": 1, "splitk": 2}
GE_OK = 0

# what each header declares and the library that exports it
SYMBOLS = ("gemm_epilogue_bf16", "gemm_epilogue_f32", "gemm_epilogue_bf16_ex",
           "gemm_epilogue_workspace_bytes", "gemm_epilogue_auto_split_k",
           "ge_release_workspace", "ge_status_string", "ge_last_config", "ge_set_option",
           "gemm_epilogue_bf16_static", "gemm_epilogue_static_scratch_bytes",
           "gemm_epilogue_bf16_fused", "gemm_epilogue_diag_bf16", "conv2d_epilogue_bf16",
           "conv2d_epilogue_workspace_bytes", "gemm_rowsum_params_bf16", "gemm_rowsum_bf16",
           "gemm_epilogue_fused_workspace_bytes", "gemm_rowsum_params_bf16_ex", "gemm_rowsum_params_workspace_bytes")
PROBE_SYMBOLS = ("ge_probe_mfma_bf16", "ge_probe_store_f32", "ge_probe_stream_mix")

DTYPE = {"f32": 0, "bf16": 1}
STRUCTURE = {"general": 0, "lower": 1, "upper": 2, "sym_lower": 3, "sym_upper": 4}


class FusedArgs(ctypes.Structure):
    """Mirror of ``ge_fused_args_t`` (include/gemm_epilogue.h)."""
    _fields_ = [
        ("M", ctypes.c_int), ("N", ctypes.c_int), ("K", ctypes.c_int), ("batch", ctypes.c_int),
        ("A", ctypes.c_void_p), ("lda", ctypes.c_int), ("transA", ctypes.c_int),
        ("B", ctypes.c_void_p), ("ldb", ctypes.c_int), ("transB", ctypes.c_int),
        ("alpha", ctypes.c_float),
        ("row_scale", ctypes.c_void_p),
        ("bias", ctypes.c_void_p),
        ("R", ctypes.c_void_p), ("ldr", ctypes.c_int), ("r_type", ctypes.c_int), ("beta", ctypes.c_float),
        ("act", ctypes.c_int),
        ("clamp_lo", ctypes.c_float), ("clamp_hi", ctypes.c_float),
        ("C", ctypes.c_void_p), ("ldc", ctypes.c_int), ("c_type", ctypes.c_int),
        ("plan", ctypes.c_int), ("split_k", ctypes.c_int),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("a_structure", ctypes.c_int),
    ]


class ConvArgs(ctypes.Structure):
    """Mirror of ``ge_conv_args_t`` (include/gemm_epilogue.h)."""
    _fields_ = [(n, ctypes.c_int) for n in ("N", "H", "W", "Cin", "Cout", "KH", "KW", "stride_h", "stride_w",
                                            "pad_h", "pad_w", "dil_h", "dil_w")] + [
        ("X", ctypes.c_void_p), ("Wt", ctypes.c_void_p), ("alpha", ctypes.c_float), ("bias", ctypes.c_void_p),
        ("R", ctypes.c_void_p), ("r_type", ctypes.c_int), ("beta", ctypes.c_float),
        ("act", ctypes.c_int), ("clamp_lo", ctypes.c_float), ("clamp_hi", ctypes.c_float),
        ("Y", ctypes.c_void_p), ("y_type", ctypes.c_int),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


_lib = None
_probes = None


class GemmEpilogueError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"gemm_epilogue status {status}: {message}")
        self.status = status


def load():
    """Load the shared library (built by ``paper_2604_01489_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships a HIP runtime of its own.  It has to be in the process before this library is, or the
    # library binds to a second copy of the runtime that knows nothing of the devices and streams torch
    # hands over (every launch then fails with "no device").
    import torch  # noqa: F401
    path = os.environ.get("GE_LIBRARY", LIB_PATH)     # another build of the same library, for A/B timing
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: run `python -m paper_2604_01489_amd.build` first")
    lib = ctypes.CDLL(path)
    c_int, c_void, c_float, c_size = ctypes.c_int, ctypes.c_void_p, ctypes.c_float, ctypes.c_size_t
    common = [c_int, c_int, c_int, c_void, c_int, c_void, c_int, c_void, c_float, c_int,
              c_void, c_int, c_int]
    lib.gemm_epilogue_bf16.restype = c_int
    lib.gemm_epilogue_bf16.argtypes = common + [c_void]
    lib.gemm_epilogue_f32.restype = c_int
    lib.gemm_epilogue_f32.argtypes = common + [c_void]
    lib.gemm_epilogue_bf16_ex.restype = c_int
    lib.gemm_epilogue_bf16_ex.argtypes = common + [c_int, c_int, c_void, c_size, c_void]
    lib.gemm_epilogue_bf16_static.restype = c_int
    lib.gemm_epilogue_bf16_static.argtypes = common + [c_int, c_int, c_void]
    lib.gemm_epilogue_static_scratch_bytes.restype = c_size
    lib.gemm_epilogue_static_scratch_bytes.argtypes = []
    lib.gemm_epilogue_workspace_bytes.restype = c_size
    lib.gemm_epilogue_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int, c_int, c_int]
    lib.gemm_epilogue_auto_split_k.restype = c_int
    lib.gemm_epilogue_auto_split_k.argtypes = [c_int, c_int, c_int, c_int]
    lib.ge_release_workspace.restype = c_int
    lib.ge_release_workspace.argtypes = []
    lib.ge_status_string.restype = ctypes.c_char_p
    lib.ge_status_string.argtypes = [c_int]
    lib.ge_last_config.restype = ctypes.c_char_p
    lib.ge_last_config.argtypes = []
    lib.gemm_epilogue_bf16_fused.restype = c_int
    lib.gemm_epilogue_bf16_fused.argtypes = [ctypes.POINTER(FusedArgs), c_void]
    lib.conv2d_epilogue_bf16.restype = c_int
    lib.conv2d_epilogue_bf16.argtypes = [ctypes.POINTER(ConvArgs), c_void]
    lib.gemm_epilogue_diag_bf16.restype = c_int
    lib.gemm_epilogue_diag_bf16.argtypes = [c_int, c_int, c_void, c_void, c_int, c_void, c_float, c_int,
                                            c_void, c_int, c_int, c_void]
    lib.gemm_rowsum_params_bf16.restype = c_int
    lib.gemm_rowsum_params_bf16.argtypes = [c_int, c_int, c_void, c_int, c_int, c_void, c_void, c_void]
    lib.gemm_rowsum_params_bf16_ex.restype = c_int
    lib.gemm_rowsum_params_bf16_ex.argtypes = [c_int, c_int, c_void, c_int, c_int, c_void, c_void, c_void, c_size, c_void]
    lib.gemm_rowsum_params_workspace_bytes.restype = c_size
    lib.gemm_rowsum_params_workspace_bytes.argtypes = [c_int, c_int, c_int]
    lib.gemm_epilogue_fused_workspace_bytes.restype = c_size
    lib.gemm_epilogue_fused_workspace_bytes.argtypes = [ctypes.POINTER(FusedArgs)]
    lib.gemm_rowsum_bf16.restype = c_int
    lib.gemm_rowsum_bf16.argtypes = [c_int, c_int, c_void, c_int, c_void, c_float, c_void, c_void]
    lib.conv2d_epilogue_workspace_bytes.restype = c_size
    lib.conv2d_epilogue_workspace_bytes.argtypes = [ctypes.POINTER(ConvArgs)]
    lib.ge_set_option.restype = c_int
    lib.ge_set_option.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
    _lib = lib
    return lib


def load_probes():
    """Load the measurement probes (``include/ge_probes.h``), a library of their own."""
    global _probes
    if _probes is not None:
        return _probes
    if not os.path.exists(PROBES_LIB_PATH):
        raise FileNotFoundError(
            f"{PROBES_LIB_PATH} is missing: run `python -m paper_2604_01489_amd.build` first")
    import torch  # noqa: F401  (as in load(): torch's HIP runtime first)
    lib = ctypes.CDLL(PROBES_LIB_PATH)
    c_int, c_void, c_float, c_size = ctypes.c_int, ctypes.c_void_p, ctypes.c_float, ctypes.c_size_t
    lib.ge_probe_mfma_bf16.restype = c_int
    lib.ge_probe_mfma_bf16.argtypes = [c_void, c_void, c_int, c_int, c_void]
    lib.ge_probe_store_f32.restype = c_int
    lib.ge_probe_store_f32.argtypes = [c_void, c_size, c_float, c_void]
    lib.ge_probe_stream_mix.restype = c_int
    lib.ge_probe_stream_mix.argtypes = [c_void, c_void, c_size, c_int, c_int, c_void]
    _probes = lib
    return lib


def set_option(name: str, value=None):
    """``ge_set_option``: a switch for timing runs and tests ("force_config", "waves", "stage_k");
    ``None`` restores the default."""
    _check(load().ge_set_option(name.encode(), None if value is None else str(value).encode()))


def status_string(status: int) -> str:
    return load().ge_status_string(int(status)).decode()


def last_config() -> str:
    return load().ge_last_config().decode()


def _check(status: int):
    if status != GE_OK:
        raise GemmEpilogueError(status, status_string(status))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _addr(t):
    return None if t is None else int(t.data_ptr())


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def raw_call(name, M, N, K, A_ptr, lda, B_ptr, ldb, bias_ptr, alpha, act, C_ptr, ldc, batch,
             stream_ptr=None, extra=()):
    """Call an entry point with plain integers as pointers; returns the status.
    Used by the host-side argument validation tests (no GPU needed for error paths)."""
    fn = getattr(load(), name)
    return int(fn(M, N, K, A_ptr, lda, B_ptr, ldb, bias_ptr, alpha, act, C_ptr, ldc, batch,
                  *extra, stream_ptr))


def _require_extent(t, rows, cols, ld, batch=1, what="operand"):
    """The tensor must hold what the sizes describe: batch*rows rows of `ld` elements, the last one
    `cols` long.  A wrong size here would otherwise become an out-of-bounds access on the device."""
    if t is None:
        return
    need = (int(batch) * int(rows) - 1) * int(ld) + int(cols)
    if rows >= 1 and cols >= 1 and batch >= 1 and ld >= cols and t.numel() < need:
        raise ValueError(f"{what}: tensor holds {t.numel()} elements, the sizes describe {need}")


def gemm_epilogue_bf16(M, N, K, A, lda, B, ldb, bias, alpha, act, C, ldc, batch=1, stream=None):
    """C = act(alpha*A@B + bias); A, B: device tensors of bf16 bit patterns
    (torch.bfloat16, int16 or uint16), bias/C: float32 device tensors."""
    _require_device(A, B, C, bias)
    _require_operands(M, N, K, A, lda, B, ldb, bias, C, ldc, batch)
    _check(load().gemm_epilogue_bf16(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(bias), alpha,
                                     ACT[act], _ptr(C), ldc, batch, _stream_handle(stream)))


def gemm_epilogue_f32(M, N, K, A, lda, B, ldb, bias, alpha, act, C, ldc, batch=1, stream=None):
    """fp32 operands, fp32 matrix instructions."""
    _require_device(A, B, C, bias)
    _require_operands(M, N, K, A, lda, B, ldb, bias, C, ldc, batch)
    _check(load().gemm_epilogue_f32(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(bias), alpha,
                                    ACT[act], _ptr(C), ldc, batch, _stream_handle(stream)))


def gemm_epilogue_bf16_ex(M, N, K, A, lda, B, ldb, bias, alpha, act, C, ldc, batch=1,
                          plan="auto", split_k=0, workspace=None, stream=None):
    _require_device(A, B, C, bias, workspace)
    _require_operands(M, N, K, A, lda, B, ldb, bias, C, ldc, batch)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().gemm_epilogue_bf16_ex(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(bias), alpha,
                                        ACT[act], _ptr(C), ldc, batch, PLAN[plan], split_k,
                                        _ptr(workspace), ws_bytes, _stream_handle(stream)))


def _require_operands(M, N, K, A, lda, B, ldb, bias, C, ldc, batch, transA=False, transB=False, R=None, ldr=0):
    _require_extent(A, K if transA else M, M if transA else K, lda, batch, "A")
    _require_extent(B, N if transB else K, K if transB else N, ldb, batch, "B")
    _require_extent(C, M, N, ldc, batch, "C")
    _require_extent(R, M, N, ldr, batch, "R")
    _require_extent(bias, 1, N, N, 1, "bias")


def gemm_epilogue_bf16_static(M, N, K, A, lda, B, ldb, bias, alpha, act, C, ldc, batch=1,
                              plan="auto", split_k=0, stream=None):
    """``gemm_epilogue_bf16_ex`` for callers that cannot allocate: split-K partials go to the
    library's fixed array of device memory (``static_scratch_bytes()``)."""
    _require_device(A, B, C, bias)
    _require_operands(M, N, K, A, lda, B, ldb, bias, C, ldc, batch)
    _check(load().gemm_epilogue_bf16_static(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(bias), alpha,
                                            ACT[act], _ptr(C), ldc, batch, PLAN[plan], split_k,
                                            _stream_handle(stream)))


def static_scratch_bytes() -> int:
    return int(load().gemm_epilogue_static_scratch_bytes())


def workspace_bytes(M, N, K, batch=1, plan="auto", split_k=0) -> int:
    return int(load().gemm_epilogue_workspace_bytes(M, N, K, batch, PLAN[plan], split_k))


def auto_split_k(M, N, K, batch=1) -> int:
    return int(load().gemm_epilogue_auto_split_k(M, N, K, batch))


def release_workspace():
    _check(load().ge_release_workspace())


def fused_args(M, N, K, A_ptr, lda, B_ptr, ldb, C_ptr, ldc, *, batch=1, transA=False, transB=False,
               alpha=1.0, row_scale_ptr=None, bias_ptr=None, R_ptr=None, ldr=0, r_type="f32", beta=1.0,
               act="none", clamp=None, c_type="f32", plan="auto", split_k=0, workspace_ptr=None,
               workspace_bytes=0, a_structure="general") -> FusedArgs:
    """Fill a ``ge_fused_args_t`` from raw addresses (no checks: that is the library's job)."""
    lo, hi = (-float("inf"), float("inf")) if clamp is None else clamp
    return FusedArgs(M, N, K, batch, A_ptr, lda, int(bool(transA)), B_ptr, ldb, int(bool(transB)),
                     alpha, row_scale_ptr, bias_ptr, R_ptr, ldr, DTYPE[r_type], beta,
                     ACT[act] if isinstance(act, str) else int(act), lo, hi,
                     C_ptr, ldc, DTYPE[c_type] if isinstance(c_type, str) else int(c_type),
                     PLAN[plan] if isinstance(plan, str) else int(plan), split_k,
                     workspace_ptr, workspace_bytes,
                     STRUCTURE[a_structure] if isinstance(a_structure, str) else int(a_structure))


def fused_workspace_bytes(args: FusedArgs) -> int:
    return int(load().gemm_epilogue_fused_workspace_bytes(ctypes.byref(args)))


def raw_fused(args: FusedArgs, stream_handle=None) -> int:
    """The status code of ``gemm_epilogue_bf16_fused`` (for argument-error tests)."""
    return int(load().gemm_epilogue_bf16_fused(ctypes.byref(args), stream_handle))


def gemm_epilogue_bf16_fused(M, N, K, A, lda, B, ldb, C, ldc, *, batch=1, transA=False, transB=False,
                             alpha=1.0, row_scale=None, bias=None, residual=None, ldr=0, beta=1.0,
                             act="none", clamp=None, plan="auto", split_k=0, workspace=None, stream=None,
                             a_structure="general"):
    """``C = round(clamp(act(alpha*row_scale[m]*(opA(A) @ opB(B)) + bias[n] + beta*R)))`` on device
    tensors.  A and B hold bf16 bits (int16/uint16/bfloat16 tensors); the output type follows
    ``C.dtype`` (float32 or bfloat16/int16), the residual's its tensor's.  ``a_structure``:
    "general", or the caller's promise that opA(A) is "lower" / "upper" triangular."""
    import torch
    _require_device(A, B, C, row_scale, bias, residual, workspace)
    _require_operands(M, N, K, A, lda, B, ldb, bias, C, ldc, batch, transA, transB, residual, ldr)
    _require_extent(row_scale, 1, M, M, 1, "row_scale")

    def kind(t):
        return "f32" if t.dtype == torch.float32 else "bf16"

    args = fused_args(M, N, K, _addr(A), lda, _addr(B), ldb, _addr(C), ldc, batch=batch, transA=transA,
                      transB=transB, alpha=alpha, row_scale_ptr=_addr(row_scale), bias_ptr=_addr(bias),
                      R_ptr=_addr(residual), ldr=ldr, r_type=kind(residual) if residual is not None else "f32",
                      beta=beta, act=act, clamp=clamp, c_type=kind(C), plan=plan, split_k=split_k,
                      workspace_ptr=_addr(workspace),
                      workspace_bytes=0 if workspace is None else workspace.numel() * workspace.element_size(),
                      a_structure=a_structure)
    _check(load().gemm_epilogue_bf16_fused(ctypes.byref(args), _stream_handle(stream)))


def conv_args(shape, X_ptr, Wt_ptr, Y_ptr, *, stride=(1, 1), pad=(0, 0), dil=(1, 1), alpha=1.0, bias_ptr=None,
              R_ptr=None, r_type="f32", beta=1.0, act="none", clamp=None, y_type="f32", workspace_ptr=None,
              workspace_bytes=0) -> ConvArgs:
    """Fill a ``ge_conv_args_t`` from raw addresses; ``shape`` = (N, H, W, Cin, Cout, KH, KW)."""
    lo, hi = (-float("inf"), float("inf")) if clamp is None else clamp
    return ConvArgs(*shape, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1], X_ptr, Wt_ptr, alpha, bias_ptr,
                    R_ptr, DTYPE[r_type], beta, ACT[act] if isinstance(act, str) else int(act), lo, hi, Y_ptr,
                    DTYPE[y_type] if isinstance(y_type, str) else int(y_type), workspace_ptr, workspace_bytes)


def conv_workspace_bytes(args: ConvArgs) -> int:
    return int(load().conv2d_epilogue_workspace_bytes(ctypes.byref(args)))


def raw_conv(args: ConvArgs) -> int:
    """The status code of ``conv2d_epilogue_bf16`` (for argument-error tests)."""
    return int(load().conv2d_epilogue_bf16(ctypes.byref(args), None))


def conv2d_epilogue_bf16(X, Wt, Y, *, stride=(1, 1), pad=(0, 0), dil=(1, 1), alpha=1.0, bias=None, residual=None,
                         beta=1.0, act="none", clamp=None, workspace=None, stream=None):
    """Channels-last convolution with the fused consumer chain on device tensors: ``X`` [N,H,W,Cin] and
    ``Wt`` [Cout,KH,KW,Cin] hold bf16 (bits), ``Y`` [N,OH,OW,Cout] is float32 or bfloat16."""
    import torch
    _require_device(X, Wt, Y, bias, residual, workspace)

    def kind(t):
        return "f32" if t.dtype == torch.float32 else "bf16"

    Nb, H, W, Cin = X.shape
    Cout, KH, KW, _ = Wt.shape
    args = conv_args((Nb, H, W, Cin, Cout, KH, KW), _addr(X), _addr(Wt), _addr(Y), stride=stride, pad=pad, dil=dil,
                     alpha=alpha, bias_ptr=_addr(bias), R_ptr=_addr(residual),
                     r_type=kind(residual) if residual is not None else "f32", beta=beta, act=act, clamp=clamp,
                     y_type=kind(Y), workspace_ptr=_addr(workspace),
                     workspace_bytes=0 if workspace is None else workspace.numel() * workspace.element_size())
    _check(load().conv2d_epilogue_bf16(ctypes.byref(args), _stream_handle(stream)))


def gemm_epilogue_diag_bf16(M, N, d, B, ldb, bias, alpha, act, C, ldc, batch=1, stream=None):
    """``C = act(alpha * d[m] * B + bias[n])``: the operator with A = diag(d), on device tensors."""
    _require_device(d, B, bias, C)
    _check(load().gemm_epilogue_diag_bf16(M, N, _ptr(d), _ptr(B), ldb, _ptr(bias), alpha, ACT[act], _ptr(C), ldc,
                                          batch, _stream_handle(stream)))


def raw_diag(M, N, d_ptr, B_ptr, ldb, bias_ptr, alpha, act, C_ptr, ldc, batch) -> int:
    """The status code of ``gemm_epilogue_diag_bf16`` (for argument-error tests)."""
    return int(load().gemm_epilogue_diag_bf16(M, N, d_ptr, B_ptr, ldb, bias_ptr, alpha, act, C_ptr, ldc, batch, None))


def gemm_rowsum_params_bf16(N, K, B, ldb, transB, bias, params, workspace=None, stream=None):
    """``params[k] = sum_n opB(B)[k, n]`` for k < K, ``params[K] = sum(bias)``: the parameter-only part of
    the row sum of a linear layer, on device tensors."""
    _require_device(B, bias, params, workspace)
    _require_extent(B, N if transB else K, K if transB else N, ldb, 1, "B")
    _require_extent(params, 1, K + 1, K + 1, 1, "params")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().gemm_rowsum_params_bf16_ex(N, K, _ptr(B), ldb, int(bool(transB)), _ptr(bias), _ptr(params),
                                             _ptr(workspace), ws_bytes, _stream_handle(stream)))


def rowsum_params_workspace_bytes(N, K, transB) -> int:
    return int(load().gemm_rowsum_params_workspace_bytes(N, K, int(bool(transB))))


def gemm_rowsum_bf16(M, K, A, lda, params, alpha, y, stream=None):
    """``y[m] = alpha * sum_k A[m, k] * params[k] + params[K]``: the row sum of the layer's output."""
    _require_device(A, params, y)
    _check(load().gemm_rowsum_bf16(M, K, _ptr(A), lda, _ptr(params), alpha, _ptr(y), _stream_handle(stream)))


def raw_rowsum_params(N, K, B_ptr, ldb, transB, bias_ptr, params_ptr) -> int:
    """Status code of ``gemm_rowsum_params_bf16`` (for argument-error tests)."""
    return int(load().gemm_rowsum_params_bf16(N, K, B_ptr, ldb, transB, bias_ptr, params_ptr, None))


def raw_rowsum(M, K, A_ptr, lda, params_ptr, alpha, y_ptr) -> int:
    """Status code of ``gemm_rowsum_bf16`` (for argument-error tests)."""
    return int(load().gemm_rowsum_bf16(M, K, A_ptr, lda, params_ptr, alpha, y_ptr, None))


def probe_mfma_bf16(operands, sink, blocks, iters, stream=None):
    """Measured ceiling: register-resident bf16 MFMA loop (include/ge_probes.h)."""
    _require_device(operands, sink)
    _check(load_probes().ge_probe_mfma_bf16(_ptr(operands), _ptr(sink), blocks, iters, _stream_handle(stream)))


def probe_store_f32(dst, value=1.0, stream=None):
    """Measured ceiling: streaming fp32 store over all of ``dst`` (include/ge_probes.h)."""
    _require_device(dst)
    _check(load_probes().ge_probe_store_f32(_ptr(dst), dst.numel(), value, _stream_handle(stream)))


def probe_stream_mix(src, dst, trips, reads, writes, stream=None):
    """Measured ceiling: a stream of ``trips`` steps that each read ``reads`` and write ``writes``
    16-byte pieces (include/ge_probes.h)."""
    _require_device(src, dst)
    nbytes = lambda t: 0 if t is None else t.numel() * t.element_size()
    if nbytes(src) < trips * reads * 16 or nbytes(dst) < max(trips * writes * 16, 16):
        raise ValueError("probe buffer too small for the trips asked for")
    _check(load_probes().ge_probe_stream_mix(_ptr(src), _ptr(dst), trips, reads, writes, _stream_handle(stream)))


def _require_device(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("gemm_epilogue takes device tensors only (there is no CPU path)")
