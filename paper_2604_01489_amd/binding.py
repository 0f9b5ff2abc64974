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

ACT = {"none": 0, "relu": 1, "gelu_tanh": 2}
PLAN = {"auto": 0, "direct": 1, "splitk": 2}
GE_OK = 0

SYMBOLS = ("gemm_epilogue_bf16", "gemm_epilogue_f32", "gemm_epilogue_bf16_ex",
           "gemm_epilogue_workspace_bytes", "gemm_epilogue_auto_split_k",
           "ge_release_workspace", "ge_status_string", "ge_last_config",
           "ge_probe_mfma_bf16", "ge_probe_store_f32")

_lib = None


class GemmEpilogueError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"gemm_epilogue status {status}: {message}")
        self.status = status


def load():
    """Load the shared library (built by ``paper_2604_01489_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
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
    lib.ge_probe_mfma_bf16.restype = c_int
    lib.ge_probe_mfma_bf16.argtypes = [c_void, c_void, c_int, c_int, c_void]
    lib.ge_probe_store_f32.restype = c_int
    lib.ge_probe_store_f32.argtypes = [c_void, c_size, c_float, c_void]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().ge_status_string(int(status)).decode()


def last_config() -> str:
    return load().ge_last_config().decode()


def _check(status: int):
    if status != GE_OK:
        raise GemmEpilogueError(status, status_string(status))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


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


def gemm_epilogue_bf16(M, N, K, A, lda, B, ldb, bias, alpha, act, C, ldc, batch=1, stream=None):
    """C = act(alpha*A@B + bias); A, B: device tensors of bf16 bit patterns
    (torch.bfloat16, int16 or uint16), bias/C: float32 device tensors."""
    _require_device(A, B, C, bias)
    _check(load().gemm_epilogue_bf16(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(bias), alpha,
                                     ACT[act], _ptr(C), ldc, batch, _stream_handle(stream)))


def gemm_epilogue_f32(M, N, K, A, lda, B, ldb, bias, alpha, act, C, ldc, batch=1, stream=None):
    """fp32 operands, fp32 matrix instructions."""
    _require_device(A, B, C, bias)
    _check(load().gemm_epilogue_f32(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(bias), alpha,
                                    ACT[act], _ptr(C), ldc, batch, _stream_handle(stream)))


def gemm_epilogue_bf16_ex(M, N, K, A, lda, B, ldb, bias, alpha, act, C, ldc, batch=1,
                          plan="auto", split_k=0, workspace=None, stream=None):
    _require_device(A, B, C, bias, workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().gemm_epilogue_bf16_ex(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(bias), alpha,
                                        ACT[act], _ptr(C), ldc, batch, PLAN[plan], split_k,
                                        _ptr(workspace), ws_bytes, _stream_handle(stream)))


def workspace_bytes(M, N, K, batch=1, plan="auto", split_k=0) -> int:
    return int(load().gemm_epilogue_workspace_bytes(M, N, K, batch, PLAN[plan], split_k))


def auto_split_k(M, N, K, batch=1) -> int:
    return int(load().gemm_epilogue_auto_split_k(M, N, K, batch))


def release_workspace():
    _check(load().ge_release_workspace())


def probe_mfma_bf16(operands, sink, blocks, iters, stream=None):
    """Measured ceiling: register-resident bf16 MFMA loop (include/ge_probes.h)."""
    _require_device(operands, sink)
    _check(load().ge_probe_mfma_bf16(_ptr(operands), _ptr(sink), blocks, iters, _stream_handle(stream)))


def probe_store_f32(dst, value=1.0, stream=None):
    """Measured ceiling: streaming fp32 store over all of ``dst`` (include/ge_probes.h)."""
    _require_device(dst)
    _check(load().ge_probe_store_f32(_ptr(dst), dst.numel(), value, _stream_handle(stream)))


def _require_device(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("gemm_epilogue takes device tensors only (there is no CPU path)")
