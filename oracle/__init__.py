"""CPU oracle for ``C = act(alpha * A @ B + bias)`` -- TEST INFRASTRUCTURE ONLY.

A thin ctypes loader around ``gemm_epilogue_oracle.c`` (plain C, fp64
accumulation, OpenMP over rows).  Only the tests, the smoke check and the CPU
baseline leg of the benchmark may import this package; the GPU library never
does, and the two share no code.

The operator follows the paper's plain row-major matmul definition (appendix
"Comparison of CuTe and CUDA Representations for Square GEMM", Fig. simp_cuda)
with the fused bias/scale/activation writeback of the Level-2 optimisation
prompt ("Fusion").
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_epilogue_oracle.c")
_LIB = os.path.join(_HERE, "libgemm_epilogue_oracle.so")

ACT = {"none": 0, "relu": 1, "gelu_tanh": 2}
_KIND = {np.dtype(np.float64): 0, np.dtype(np.float32): 1, np.dtype(np.uint16): 2}

_FUSED_SRC = os.path.join(_HERE, "gemm_fused_oracle.c")
_FUSED_LIB = os.path.join(_HERE, "libgemm_fused_oracle.so")
_CONV_SRC = os.path.join(_HERE, "conv_oracle.c")
_CONV_LIB = os.path.join(_HERE, "libconv_oracle.so")
_SYMM_SRC = os.path.join(_HERE, "gemm_symm_oracle.c")
_SYMM_LIB = os.path.join(_HERE, "libgemm_symm_oracle.so")
OUT = {"f64": 0, "f32": 1, "bf16": 2}

_lib = None
_fused = None
_conv = None
_symm = None


def compile_source(src: str, out: str) -> str:
    """gcc line for the oracle: no fast-math, no contraction, OpenMP."""
    cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
           "-shared", "-fPIC", "-o", out, src, "-lm"]
    subprocess.run(cmd, check=True)
    return out


def build(force: bool = False) -> str:
    """Compile the oracles that are missing or older than their source. Returns the path of the
    plain operator's library."""
    for src, lib in ((_SRC, _LIB), (_FUSED_SRC, _FUSED_LIB), (_CONV_SRC, _CONV_LIB), (_SYMM_SRC, _SYMM_LIB)):
        if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
            compile_source(src, lib)
    return _LIB


def use_library(path: str | None) -> None:
    """Point the loader at another build of the oracle (the mutation tests plant
    mistakes in copies of the source); ``None`` returns to the real one."""
    global _lib
    _lib = None if path is None else _bind(ctypes.CDLL(path))


def _bind(lib):
    lib.oracle_gemm_epilogue.restype = ctypes.c_int
    lib.oracle_gemm_epilogue.argtypes = [
        ctypes.c_int, ctypes.c_int, ctypes.c_int,
        ctypes.c_void_p, ctypes.c_long, ctypes.c_void_p, ctypes.c_long,
        ctypes.c_int, ctypes.c_void_p, ctypes.c_double, ctypes.c_int,
        ctypes.c_void_p, ctypes.c_long, ctypes.c_int]
    lib.oracle_num_threads.restype = ctypes.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(ctypes.CDLL(build()))
    return _lib


def num_threads() -> int:
    """OpenMP threads the oracle will use."""
    return int(_load().oracle_num_threads())


def gemm_epilogue(A, B, bias=None, alpha=1.0, act="none", *, M=None, N=None, K=None,
                  lda=None, ldb=None, ldc=None, batch=1):
    """Reference result as an fp64 array.

    ``A`` and ``B`` are numpy arrays of one dtype: float64, float32, or uint16
    holding bf16 bit patterns.  With 2-D (or 3-D batched) arrays the shapes and
    packed leading dimensions are taken from them.  With 1-D buffers the caller
    gives ``M, N, K, lda, ldb, ldc, batch`` and gets back a flat buffer of
    ``batch*M*ldc`` doubles whose padding (columns ``>= N``) is NaN so that a
    read of it cannot go unnoticed.

    ``bias`` (length N or None) and ``alpha`` are widened exactly to fp64.
    """
    lib = _load()
    A = np.ascontiguousarray(A)
    B = np.ascontiguousarray(B)
    if A.dtype != B.dtype or A.dtype not in _KIND:
        raise TypeError("A and B must share a dtype among float64, float32, uint16(bf16 bits)")
    flat = A.ndim == 1
    if not flat:
        if A.ndim == 2:
            A3, B3 = A[None], B[None]
        else:
            A3, B3 = A, B
        batch, M, K = A3.shape
        b2, K2, N = B3.shape
        if b2 != batch or K2 != K:
            raise ValueError("shape mismatch")
        lda, ldb, ldc = K, N, N
    else:
        if None in (M, N, K, lda, ldb, ldc):
            raise ValueError("flat buffers need M, N, K, lda, ldb, ldc")
        if A.size < batch * M * lda - (lda - K) or B.size < batch * K * ldb - (ldb - N):
            raise ValueError("buffer too small")
    if bias is not None:
        bias64 = np.ascontiguousarray(np.asarray(bias), dtype=np.float64)
        if bias64.shape != (N,):
            raise ValueError("bias must have length N")
        bias_p = bias64.ctypes.data_as(ctypes.c_void_p)
    else:
        bias_p = None
    C = np.full(batch * M * ldc, np.nan, dtype=np.float64)
    rc = lib.oracle_gemm_epilogue(
        int(M), int(N), int(K), A.ctypes.data_as(ctypes.c_void_p), int(lda),
        B.ctypes.data_as(ctypes.c_void_p), int(ldb), _KIND[A.dtype], bias_p,
        float(alpha), ACT[act], C.ctypes.data_as(ctypes.c_void_p), int(ldc), int(batch))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    if flat:
        return C
    C = C.reshape(batch, M, N)
    return C[0] if np.ndim(A) == 2 else C


# ---------------------------------------------------------------------------------------------
# the widened operator: stored-transposed operands, row scale, residual, clamp, rounded output
# ---------------------------------------------------------------------------------------------
def _bind_fused(lib):
    c = ctypes
    lib.oracle_gemm_fused.restype = c.c_int
    lib.oracle_gemm_fused.argtypes = [
        c.c_int, c.c_int, c.c_int, c.c_int,
        c.c_void_p, c.c_long, c.c_int, c.c_void_p, c.c_long, c.c_int, c.c_int,
        c.c_double, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_long, c.c_int, c.c_double,
        c.c_int, c.c_double, c.c_double, c.c_int,
        c.c_void_p, c.c_long]
    lib.oracle_round_f32_to_bf16.restype = c.c_float
    lib.oracle_round_f32_to_bf16.argtypes = [c.c_float]
    return lib


def use_fused_library(path: str | None) -> None:
    """As ``use_library`` for the widened operator's oracle."""
    global _fused
    _fused = None if path is None else _bind_fused(ctypes.CDLL(path))


def _load_fused():
    global _fused
    if _fused is None:
        build()
        _fused = _bind_fused(ctypes.CDLL(_FUSED_LIB))
    return _fused


def round_f32_to_bf16(x: float) -> float:
    """The oracle's fp32 -> bf16 rounding (nearest, ties to even), as a float."""
    return float(_load_fused().oracle_round_f32_to_bf16(float(x)))


def gemm_fused(M, N, K, A, B, *, batch=1, transA=False, transB=False, lda=None, ldb=None,
               alpha=1.0, row_scale=None, bias=None, residual=None, ldr=None, beta=1.0,
               act="none", clamp=None, out="f64"):
    """Reference for ``round_out(clamp(act(alpha*row_scale[m]*(opA(A) @ opB(B)) + bias[n] + beta*R)))``.

    ``M, N, K`` are the logical sizes.  ``A`` holds ``batch`` matrices stored M x lda
    (``transA=False``) or K x lda (``transA=True``), ``B`` K x ldb or N x ldb, ``residual`` M x ldr;
    any array shape is accepted, the C-order content is the storage.  Leading dimensions default
    to packed.  A and B share a dtype among float64, float32, uint16 (bf16 bits); the residual may
    be any of the three.  ``clamp`` is ``(lo, hi)`` or None.  Returns fp64 values of shape
    [batch, M, N] (already rounded to fp32 / bf16 when ``out`` says so).
    """
    lib = _load_fused()
    A = np.ascontiguousarray(A).ravel()
    B = np.ascontiguousarray(B).ravel()
    if A.dtype != B.dtype or A.dtype not in _KIND:
        raise TypeError("A and B must share a dtype among float64, float32, uint16(bf16 bits)")
    lda = (M if transA else K) if lda is None else lda
    ldb = (K if transB else N) if ldb is None else ldb
    if A.size < batch * (K if transA else M) * lda or B.size < batch * (N if transB else K) * ldb:
        raise ValueError("operand buffer too small")

    def vec(x, n, name):
        if x is None:
            return None, None
        v = np.ascontiguousarray(np.asarray(x), dtype=np.float64)
        if v.shape != (n,):
            raise ValueError(f"{name} must have length {n}")
        return v, v.ctypes.data_as(ctypes.c_void_p)

    rs_keep, rs_p = vec(row_scale, M, "row_scale")
    bias_keep, bias_p = vec(bias, N, "bias")
    if residual is not None:
        R = np.ascontiguousarray(residual).ravel()
        if R.dtype not in _KIND:
            raise TypeError("residual dtype")
        ldr = N if ldr is None else ldr
        if R.size < batch * M * ldr:
            raise ValueError("residual buffer too small")
        r_p, r_kind = R.ctypes.data_as(ctypes.c_void_p), _KIND[R.dtype]
    else:
        r_p, r_kind, ldr = None, 0, 0
    lo, hi = (-np.inf, np.inf) if clamp is None else clamp
    C = np.full(batch * M * N, np.nan, dtype=np.float64)
    rc = lib.oracle_gemm_fused(
        int(M), int(N), int(K), int(batch),
        A.ctypes.data_as(ctypes.c_void_p), int(lda), int(bool(transA)),
        B.ctypes.data_as(ctypes.c_void_p), int(ldb), int(bool(transB)), _KIND[A.dtype],
        float(alpha), rs_p, bias_p, r_p, int(ldr), r_kind, float(beta),
        ACT[act], float(lo), float(hi), OUT[out],
        C.ctypes.data_as(ctypes.c_void_p), int(N))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return C.reshape(batch, M, N)


# ---------------------------------------------------------------------------------------------
# symmetric operand given by one stored triangle
# ---------------------------------------------------------------------------------------------
UPLO = {"lower": 0, "upper": 1}


def _bind_symm(lib):
    c = ctypes
    lib.oracle_gemm_symm.restype = c.c_int
    lib.oracle_gemm_symm.argtypes = [
        c.c_int, c.c_int, c.c_int,
        c.c_void_p, c.c_long, c.c_int, c.c_void_p, c.c_long, c.c_int, c.c_int,
        c.c_double, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_long, c.c_int, c.c_double,
        c.c_int, c.c_double, c.c_double, c.c_int,
        c.c_void_p, c.c_long]
    return lib


def use_symm_library(path: str | None) -> None:
    """As ``use_library`` for the symmetric-operand oracle."""
    global _symm
    _symm = None if path is None else _bind_symm(ctypes.CDLL(path))


def _load_symm():
    global _symm
    if _symm is None:
        build()
        _symm = _bind_symm(ctypes.CDLL(_SYMM_LIB))
    return _symm


def gemm_symm(M, N, A, B, *, uplo="lower", batch=1, transB=False, lda=None, ldb=None, alpha=1.0,
              row_scale=None, bias=None, residual=None, ldr=None, beta=1.0, act="none", clamp=None, out="f64"):
    """Reference for the widened operator's chain on ``S @ opB(B)``, S the symmetric M x M matrix whose
    ``uplo`` triangle is stored in ``A`` (M x lda per batch); the other triangle of ``A`` is never read.
    ``B`` is M x ldb (K = M) or, with ``transB``, N x ldb.  Dtypes and the remaining arguments as for
    ``gemm_fused``.  Returns fp64 values of shape [batch, M, N]."""
    lib = _load_symm()
    A = np.ascontiguousarray(A).ravel()
    B = np.ascontiguousarray(B).ravel()
    if A.dtype != B.dtype or A.dtype not in _KIND:
        raise TypeError("A and B must share a dtype among float64, float32, uint16(bf16 bits)")
    lda = M if lda is None else lda
    ldb = (M if transB else N) if ldb is None else ldb
    if A.size < batch * M * lda or B.size < batch * (N if transB else M) * ldb:
        raise ValueError("operand buffer too small")

    def vec(x, n, name):
        if x is None:
            return None, None
        v = np.ascontiguousarray(np.asarray(x), dtype=np.float64)
        if v.shape != (n,):
            raise ValueError(f"{name} must have length {n}")
        return v, v.ctypes.data_as(ctypes.c_void_p)

    rs_keep, rs_p = vec(row_scale, M, "row_scale")
    bias_keep, bias_p = vec(bias, N, "bias")
    if residual is not None:
        R = np.ascontiguousarray(residual).ravel()
        if R.dtype not in _KIND:
            raise TypeError("residual dtype")
        ldr = N if ldr is None else ldr
        if R.size < batch * M * ldr:
            raise ValueError("residual buffer too small")
        r_p, r_kind = R.ctypes.data_as(ctypes.c_void_p), _KIND[R.dtype]
    else:
        r_p, r_kind, ldr = None, 0, 0
    lo, hi = (-np.inf, np.inf) if clamp is None else clamp
    C = np.full(batch * M * N, np.nan, dtype=np.float64)
    rc = lib.oracle_gemm_symm(
        int(M), int(N), int(batch), A.ctypes.data_as(ctypes.c_void_p), int(lda), UPLO[uplo],
        B.ctypes.data_as(ctypes.c_void_p), int(ldb), int(bool(transB)), _KIND[A.dtype],
        float(alpha), rs_p, bias_p, r_p, int(ldr), r_kind, float(beta),
        ACT[act], float(lo), float(hi), OUT[out], C.ctypes.data_as(ctypes.c_void_p), int(N))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return C.reshape(batch, M, N)


# ---------------------------------------------------------------------------------------------
# convolution front-end (channels-last), same consumer chain
# ---------------------------------------------------------------------------------------------
def _bind_conv(lib):
    c = ctypes
    lib.oracle_conv2d_nhwc.restype = c.c_int
    lib.oracle_conv2d_nhwc.argtypes = [c.c_int] * 13 + [
        c.c_void_p, c.c_void_p, c.c_int, c.c_double, c.c_void_p,
        c.c_void_p, c.c_int, c.c_double, c.c_int, c.c_double, c.c_double, c.c_int, c.c_void_p]
    lib.oracle_conv_out_size.restype = c.c_int
    lib.oracle_conv_out_size.argtypes = [c.c_int] * 5
    return lib


def use_conv_library(path: str | None) -> None:
    """As ``use_library`` for the convolution oracle."""
    global _conv
    _conv = None if path is None else _bind_conv(ctypes.CDLL(path))


def _load_conv():
    global _conv
    if _conv is None:
        build()
        _conv = _bind_conv(ctypes.CDLL(_CONV_LIB))
    return _conv


def conv_out_size(size: int, k: int, stride: int = 1, pad: int = 0, dil: int = 1) -> int:
    return int(_load_conv().oracle_conv_out_size(size, k, stride, pad, dil))


def conv2d_nhwc(X, Wt, *, stride=(1, 1), pad=(0, 0), dil=(1, 1), alpha=1.0, bias=None, residual=None,
                beta=1.0, act="none", clamp=None, out="f64"):
    """Reference convolution, channels-last: ``X`` [N,H,W,Cin], ``Wt`` [Cout,KH,KW,Cin] of one dtype
    among float64, float32, uint16 (bf16 bits); ``residual`` [N,OH,OW,Cout] of any of them.
    Returns fp64 [N,OH,OW,Cout] (rounded to fp32 / bf16 when ``out`` says so)."""
    lib = _load_conv()
    X = np.ascontiguousarray(X)
    Wt = np.ascontiguousarray(Wt)
    if X.dtype != Wt.dtype or X.dtype not in _KIND or X.ndim != 4 or Wt.ndim != 4:
        raise TypeError("X and Wt must be 4-D arrays of one dtype among float64, float32, uint16(bf16 bits)")
    Nb, H, W, Cin = X.shape
    Cout, KH, KW, Cin2 = Wt.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    OH = conv_out_size(H, KH, stride[0], pad[0], dil[0])
    OW = conv_out_size(W, KW, stride[1], pad[1], dil[1])
    if OH < 1 or OW < 1:
        raise ValueError("empty output")
    bias_p = None
    if bias is not None:
        bias64 = np.ascontiguousarray(np.asarray(bias), dtype=np.float64)
        if bias64.shape != (Cout,):
            raise ValueError("bias must have length Cout")
        bias_p = bias64.ctypes.data_as(ctypes.c_void_p)
    r_p, r_kind = None, 0
    if residual is not None:
        R = np.ascontiguousarray(residual)
        if R.shape != (Nb, OH, OW, Cout) or R.dtype not in _KIND:
            raise ValueError("residual must be [N,OH,OW,Cout]")
        r_p, r_kind = R.ctypes.data_as(ctypes.c_void_p), _KIND[R.dtype]
    lo, hi = (-np.inf, np.inf) if clamp is None else clamp
    Y = np.full((Nb, OH, OW, Cout), np.nan, dtype=np.float64)
    rc = lib.oracle_conv2d_nhwc(Nb, H, W, Cin, Cout, KH, KW, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1],
                                X.ctypes.data_as(ctypes.c_void_p), Wt.ctypes.data_as(ctypes.c_void_p), _KIND[X.dtype],
                                float(alpha), bias_p, r_p, r_kind, float(beta), ACT[act], float(lo), float(hi),
                                OUT[out], Y.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return Y


def gemm_rowsum(A, B, bias=None, alpha=1.0):
    """Reference for the row sum of a linear layer, ``y[m] = sum_n (alpha * (A @ B)[m, n] + bias[n])``,
    as an fp64 vector of length M (Level-2 optimisation prompt, "First priority: algebraic
    simplification": the sum over the output dimension of a linear layer).

    The definition written out: the full product by the pinned GEMM oracle (fp64 sums over k, no
    activation), then the sum over n of every row in fp64.  The GPU path never forms the product: it
    uses the collapsed form ``alpha * A @ (B @ 1) + sum(bias)``, which a pin ties to this definition.
    A: (M, K), B: (K, N) as the operator reads it (a weight matrix stored N x K is passed transposed).
    """
    C = gemm_epilogue(A, B, bias, alpha, "none")
    if C.ndim == 3:
        C = C[0]
    return np.sum(C, axis=1, dtype=np.float64)
