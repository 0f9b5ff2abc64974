"""Seeded synthetic inputs for the GEMM + epilogue workloads.

This module is the only code the GPU library's tests and the CPU oracle's tests
have in common.  It draws numbers and rounds them; it contains none of the
operator's arithmetic.

Generator (counter based, so any element can be regenerated on its own):
    key(seed, stream) = mix64(seed * 0xD1342543DE82EF95 + stream * 0x9E3779B97F4A7C15 + 1)
    word(i)           = mix64(key + (i + 1) * 0x9E3779B97F4A7C15)        (mod 2^64)
    mix64             = the splitmix64 output function (Steele, Lea, Flood 2014)
    u(i)              = (word(i) >> 11) * 2^-53                          in [0, 1)
    uniform(a, b)     = a + (b - a) * u(i), rounded once to fp32
    normal            = sqrt(-2 ln(1 - u(2i))) * cos(2 pi u(2i+1)), fp64, rounded once to fp32
Streams: 0 = A, 1 = B, 2 = bias.  Elements are numbered in row-major order of
the logical (batch, rows, cols) tensor, so a leading dimension larger than the
row length does not change the values.

The workloads below are the five synthetic stand-ins for the matmul and fused
matmul shapes the paper evaluates on (its benchmark suite is not reproduced).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_SEEDMUL = np.uint64(0xD1342543DE82EF95)
STREAM_A, STREAM_B, STREAM_BIAS = 0, 1, 2


def _mix64(z: np.ndarray) -> np.ndarray:
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= np.uint64(0xBF58476D1CE4E5B9)
    z ^= z >> np.uint64(27)
    z *= np.uint64(0x94D049BB133111EB)
    z ^= z >> np.uint64(31)
    return z


def _key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = np.array([np.uint64(seed) * _SEEDMUL + np.uint64(stream) * _GOLD + np.uint64(1)],
                     dtype=np.uint64)
        return _mix64(k)[0]


def _unit(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """u(i) for i in [start, start+count) as fp64 in [0, 1)."""
    with np.errstate(over="ignore"):
        i = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        w = _mix64(_key(seed, stream) + i * _GOLD)
    return (w >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


_CHUNK = 1 << 20
_THREADS = max(1, min(16, len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else 4))


def _chunked(n: int, fill) -> np.ndarray:
    """out[s:s+c] = fill(s, c) over chunks; chunks are independent (counter based),
    so they are spread over a few threads."""
    out = np.empty(n, dtype=np.float32)

    def work(s):
        c = min(_CHUNK, n - s)
        out[s:s + c] = fill(s, c)

    starts = range(0, n, _CHUNK)
    if n <= _CHUNK or _THREADS == 1:
        for s in starts:
            work(s)
    else:
        with ThreadPoolExecutor(_THREADS) as pool:
            list(pool.map(work, starts))
    return out


def uniform(seed: int, stream: int, n: int, lo: float, hi: float, start: int = 0) -> np.ndarray:
    """n fp32 samples of U(lo, hi): elements start .. start+n-1 of the stream."""
    return _chunked(n, lambda s, c: (lo + (hi - lo) * _unit(seed, stream, start + s, c)).astype(np.float32))


def normal(seed: int, stream: int, n: int, scale: float = 1.0, start: int = 0) -> np.ndarray:
    """n fp32 samples of scale * N(0, 1) (Box-Muller, cosine branch)."""
    def fill(s, c):
        u = _unit(seed, stream, 2 * (start + s), 2 * c)
        r = np.sqrt(-2.0 * np.log1p(-u[0::2]))
        return (scale * r * np.cos(2.0 * np.pi * u[1::2])).astype(np.float32)
    return _chunked(n, fill)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the 16-bit patterns.

    Inputs are finite by construction; NaN handling is not needed.
    """
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration: shapes, distributions and epilogue."""
    name: str
    dtype: str            # "bf16" or "f32": element type of A and B
    M: int
    N: int
    K: int
    batch: int
    seed: int
    dist: str             # "uniform" (U(-1,1)) or "normal"
    scale: float          # multiplies normal samples (ignored for uniform)
    alpha: float
    bias: tuple | None    # (lo, hi) of the uniform bias, "zero", or None
    act: str

    @property
    def flops(self) -> float:
        return 2.0 * self.M * self.N * self.K * self.batch

    @property
    def algorithmic_bytes(self) -> float:
        """Read A, B and bias once, write C once."""
        e = 2 if self.dtype == "bf16" else 4
        nb = 0 if self.bias is None else 4 * self.N
        return float(self.batch * (self.M * self.K + self.K * self.N) * e
                     + self.batch * self.M * self.N * 4 + nb)


WORKLOADS = {
    "c1_f32_256": Workload("c1_f32_256", "f32", 256, 256, 256, 1, 0, "uniform", 1.0, 1.0, None, "none"),
    "c2_bf16_4096": Workload("c2_bf16_4096", "bf16", 4096, 4096, 4096, 1, 1, "normal",
                             4096 ** -0.5, 1.0, None, "none"),
    "c3_bf16_8192_bias_gelu": Workload("c3_bf16_8192_bias_gelu", "bf16", 8192, 8192, 8192, 1, 2,
                                       "normal", 8192 ** -0.5, 0.5, (-0.1, 0.1), "gelu_tanh"),
    "c4_bf16_batched_512x512x64": Workload("c4_bf16_batched_512x512x64", "bf16", 512, 512, 64, 256, 3,
                                           "normal", 1.0, 1.0, (-1.0, 1.0), "relu"),
    "c5_bf16_splitk_1024x1024x65536": Workload("c5_bf16_splitk_1024x1024x65536", "bf16", 1024, 1024,
                                               65536, 1, 4, "uniform", 1.0, 1.0 / 256.0, "zero", "none"),
    # a large fp32 product: c1's recipe (U(-1,1), no bias, no activation) at a size that fills the chip,
    # for the fp32 matrix-instruction roofline (c1 itself is bound by launch latency)
    "c13_f32_8192x8192x2048": Workload("c13_f32_8192x8192x2048", "f32", 8192, 8192, 2048, 1, 13, "uniform", 1.0, 1.0,
                                       None, "none"),
}


def _draw(w: Workload, stream: int, n: int, start: int = 0) -> np.ndarray:
    if w.dist == "uniform":
        return uniform(w.seed, stream, n, -1.0, 1.0, start)
    return normal(w.seed, stream, n, w.scale, start)


def make_bias(w: Workload):
    if w.bias is None:
        return None
    if w.bias == "zero":
        return np.zeros(w.N, dtype=np.float32)
    return uniform(w.seed, STREAM_BIAS, w.N, w.bias[0], w.bias[1])


def make_operand(w: Workload, which: str, row_start: int = 0, rows: int | None = None,
                 batch_index: int | None = None) -> np.ndarray:
    """Rows [row_start, row_start+rows) of A ("A": M x K) or B ("B": K x N).

    With ``batch_index`` None all batches are produced (shape (batch, rows, cols));
    otherwise only that batch (shape (rows, cols)).  bf16 workloads return uint16
    bit patterns (the fp32 sample rounded to nearest even), fp32 workloads float32.
    """
    nrows, ncols = (w.M, w.K) if which == "A" else (w.K, w.N)
    stream = STREAM_A if which == "A" else STREAM_B
    rows = nrows - row_start if rows is None else rows
    batches = range(w.batch) if batch_index is None else [batch_index]
    parts = []
    for b in batches:
        start = (b * nrows + row_start) * ncols
        x = _draw(w, stream, rows * ncols, start).reshape(rows, ncols)
        parts.append(to_bf16_bits(x) if w.dtype == "bf16" else x)
    return parts[0] if batch_index is not None else np.stack(parts)


def make_inputs(w: Workload):
    """(A, B, bias) for the whole workload; A, B carry a leading batch axis."""
    return make_operand(w, "A"), make_operand(w, "B"), make_bias(w)


# ---------------------------------------------------------------------------------------------
# workloads of the widened operator (operands stored either way round, row scale, residual,
# clamp, bf16 output): the same generator, plus the storage layout of each operand
# ---------------------------------------------------------------------------------------------
STREAM_ROW_SCALE = 7
STREAM_RESIDUAL = 8


@dataclass(frozen=True)
class FusedWorkload:
    name: str
    base: Workload        # shapes, seed, distributions, alpha, bias, activation
    transA: bool          # A stored K x M
    transB: bool          # B stored N x K
    row_scale: bool       # fp32[M] ~ U(0.5, 1.5)
    residual: str | None  # None, "f32" or "bf16": [batch, M, N] ~ U(-1, 1)
    beta: float
    clamp: tuple | None
    out: str              # "f32" or "bf16"
    a_structure: str = "general"   # "lower" / "upper": the other triangle of A (as the operator reads it) is zero

    @property
    def flops(self) -> float:
        """Multiply-adds with a nonzero A, times two: all of them, or those of the kept triangle."""
        w = self.base
        if self.a_structure == "general":
            return w.flops
        if self.a_structure == "lower":
            kept = sum(min(m + 1, w.K) for m in range(w.M))
        else:
            kept = sum(max(w.K - m, 0) for m in range(w.M))
        return 2.0 * w.batch * w.N * kept

    @property
    def algorithmic_bytes(self) -> float:
        """Read A, B, bias, row scale and the residual once, write C once."""
        w = self.base
        mn = w.batch * w.M * w.N
        r = 0 if self.residual is None else mn * (4 if self.residual == "f32" else 2)
        return float(w.batch * (w.M * w.K + w.K * w.N) * 2 + mn * (4 if self.out == "f32" else 2) + r
                     + (0 if w.bias is None else 4 * w.N) + (4 * w.M if self.row_scale else 0))


def _fw(name, M, N, K, batch, seed, dist, scale, alpha, bias, act, **kw):
    return FusedWorkload(name, Workload(name, "bf16", M, N, K, batch, seed, dist, scale, alpha, bias, act), **kw)


FUSED_WORKLOADS = {
    # a linear layer as frameworks store it (weights N x K), bf16 activations out
    "c6_fused_nt_8192_bias_gelu_bf16out": _fw(
        "c6_fused_nt_8192_bias_gelu_bf16out", 8192, 8192, 8192, 1, 6, "normal", 8192 ** -0.5, 0.5, (-0.1, 0.1),
        "gelu_tanh", transA=False, transB=True, row_scale=False, residual=None, beta=0.0, clamp=None, out="bf16"),
    # both operands stored against the grain of the matrix unit, full consumer chain
    "c7_fused_tn_8192_chain": _fw(
        "c7_fused_tn_8192_chain", 8192, 8192, 8192, 1, 7, "normal", 8192 ** -0.5, 1.0, (-0.1, 0.1),
        "relu", transA=True, transB=False, row_scale=True, residual="bf16", beta=0.5, clamp=(0.0, 6.0), out="bf16"),
    # the batched small-K shape with bf16 residual in and bf16 out: half the store stream
    "c8_fused_batched_512x512x64_bf16out": _fw(
        "c8_fused_batched_512x512x64_bf16out", 512, 512, 64, 256, 8, "normal", 1.0, 1.0, (-1.0, 1.0),
        "relu", transA=False, transB=False, row_scale=False, residual=None, beta=0.0, clamp=None, out="bf16"),
    # a lower-triangular A (the caller says so): the multiply skips the zero K ranges of every tile row
    "c11_fused_lower_8192_bias_relu": _fw(
        "c11_fused_lower_8192_bias_relu", 8192, 8192, 8192, 1, 11, "normal", 8192 ** -0.5, 0.5, (-0.1, 0.1),
        "relu", transA=False, transB=False, row_scale=False, residual=None, beta=0.0, clamp=None, out="f32",
        a_structure="lower"),
}


def make_fused_inputs(fw: FusedWorkload):
    """Storage arrays of a fused workload: dict with A (batch, rowsA, colsA), B, bias, row_scale,
    residual (or None each).  bf16 arrays are uint16 bit patterns."""
    w = fw.base
    A = make_operand(w, "A")
    B = make_operand(w, "B")
    if fw.a_structure == "lower":
        A = np.tril(A)                      # the last two axes: A[b, m, k] = 0 for k > m
    elif fw.a_structure == "upper":
        A = np.triu(A)
    if fw.transA:
        A = np.ascontiguousarray(A.transpose(0, 2, 1))
    if fw.transB:
        B = np.ascontiguousarray(B.transpose(0, 2, 1))
    rs = uniform(w.seed, STREAM_ROW_SCALE, w.M, 0.5, 1.5) if fw.row_scale else None
    R = None
    if fw.residual is not None:
        R = uniform(w.seed, STREAM_RESIDUAL, w.batch * w.M * w.N, -1.0, 1.0).reshape(w.batch, w.M, w.N)
        if fw.residual == "bf16":
            R = to_bf16_bits(R)
    return {"A": A, "B": B, "bias": make_bias(w), "row_scale": rs, "residual": R}


# ---------------------------------------------------------------------------------------------
# structured operand: A = diag(d).  K = M for the GEMM this replaces; the entry point itself
# touches only d, B, bias and C.
# ---------------------------------------------------------------------------------------------
DIAG_WORKLOADS = {
    "c9_diag_bf16_8192": Workload("c9_diag_bf16_8192", "bf16", 8192, 8192, 8192, 1, 9, "normal", 1.0, 0.5,
                                  (-0.1, 0.1), "relu"),
}


# ---------------------------------------------------------------------------------------------
# symmetric operand given by its lower triangle, few output columns (K = M): a stream of A
# ---------------------------------------------------------------------------------------------
SYMM_WORKLOADS = {
    "c14_symm_lower_16384_n16": Workload("c14_symm_lower_16384_n16", "bf16", 16384, 16, 16384, 1, 14, "normal",
                                         16384 ** -0.5, 0.5, (-0.1, 0.1), "relu"),
}


def make_symm_inputs(w: Workload):
    """(A bf16 bits [M, M] drawn in full -- only its lower triangle is meant to be read --, B bf16 bits
    [M, N] ~ N(0, 1), bias).  A ~ N(0, 1) * M^-1/2."""
    A = make_operand(w, "A")[0]
    B = to_bf16_bits(normal(w.seed, STREAM_B, w.K * w.N, 1.0).reshape(w.K, w.N))
    return A, B, make_bias(w)


def symm_algorithmic_bytes(w: Workload) -> float:
    """Read the stored triangle of A, B and the bias once, write C (fp32) once."""
    return float(w.M * (w.M + 1) // 2 * 2 + w.K * w.N * 2 + 4 * w.N + w.M * w.N * 4)


# ---------------------------------------------------------------------------------------------
# row sum of a linear layer: y = sum_n (alpha x W^T + b); W stored N x K as frameworks keep it
# ---------------------------------------------------------------------------------------------
ROWSUM_WORKLOADS = {
    "c12_rowsum_linear_8192": Workload("c12_rowsum_linear_8192", "bf16", 8192, 8192, 8192, 1, 12, "normal",
                                       8192 ** -0.5, 0.5, (-0.1, 0.1), "none"),
}


def make_rowsum_inputs(w: Workload):
    """(A bf16 bits [M, K], W bf16 bits [N, K] -- the operator's B is its transpose --, bias fp32[N])."""
    A = make_operand(w, "A")[0]
    Wt = np.ascontiguousarray(make_operand(w, "B")[0].T)
    return A, Wt, make_bias(w)


def rowsum_algorithmic_bytes(w: Workload) -> float:
    """Read A, the weights and the bias once, write y once."""
    return float((w.M * w.K + w.K * w.N) * 2 + 4 * w.N + 4 * w.M)


def make_diag_inputs(w: Workload):
    """(d fp32[M] ~ U(0.5, 1.5), B bf16 bits [batch, M, N], bias)."""
    d = uniform(w.seed, STREAM_ROW_SCALE, w.M, 0.5, 1.5)
    parts = [to_bf16_bits(_draw(w, STREAM_B, w.M * w.N, b * w.M * w.N).reshape(w.M, w.N)) for b in range(w.batch)]
    return d, np.stack(parts), make_bias(w)


def diag_algorithmic_bytes(w: Workload) -> float:
    """Read B, d and bias once, write C once."""
    return float(w.batch * w.M * w.N * (2 + 4) + 4 * w.M + (0 if w.bias is None else 4 * w.N))


# ---------------------------------------------------------------------------------------------
# convolution front-end (channels-last): a 3x3 layer of a residual network's middle stage
# ---------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class ConvWorkload:
    name: str
    N: int
    H: int
    W: int
    Cin: int
    Cout: int
    KH: int
    KW: int
    stride: tuple
    pad: tuple
    dil: tuple
    seed: int
    alpha: float
    bias: tuple | None
    residual: str | None
    beta: float
    act: str
    clamp: tuple | None
    out: str

    def out_hw(self):
        oh = (self.H + 2 * self.pad[0] - self.dil[0] * (self.KH - 1) - 1) // self.stride[0] + 1
        ow = (self.W + 2 * self.pad[1] - self.dil[1] * (self.KW - 1) - 1) // self.stride[1] + 1
        return oh, ow

    @property
    def flops(self) -> float:
        oh, ow = self.out_hw()
        return 2.0 * self.N * oh * ow * self.Cout * self.KH * self.KW * self.Cin

    @property
    def algorithmic_bytes(self) -> float:
        oh, ow = self.out_hw()
        y = self.N * oh * ow * self.Cout
        r = 0 if self.residual is None else y * (4 if self.residual == "f32" else 2)
        return float(self.N * self.H * self.W * self.Cin * 2 + self.Cout * self.KH * self.KW * self.Cin * 2
                     + y * (4 if self.out == "f32" else 2) + r + (0 if self.bias is None else 4 * self.Cout))


CONV_WORKLOADS = {
    "c10_conv3x3_256_bf16out": ConvWorkload("c10_conv3x3_256_bf16out", 32, 56, 56, 256, 256, 3, 3, (1, 1), (1, 1), (1, 1),
                                            10, 1.0, (-0.1, 0.1), "bf16", 1.0, "relu", None, "bf16"),
    # the first layer of a residual network: 3 input channels, 7 x 7, stride 2, padding 3, 64 filters; bound by the
    # bytes of its input and output (7.6 GFLOP over 61 MB), not by the matrix pipes
    "c15_conv7x7_first_layer_bf16out": ConvWorkload("c15_conv7x7_first_layer_bf16out", 32, 224, 224, 3, 64, 7, 7, (2, 2), (3, 3),
                                                    (1, 1), 15, 1.0, (-0.1, 0.1), None, 1.0, "relu", None, "bf16"),
}
# which roofline bounds a convolution workload: the matrix pipes, or (few channels) the bytes moved
CONV_BOUND = {"c10_conv3x3_256_bf16out": "mfma", "c15_conv7x7_first_layer_bf16out": "hbm"}


def make_conv_inputs(cw: ConvWorkload, images=None):
    """X [n,H,W,Cin] ~ N(0,1), Wt [Cout,KH,KW,Cin] ~ N(0,1)/sqrt(KH*KW*Cin) (bf16 bits), bias, residual
    [n,OH,OW,Cout] ~ U(-1,1); ``images`` selects image indices (default all), each image's values
    being the same whichever subset is produced."""
    images = range(cw.N) if images is None else images
    oh, ow = cw.out_hw()
    per_x, per_y = cw.H * cw.W * cw.Cin, oh * ow * cw.Cout
    X = np.stack([to_bf16_bits(normal(cw.seed, STREAM_A, per_x, 1.0, i * per_x).reshape(cw.H, cw.W, cw.Cin))
                  for i in images])
    kk = cw.KH * cw.KW * cw.Cin
    Wt = to_bf16_bits(normal(cw.seed, STREAM_B, cw.Cout * kk, kk ** -0.5).reshape(cw.Cout, cw.KH, cw.KW, cw.Cin))
    bias = None if cw.bias is None else uniform(cw.seed, STREAM_BIAS, cw.Cout, cw.bias[0], cw.bias[1])
    R = None
    if cw.residual is not None:
        R = np.stack([uniform(cw.seed, STREAM_RESIDUAL, per_y, -1.0, 1.0, i * per_y).reshape(oh, ow, cw.Cout)
                      for i in images])
        if cw.residual == "bf16":
            R = to_bf16_bits(R)
    return {"X": X, "Wt": Wt, "bias": bias, "residual": R}
