"""Pins for the CPU oracle: every check compares it with something other than itself.

The paper prints no worked numeric GEMM example, so the pins are exact rational
brute force, closed forms and identities of C = act(alpha*A@B + bias) (naive
matmul definition: appendix "Comparison of CuTe and CUDA Representations for
Square GEMM", Fig. simp_cuda; fused writeback: Level-2 optimisation prompt,
"Fusion").  Shapes are non-square and data asymmetric so that a transposed or
mis-strided operand cannot pass.
"""
from fractions import Fraction
import math

import numpy as np
import pytest

from paper_2604_01489_amd import inputs as gen


def _rng(seed):
    return np.random.default_rng(seed)


def _ulp_close(x, ref, ulps=2):
    ref = np.asarray(ref, dtype=np.float64)
    return np.all(np.abs(np.asarray(x) - ref) <= ulps * np.spacing(np.maximum(np.abs(ref), 1e-300)))


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (4, 2, 9), (7, 3, 2)])
def test_brute_force_exact_rationals(oracle, M, N, K):
    """Exact rational arithmetic, columns outermost: an independent formulation."""
    r = _rng(10 + M)
    A = r.uniform(-1, 1, (M, K)).astype(np.float32)
    B = r.uniform(-1, 1, (K, N)).astype(np.float32)
    bias = r.uniform(-1, 1, N).astype(np.float32)
    alpha = np.float32(0.75)
    got = oracle.gemm_epilogue(A, B, bias, float(alpha), "none")
    for n in range(N):
        for m in range(M):
            s = Fraction(0)
            for k in range(K):
                s += Fraction(float(A[m, k])) * Fraction(float(B[k, n]))
            exact = Fraction(float(alpha)) * s + Fraction(float(bias[n]))
            ref = float(exact)
            assert abs(got[m, n] - ref) <= 4 * np.spacing(max(abs(ref), 1e-3)), (m, n)


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
def test_small_integers_are_exact(oracle, dtype):
    """Integer-valued operands: every product and partial sum is exact."""
    r = _rng(3)
    M, N, K = 9, 13, 21
    Ai = r.integers(-8, 9, (M, K))
    Bi = r.integers(-8, 9, (K, N))
    want = (Ai @ Bi).astype(np.float64)
    if dtype == "f64":
        A, B = Ai.astype(np.float64), Bi.astype(np.float64)
    elif dtype == "f32":
        A, B = Ai.astype(np.float32), Bi.astype(np.float32)
    else:
        A, B = gen.to_bf16_bits(Ai.astype(np.float32)), gen.to_bf16_bits(Bi.astype(np.float32))
    got = oracle.gemm_epilogue(A, B)
    assert np.array_equal(got, want)


def test_bf16_widening_matches_bit_definition(oracle):
    """bf16 operands enter as the fp32 value with the same upper 16 bits."""
    r = _rng(5)
    A32 = r.normal(size=(6, 10)).astype(np.float32)
    B32 = r.normal(size=(10, 4)).astype(np.float32)
    Ab, Bb = gen.to_bf16_bits(A32), gen.to_bf16_bits(B32)
    got = oracle.gemm_epilogue(Ab, Bb)
    want = oracle.gemm_epilogue(gen.bf16_bits_to_f32(Ab).astype(np.float64),
                                gen.bf16_bits_to_f32(Bb).astype(np.float64))
    assert np.array_equal(got, want)
    # and differs from the unrounded fp32 product (rounding really happened)
    assert not np.array_equal(got, oracle.gemm_epilogue(A32, B32))


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("act", ["none", "relu", "gelu_tanh"])
def test_identity_B(oracle, act):
    r = _rng(7)
    M, K = 11, 6
    A = r.uniform(-2, 2, (M, K))
    bias = r.uniform(-1, 1, K)
    alpha = 0.5
    got = oracle.gemm_epilogue(A, np.eye(K), bias, alpha, act)
    v = alpha * A + bias[None, :]
    if act == "none":
        assert np.array_equal(got, v)
    elif act == "relu":
        assert np.array_equal(got, np.where(v > 0, v, 0.0))
    else:
        want = [[0.5 * x * (1 + math.tanh(math.sqrt(2 / math.pi) * (x + 0.044715 * x ** 3))) for x in row]
                for row in v]
        assert _ulp_close(got, want, 4)


def test_all_ones(oracle):
    M, N, K = 5, 8, 300
    bias = np.arange(N, dtype=np.float64) - 3.0
    alpha = 0.25
    got = oracle.gemm_epilogue(np.ones((M, K)), np.ones((K, N)), bias, alpha, "none")
    assert np.array_equal(got, np.broadcast_to(K * alpha + bias, (M, N)))
    got = oracle.gemm_epilogue(np.ones((M, K)), np.ones((K, N)), bias - 80.0, alpha, "relu")
    assert np.array_equal(got, np.broadcast_to(np.maximum(K * alpha + bias - 80.0, 0.0), (M, N)))


def test_linearity_in_alpha(oracle):
    r = _rng(9)
    A = r.normal(size=(6, 17))
    B = r.normal(size=(17, 5))
    c1 = oracle.gemm_epilogue(A, B, None, 0.375)
    assert np.array_equal(oracle.gemm_epilogue(A, B, None, 0.75), 2.0 * c1)
    assert np.array_equal(oracle.gemm_epilogue(A, B, None, -0.375), -c1)
    c2 = oracle.gemm_epilogue(A, B, None, 1.625)
    assert _ulp_close(oracle.gemm_epilogue(A, B, None, 2.0), c1 + c2, 4)
    assert np.array_equal(oracle.gemm_epilogue(A, B, None, 0.0), np.zeros((6, 5)))


def test_transposition_identity(oracle):
    """(A B)^T = B^T A^T, same k order on both sides, so equality is exact."""
    r = _rng(11)
    A = r.normal(size=(7, 12))
    B = r.normal(size=(12, 4))
    c = oracle.gemm_epilogue(A, B)
    ct = oracle.gemm_epilogue(np.ascontiguousarray(B.T), np.ascontiguousarray(A.T))
    assert np.array_equal(c.T, ct)


def test_matches_library_matmul(oracle):
    """Special case alpha=1, no bias, no activation is a textbook matmul."""
    r = _rng(13)
    A = r.normal(size=(33, 47))
    B = r.normal(size=(47, 29))
    got = oracle.gemm_epilogue(A, B)
    want = A @ B
    assert np.max(np.abs(got - want)) <= 64 * np.finfo(np.float64).eps * np.max(np.abs(A) @ np.abs(B))
    # B given as (N, K) by mistake would have a different shape/result
    assert np.max(np.abs(got - (A[:, :29] @ B[:29, :]))) > 1e-3


def test_bias_difference_and_axis(oracle):
    r = _rng(15)
    A = r.normal(size=(5, 9))
    B = r.normal(size=(9, 7))
    bias = r.uniform(-1, 1, 7)
    d = oracle.gemm_epilogue(A, B, bias, 1.5) - oracle.gemm_epilogue(A, B, None, 1.5)
    assert np.max(np.abs(d - bias[None, :])) <= 8 * np.finfo(np.float64).eps * 10
    # bias is added after the scale: doubling alpha must not double the bias
    d2 = oracle.gemm_epilogue(A, B, bias, 3.0) - oracle.gemm_epilogue(A, B, None, 3.0)
    assert np.max(np.abs(d2 - bias[None, :])) <= 8 * np.finfo(np.float64).eps * 20


# ---------------------------------------------------------------- activations
def test_relu_identities(oracle):
    r = _rng(17)
    A = r.normal(size=(8, 10))
    B = r.normal(size=(10, 6))
    bias = r.uniform(-1, 1, 6)
    v = oracle.gemm_epilogue(A, B, bias, 0.5, "none")
    y = oracle.gemm_epilogue(A, B, bias, 0.5, "relu")
    assert np.array_equal(y, (v + np.abs(v)) / 2)
    assert (v < 0).any() and (v > 0).any()
    assert np.all(y >= 0) and np.array_equal(y[v >= 0], v[v >= 0])


def test_gelu_tanh_identities(oracle):
    """g(0)=0; g(v)-g(-v)=v; g(v)->v for large v, ->0 for very negative v; an
    independent evaluation through exp; and the library's tanh-GELU in fp64."""
    import torch
    v = np.concatenate([np.linspace(-12, 12, 2001), [0.0, 1e-8, -1e-8, 30.0, -30.0]])
    K = v.size
    A = v[None, :]                      # 1 x K
    g = oracle.gemm_epilogue(np.ascontiguousarray(A.T), np.ones((1, 1)), None, 1.0, "gelu_tanh")[:, 0]
    gm = oracle.gemm_epilogue(np.ascontiguousarray(-A.T), np.ones((1, 1)), None, 1.0, "gelu_tanh")[:, 0]
    assert g[v == 0.0][0] == 0.0
    assert np.max(np.abs((g - gm) - v)) <= 4e-15 * np.maximum(1, np.abs(v)).max()
    assert g[-2] == 30.0 and abs(g[-1]) < 1e-300 and g[-1] <= 0.0
    u = math.sqrt(2 / math.pi) * (v + 0.044715 * v ** 3)
    with np.errstate(over="ignore"):
        alt = 0.5 * v * (1 + (1 - 2 / (1 + np.exp(2 * u))))
    assert np.max(np.abs(g - alt)) <= 1e-14
    lib = torch.nn.functional.gelu(torch.from_numpy(v), approximate="tanh").numpy()
    assert np.max(np.abs(g - lib)) <= 1e-14
    # it is the tanh form, not the erf form
    erf = torch.nn.functional.gelu(torch.from_numpy(v)).numpy()
    assert np.max(np.abs(g - erf)) > 1e-4
    assert K > 0


def test_epilogue_order_scale_then_bias_then_act(oracle):
    A = np.array([[2.0]])
    B = np.array([[3.0]])
    bias = np.array([-10.0])
    assert oracle.gemm_epilogue(A, B, bias, 0.5, "none")[0, 0] == -7.0       # 0.5*6 - 10
    assert oracle.gemm_epilogue(A, B, bias, 0.5, "relu")[0, 0] == 0.0
    assert oracle.gemm_epilogue(A, B, -bias, 0.5, "relu")[0, 0] == 13.0


# ---------------------------------------------------------------- layout
def test_batch_equals_per_slice(oracle):
    r = _rng(19)
    A = r.normal(size=(3, 4, 6))
    B = r.normal(size=(3, 6, 5))
    bias = r.normal(size=5)
    got = oracle.gemm_epilogue(A, B, bias, 0.5, "relu")
    for b in range(3):
        assert np.array_equal(got[b], oracle.gemm_epilogue(A[b], B[b], bias, 0.5, "relu"))
    assert not np.array_equal(got[0], got[1])


def test_padded_leading_dimensions(oracle):
    """lda > K, ldb > N, ldc > N: padding is never read (NaN-filled) nor written."""
    r = _rng(21)
    M, N, K, batch = 5, 3, 4, 2
    lda, ldb, ldc = 7, 6, 5
    A = r.normal(size=(batch, M, K))
    B = r.normal(size=(batch, K, N))
    Ap = np.full((batch, M, lda), np.nan); Ap[:, :, :K] = A
    Bp = np.full((batch, K, ldb), np.nan); Bp[:, :, :N] = B
    flat = oracle.gemm_epilogue(Ap.ravel(), Bp.ravel(), None, 1.0, "none",
                                M=M, N=N, K=K, lda=lda, ldb=ldb, ldc=ldc, batch=batch)
    Cp = flat.reshape(batch, M, ldc)
    assert np.array_equal(Cp[:, :, :N], oracle.gemm_epilogue(A, B))
    assert np.all(np.isnan(Cp[:, :, N:]))


def test_rejects_bad_arguments(oracle):
    A = np.ones(4); B = np.ones(4)
    with pytest.raises(ValueError):
        oracle.gemm_epilogue(A, B, M=2, N=2, K=2, lda=1, ldb=2, ldc=2)
    with pytest.raises(KeyError):
        oracle.gemm_epilogue(np.ones((2, 2)), np.ones((2, 2)), act="swish")


def test_thread_count_does_not_change_bits(oracle):
    import os, subprocess, sys, hashlib
    code = ("import numpy as np, oracle, hashlib;"
            "r=np.random.default_rng(1);A=r.normal(size=(37,300));B=r.normal(size=(300,41));"
            "print(hashlib.sha256(oracle.gemm_epilogue(A,B,None,0.3,'gelu_tanh').tobytes()).hexdigest())")
    outs = set()
    for t in ("1", "3", "8"):
        env = dict(os.environ, OMP_NUM_THREADS=t)
        root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
        outs.add(subprocess.run([sys.executable, "-c", code], env=env, cwd=root, check=True,
                                capture_output=True, text=True).stdout.strip())
    assert len(outs) == 1
