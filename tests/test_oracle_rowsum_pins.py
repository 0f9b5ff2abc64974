"""Pins of oracle.gemm_rowsum (the row sum of a linear layer) to something other than itself: exact
rational brute force, closed forms, the collapsed formulation in a library routine, and the mistakes a
two-line function can still make (wrong axis, bias forgotten or scaled, alpha misplaced)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2604_01489_amd import inputs as gen


@pytest.fixture(scope="module", autouse=True)
def _built():
    oracle.build()


def _bf16_vals(seed, stream, shape, lo=-2.0, hi=2.0):
    bits = gen.to_bf16_bits(gen.uniform(seed, stream, int(np.prod(shape)), lo, hi).reshape(shape))
    return bits, gen.bf16_bits_to_f32(bits).astype(np.float64)


def test_exact_rational_brute_force():
    """Small integers: every product and sum is exact in fp64, and python fractions give the truth."""
    rng = np.random.default_rng(7)
    M, N, K = 5, 7, 4                                         # all different: a wrong axis cannot pass
    A = rng.integers(-4, 5, size=(M, K)).astype(np.float64)
    B = rng.integers(-4, 5, size=(K, N)).astype(np.float64)
    bias = rng.integers(-3, 4, size=N).astype(np.float64)
    alpha = 0.5
    want = []
    for m in range(M):
        tot = Fraction(0)
        for n in range(N):
            dot = sum(Fraction(int(A[m, k])) * Fraction(int(B[k, n])) for k in range(K))
            tot += Fraction(1, 2) * dot + Fraction(int(bias[n]))
        want.append(float(tot))
    got = oracle.gemm_rowsum(A, B, bias, alpha)
    assert got.shape == (M,)
    assert np.array_equal(got, np.array(want))


def test_closed_form_ones():
    """A and B of ones: every product entry is K, so y = alpha*K*N + sum(bias) for every row."""
    M, N, K = 6, 10, 12
    bias = np.arange(N, dtype=np.float64) * 0.25 - 1.0
    got = oracle.gemm_rowsum(np.ones((M, K)), np.ones((K, N)), bias, 0.75)
    assert np.array_equal(got, np.full(M, 0.75 * K * N + bias.sum()))


def test_bias_enters_once_per_column_unscaled():
    M, N, K = 3, 9, 5
    A, B = np.zeros((M, K)), np.zeros((K, N))
    bias = np.linspace(-1.0, 2.0, N)
    assert np.allclose(oracle.gemm_rowsum(A, B, bias, 123.0), bias.sum(), rtol=0, atol=1e-15)   # alpha does not touch it
    assert np.array_equal(oracle.gemm_rowsum(A, B, None, 2.0), np.zeros(M))


def test_alpha_scales_the_product_only():
    rng = np.random.default_rng(3)
    A, B, bias = rng.standard_normal((4, 6)), rng.standard_normal((6, 8)), rng.standard_normal(8)
    y1 = oracle.gemm_rowsum(A, B, bias, 1.0)
    y3 = oracle.gemm_rowsum(A, B, bias, 3.0)
    assert np.allclose(y3 - bias.sum(), 3.0 * (y1 - bias.sum()), rtol=1e-13, atol=1e-13)


def test_collapsed_form_in_a_library_routine():
    """The identity the GPU path relies on, evaluated independently with numpy in fp64 on bf16-valued
    inputs of a realistic shape: alpha * A @ (B @ 1) + sum(bias)."""
    M, N, K = 37, 129, 200
    Ab, A = _bf16_vals(1, gen.STREAM_A, (M, K))
    Bb, B = _bf16_vals(1, gen.STREAM_B, (K, N))
    bias = gen.uniform(1, gen.STREAM_BIAS, N, -1.0, 1.0).astype(np.float64)     # fp32 values, fp64 arithmetic below
    want = 0.5 * (A @ B.sum(axis=1)) + bias.sum()
    got = oracle.gemm_rowsum(Ab, Bb, bias, 0.5)
    scale = np.abs(A) @ np.abs(B).sum(axis=1) + np.abs(bias).sum()
    assert np.all(np.abs(got - want) <= 1e-13 * scale)


def test_rows_are_independent_and_ordered():
    """Row m of the result depends on row m of A only, and rows keep their order."""
    rng = np.random.default_rng(5)
    A, B = rng.standard_normal((6, 5)), rng.standard_normal((5, 4))
    y = oracle.gemm_rowsum(A, B)
    perm = np.array([3, 0, 5, 1, 4, 2])
    assert np.array_equal(oracle.gemm_rowsum(A[perm], B), y[perm])
    A2 = A.copy()
    A2[2] += 1.0
    y2 = oracle.gemm_rowsum(A2, B)
    assert np.array_equal(np.delete(y2, 2), np.delete(y, 2)) and y2[2] != y[2]
    assert np.isclose(y2[2] - y[2], B.sum(), rtol=1e-12)
