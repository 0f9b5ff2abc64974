"""Pins of the symmetric-operand oracle (oracle/gemm_symm_oracle.c) to things other than itself.

The paper's optimisation prompt ("Rules for GEMM") names the symmetric operand as a structure whose
reads can be reduced; what is computed is the ordinary product with the full symmetric matrix that
one stored triangle stands for.  The pins: exact rational arithmetic on tiny inputs, the separately
pinned oracle of the widened operator on the explicitly mirrored dense matrix, a library matmul,
closed forms, and the property that the unread triangle may hold anything."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2604_01489_amd import inputs as gen


def mirrored(A, uplo):
    """The full symmetric matrix a stored triangle stands for, by numpy indexing (no arithmetic)."""
    A = np.asarray(A)
    return np.where(np.tri(A.shape[0], dtype=bool), A, A.T) if uplo == "lower" else np.where(np.tri(A.shape[0], dtype=bool).T, A, A.T)


def small_ints(seed, shape, lo=-4, hi=5):
    return np.random.default_rng(seed).integers(lo, hi, shape).astype(np.float64)


@pytest.mark.parametrize("uplo", ["lower", "upper"])
def test_exact_rational_brute_force(oracle, uplo):
    """Tiny case in python Fractions, k outermost (another loop order), reading the triangle by its
    definition: S[m,k] = A[max(m,k), min(m,k)] for lower, A[min, max] for upper."""
    M, N = 5, 3
    A = small_ints(1, (M, M)) / 4.0
    B = small_ints(2, (M, N)) / 8.0
    bias = small_ints(3, (N,)) / 2.0
    alpha = 0.75
    acc = [[Fraction(0) for _ in range(N)] for _ in range(M)]
    for k in range(M):
        for m in range(M):
            i, j = (max(m, k), min(m, k)) if uplo == "lower" else (min(m, k), max(m, k))
            for n in range(N):
                acc[m][n] += Fraction(A[i, j]) * Fraction(B[k, n])
    want = np.array([[float(Fraction(alpha) * acc[m][n] + Fraction(bias[n])) for n in range(N)] for m in range(M)])
    got = oracle.gemm_symm(M, N, A, B, uplo=uplo, alpha=alpha, bias=bias)[0]
    assert np.array_equal(got, want)


@pytest.mark.parametrize("uplo", ["lower", "upper"])
@pytest.mark.parametrize("transB", [False, True])
def test_equals_the_widened_oracle_on_the_mirrored_matrix(oracle, uplo, transB):
    """Whole chain, bf16 operands, padded leading dimensions, two batches: identical (same k order, same
    fp64 arithmetic) to the pinned oracle of the widened operator given the dense mirrored matrix."""
    M, N, batch, lda, ldb = 23, 9, 2, 27, 30
    A = gen.to_bf16_bits(gen.normal(5, 0, batch * M * lda, 1.0).reshape(batch, M, lda))
    B = gen.to_bf16_bits(gen.normal(5, 1, batch * max(M, N) * ldb, 1.0).reshape(batch, max(M, N), ldb))[:, :(N if transB else M)]
    rs = gen.uniform(5, 7, M, 0.5, 1.5).astype(np.float64)
    bias = gen.uniform(5, 2, N, -1, 1).astype(np.float64)
    R = gen.uniform(5, 8, batch * M * N, -1, 1).reshape(batch, M, N)
    dense = np.stack([mirrored(A[b][:, :M], uplo) for b in range(batch)])
    kw = dict(alpha=0.3, row_scale=rs, bias=bias, residual=R, beta=0.5, act="gelu_tanh", clamp=(-0.1, 2.0), out="bf16")
    want = oracle.gemm_fused(M, N, M, np.ascontiguousarray(dense), np.ascontiguousarray(B), batch=batch, transB=transB, ldb=ldb, **kw)
    got = oracle.gemm_symm(M, N, A, np.ascontiguousarray(B), uplo=uplo, batch=batch, transB=transB, lda=lda, ldb=ldb, **kw)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("uplo", ["lower", "upper"])
def test_library_matmul_on_integers(oracle, uplo):
    """Small integers: every product and sum is exact, so numpy's matmul on the mirrored matrix must
    agree exactly whatever its summation order."""
    M, N = 40, 17
    A, B = small_ints(11, (M, M)), small_ints(12, (M, N))
    assert np.array_equal(oracle.gemm_symm(M, N, A, B, uplo=uplo)[0], mirrored(A, uplo) @ B)


@pytest.mark.parametrize("uplo", ["lower", "upper"])
def test_the_other_triangle_is_never_read(oracle, uplo):
    M, N = 19, 6
    A, B = small_ints(21, (M, M)), small_ints(22, (M, N))
    clean = oracle.gemm_symm(M, N, A, B, uplo=uplo)[0]
    poisoned = A.copy()
    unread = ~np.tri(M, dtype=bool) if uplo == "lower" else ~np.tri(M, dtype=bool).T
    poisoned[unread] = np.nan
    got = oracle.gemm_symm(M, N, poisoned, B, uplo=uplo)[0]
    assert np.all(np.isfinite(got)) and np.array_equal(got, clean)


def test_the_two_readings_agree_on_a_symmetric_array_and_differ_on_another(oracle):
    M, N = 12, 5
    T = small_ints(31, (M, M))
    S = T + T.T
    B = small_ints(32, (M, N))
    assert np.array_equal(oracle.gemm_symm(M, N, S, B, uplo="lower")[0], oracle.gemm_symm(M, N, S, B, uplo="upper")[0])
    assert np.array_equal(oracle.gemm_symm(M, N, S, B, uplo="lower")[0], S @ B)
    lower, upper = oracle.gemm_symm(M, N, T, B, uplo="lower")[0], oracle.gemm_symm(M, N, T, B, uplo="upper")[0]
    assert not np.array_equal(lower, upper)
    # lower reading of T is the upper reading of its transpose
    assert np.array_equal(lower, oracle.gemm_symm(M, N, np.ascontiguousarray(T.T), B, uplo="upper")[0])


def test_closed_forms(oracle):
    """All-ones triangle: S is all ones, every row of C is the column sums of B (a dropped mirror or a
    diagonal counted twice changes it).  Diagonal only: C = d[m] * B[m,:]."""
    M, N = 9, 4
    B = small_ints(41, (M, N))
    ones_lower = np.tril(np.ones((M, M)))
    assert np.array_equal(oracle.gemm_symm(M, N, ones_lower, B, uplo="lower")[0], np.tile(B.sum(axis=0), (M, 1)))
    ones_upper = np.triu(np.ones((M, M)))
    assert np.array_equal(oracle.gemm_symm(M, N, ones_upper, B, uplo="upper")[0], np.tile(B.sum(axis=0), (M, 1)))
    d = np.arange(1.0, M + 1)
    assert np.array_equal(oracle.gemm_symm(M, N, np.diag(d), B)[0], d[:, None] * B)


def test_identity_and_batches(oracle):
    """A = I gives the chain on B; batch b equals the single-problem call on slice b."""
    M, N, batch = 7, 5, 3
    B = small_ints(51, (batch, M, N))
    bias = small_ints(52, (N,))
    got = oracle.gemm_symm(M, N, np.stack([np.eye(M)] * batch), B, batch=batch, alpha=2.0, bias=bias, act="relu")
    assert np.array_equal(got, np.maximum(2.0 * B + bias, 0.0))
    A = small_ints(53, (batch, M, M))
    whole = oracle.gemm_symm(M, N, A, B, batch=batch, uplo="upper")
    for b in range(batch):
        assert np.array_equal(whole[b], oracle.gemm_symm(M, N, A[b], B[b], uplo="upper")[0])


def test_bad_arguments_are_rejected(oracle):
    A, B = np.zeros((4, 4)), np.zeros((4, 3))
    with pytest.raises(ValueError):
        oracle.gemm_symm(4, 3, A, B, lda=3)
    with pytest.raises(ValueError):
        oracle.gemm_symm(4, 3, A, B, clamp=(1.0, 0.0))
    with pytest.raises(KeyError):
        oracle.gemm_symm(4, 3, A, B, uplo="full")
