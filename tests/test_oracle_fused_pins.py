"""Pins for the oracle of the widened operator (oracle/gemm_fused_oracle.c).

    C = round_out(clamp(act(alpha*row_scale[m]*(opA(A) @ opB(B)) + bias[n] + beta*R)))

Every check compares it with something other than itself: exact rational brute
force, the separately pinned plain oracle, numpy on transposed copies, identities
of the consumer chain (Level-2 optimisation prompt, "Fusion" and its list of
consumer operations), and a library bfloat16 conversion for the output rounding.
Shapes are non-square and all extras are asymmetric, so that a swapped index, a
term applied at the wrong place or a wrong broadcast axis cannot pass.
"""
from fractions import Fraction
import itertools

import numpy as np
import pytest

from paper_2604_01489_amd import inputs as gen


def _rng(seed):
    return np.random.default_rng(seed)


def _store(X, trans, ld=None, fill=np.nan):
    """Storage of logical X (rows x cols): X or X.T with a padded leading dimension."""
    S = X.T if trans else X
    ld = S.shape[1] if ld is None else ld
    out = np.full((S.shape[0], ld), fill, dtype=X.dtype)
    out[:, :S.shape[1]] = S
    return out


FLAGS = list(itertools.product([False, True], repeat=2))


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("transA,transB", FLAGS)
def test_brute_force_exact_rationals(oracle, transA, transB):
    """The whole chain in exact rationals (relu keeps it rational), columns outermost."""
    r = _rng(40 + 2 * transA + transB)
    M, N, K, batch = 3, 4, 5, 2
    A = r.uniform(-1, 1, (batch, M, K)).astype(np.float32)
    B = r.uniform(-1, 1, (batch, K, N)).astype(np.float32)
    R = r.uniform(-1, 1, (batch, M, N)).astype(np.float32)
    rs = r.uniform(0.5, 2, M).astype(np.float32)
    bias = r.uniform(-1, 1, N).astype(np.float32)
    alpha, beta, lo, hi = 0.75, -0.5, 0.125, 0.875
    lda, ldb, ldr = (M if transA else K) + 3, (K if transB else N) + 2, N + 1
    As = np.stack([_store(A[b], transA, lda) for b in range(batch)])
    Bs = np.stack([_store(B[b], transB, ldb) for b in range(batch)])
    Rs = np.stack([_store(R[b], False, ldr) for b in range(batch)])
    got = oracle.gemm_fused(M, N, K, As, Bs, batch=batch, transA=transA, transB=transB, lda=lda, ldb=ldb,
                            alpha=alpha, row_scale=rs, bias=bias, residual=Rs, ldr=ldr, beta=beta,
                            act="relu", clamp=(lo, hi))
    F = lambda x: Fraction(float(x))
    for b in range(batch):
        for n in range(N):
            for m in range(M):
                p = sum(F(A[b, m, k]) * F(B[b, k, n]) for k in range(K))
                v = F(alpha) * F(rs[m]) * p + F(bias[n]) + F(beta) * F(R[b, m, n])
                y = max(v, Fraction(0))
                y = min(max(y, F(lo)), F(hi))
                ref = float(y)
                assert abs(got[b, m, n] - ref) <= 4 * np.spacing(max(abs(ref), 1e-3)), (b, m, n)
    # the clamp bit on both sides and left something inside, or this case pins nothing
    assert (got == lo).any() and (got == hi).any() and ((got > lo) & (got < hi)).any()


# ---------------------------------------------------------------- stored-transposed operands
@pytest.mark.parametrize("transA,transB", FLAGS)
@pytest.mark.parametrize("dtype", ["f64", "bf16"])
def test_layout_flags_change_storage_not_result(oracle, transA, transB, dtype):
    """With the extras off the result is the plain oracle's (pinned on its own) on the logical
    operands, bit for bit, whatever the storage."""
    r = _rng(7)
    M, N, K, batch = 6, 9, 11, 3
    A = r.normal(size=(batch, M, K))
    B = r.normal(size=(batch, K, N))
    bias = r.normal(size=N)
    if dtype == "bf16":
        A, B = gen.to_bf16_bits(A.astype(np.float32)), gen.to_bf16_bits(B.astype(np.float32))
        fill = np.uint16(0x7FC0)
    else:
        fill = np.nan
    lda, ldb = (M if transA else K) + 2, (K if transB else N) + 5
    As = np.stack([_store(A[b], transA, lda, fill) for b in range(batch)])
    Bs = np.stack([_store(B[b], transB, ldb, fill) for b in range(batch)])
    got = oracle.gemm_fused(M, N, K, As, Bs, batch=batch, transA=transA, transB=transB, lda=lda, ldb=ldb,
                            alpha=1.25, bias=bias, act="gelu_tanh")
    want = oracle.gemm_epilogue(A, B, bias, 1.25, "gelu_tanh")
    assert np.array_equal(got, want)


@pytest.mark.parametrize("transA,transB", FLAGS)
def test_against_numpy_matmul(oracle, transA, transB):
    r = _rng(11)
    M, N, K = 8, 5, 13
    A = r.normal(size=(M, K))
    B = r.normal(size=(K, N))
    got = oracle.gemm_fused(M, N, K, _store(A, transA), _store(B, transB), transA=transA, transB=transB)[0]
    assert np.allclose(got, A @ B, rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- row scale
def test_row_scale_is_diag_times_product(oracle):
    """Powers of two fold into A exactly: diag(d)*(A@B) == (diag(d)*A)@B, and the bias is not scaled."""
    r = _rng(12)
    M, N, K = 5, 7, 9
    A = r.normal(size=(M, K))
    B = r.normal(size=(K, N))
    bias = r.normal(size=N)
    d = 2.0 ** r.integers(-3, 4, M)
    got = oracle.gemm_fused(M, N, K, A, B, row_scale=d, bias=bias, alpha=0.5)[0]
    want = oracle.gemm_epilogue(d[:, None] * A, B, bias, 0.5, "none")
    assert np.array_equal(got, want)
    # per row, not per column
    d2 = np.arange(1.0, M + 1)
    g2 = oracle.gemm_fused(M, N, K, A, B, row_scale=d2)[0]
    assert np.allclose(g2, d2[:, None] * (A @ B), rtol=1e-13)


def test_diagonal_times_dense_special_case(oracle):
    """A = I: the operator reduces to the row scaling diag(d) @ B of the paper's diagonal-matmul case."""
    r = _rng(13)
    M, N = 6, 10
    B = r.normal(size=(M, N))
    d = r.normal(size=M)
    got = oracle.gemm_fused(M, N, M, np.eye(M), B, row_scale=d)[0]
    assert np.array_equal(got, d[:, None] * B)


# ---------------------------------------------------------------- residual
def test_residual_enters_before_activation_with_beta(oracle):
    r = _rng(14)
    M, N, K, batch = 4, 6, 3, 2
    A = r.normal(size=(batch, M, K))
    B = r.normal(size=(batch, K, N))
    R = r.normal(size=(batch, M, N))
    base = np.einsum("bmk,bkn->bmn", A, B)
    got = oracle.gemm_fused(M, N, K, A, B, batch=batch, residual=R, beta=-2.0, act="relu")
    assert np.allclose(got, np.maximum(base - 2.0 * R, 0.0), rtol=1e-13, atol=1e-13)
    # not relu(base) + beta*R, and not unscaled
    assert not np.allclose(got, np.maximum(base, 0.0) - 2.0 * R)
    assert not np.allclose(got, np.maximum(base + R, 0.0))
    # beta = 0 removes it; NaN padding beyond N is never read
    Rp = np.full((batch, M, N + 3), np.nan)
    Rp[:, :, :N] = R
    g0 = oracle.gemm_fused(M, N, K, A, B, batch=batch, residual=Rp, ldr=N + 3, beta=1.0)
    assert np.allclose(g0, base + R, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("rdtype", ["f32", "bf16"])
def test_residual_dtypes_widen_exactly(oracle, rdtype):
    r = _rng(15)
    M, N, K = 3, 5, 4
    A = r.normal(size=(M, K))
    B = r.normal(size=(K, N))
    R32 = r.normal(size=(M, N)).astype(np.float32)
    if rdtype == "bf16":
        Rs = gen.to_bf16_bits(R32)
        Rv = gen.bf16_bits_to_f32(Rs).astype(np.float64)
    else:
        Rs, Rv = R32, R32.astype(np.float64)
    got = oracle.gemm_fused(M, N, K, A, B, residual=Rs)[0]
    assert np.array_equal(got, oracle.gemm_fused(M, N, K, A, B, residual=Rv)[0])
    assert np.allclose(got, A @ B + Rv, rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- clamp
def test_clamp_follows_activation(oracle):
    r = _rng(16)
    M, N, K = 6, 8, 5
    A = r.normal(size=(M, K))
    B = r.normal(size=(K, N))
    pre = oracle.gemm_fused(M, N, K, A, B, alpha=2.0, act="gelu_tanh")[0]
    got = oracle.gemm_fused(M, N, K, A, B, alpha=2.0, act="gelu_tanh", clamp=(-0.1, 1.5))[0]
    assert np.array_equal(got, np.clip(pre, -0.1, 1.5))
    assert (got == -0.1).any() and (got == 1.5).any()
    # clamping the pre-activation instead gives something else
    lin = 2.0 * (A @ B)
    c = np.clip(lin, -0.1, 1.5)
    wrong = 0.5 * c * (1 + np.tanh(0.7978845608028654 * (c + 0.044715 * c ** 3)))
    assert not np.allclose(got, wrong)
    with pytest.raises(ValueError):
        oracle.gemm_fused(M, N, K, A, B, clamp=(1.0, -1.0))


# ---------------------------------------------------------------- output rounding
def test_bf16_rounding_matches_library_conversion(oracle):
    import torch
    r = _rng(17)
    x = np.concatenate([
        r.normal(size=4000).astype(np.float32) * np.float32(10.0) ** r.integers(-6, 7, 4000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 65504.0, 3.3895314e38, 1e-40, -1e-40, np.inf, -np.inf], dtype=np.float32),
    ])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.round_f32_to_bf16(v) for v in x], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.isnan(oracle.round_f32_to_bf16(float("nan")))


def test_bf16_rounding_ties_go_to_even(oracle):
    u = 2.0 ** -7                      # bf16 spacing in [1, 2)
    assert oracle.round_f32_to_bf16(1.0 + u / 2) == 1.0                 # tie, lower neighbour is even
    assert oracle.round_f32_to_bf16(1.0 + 3 * u / 2) == 1.0 + 2 * u     # tie, upper neighbour is even
    assert oracle.round_f32_to_bf16(1.0 + u / 2 + 2.0 ** -23) == 1.0 + u
    assert oracle.round_f32_to_bf16(1.0 + u / 2 - 2.0 ** -23) == 1.0
    assert oracle.round_f32_to_bf16(-(1.0 + 3 * u / 2)) == -(1.0 + 2 * u)
    assert oracle.round_f32_to_bf16(2.0 - u / 2) == 2.0                 # carries into the exponent


@pytest.mark.parametrize("out", ["f32", "bf16"])
def test_output_rounding_is_applied_last(oracle, out):
    import torch
    r = _rng(18)
    M, N, K = 7, 9, 6
    A = r.normal(size=(M, K))
    B = r.normal(size=(K, N))
    bias = r.normal(size=N)
    full = oracle.gemm_fused(M, N, K, A, B, bias=bias, act="gelu_tanh", clamp=(-0.05, 2.0))[0]
    got = oracle.gemm_fused(M, N, K, A, B, bias=bias, act="gelu_tanh", clamp=(-0.05, 2.0), out=out)[0]
    f32 = full.astype(np.float32)
    if out == "f32":
        want = f32.astype(np.float64)
    else:
        want = torch.from_numpy(f32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, want)
    assert not np.array_equal(got, full)


# ---------------------------------------------------------------- argument checks
def test_rejects_bad_arguments(oracle):
    A = np.zeros((4, 3))
    B = np.zeros((3, 5))
    with pytest.raises(ValueError):
        oracle.gemm_fused(4, 5, 3, A, B, lda=2)
    with pytest.raises(ValueError):
        oracle.gemm_fused(4, 5, 3, A, B, bias=np.zeros(4))
    with pytest.raises(ValueError):
        oracle.gemm_fused(4, 5, 3, A, B, row_scale=np.zeros(5))
    with pytest.raises(ValueError):
        oracle.gemm_fused(4, 5, 3, A, B, residual=np.zeros((4, 4)))
