"""GPU parity of the row sum of a linear layer (gemm_rowsum_params_bf16 + gemm_rowsum_bf16, the collapsed
form) against its CPU oracle (the definition: full product, then the sum over the output dimension)."""
import numpy as np
import pytest

from gpu_util import to_device

pytestmark = pytest.mark.gpu

REL_FRO_TOL = 1e-3
ELEM_TOL = 1e-2


def run_rowsum_case(oracle, M, N, K, *, transB=False, alpha=1.0, with_bias=True, pad=(0, 0), misalign=0, seed=0):
    """``pad`` = extra elements on (lda, ldb); ``misalign`` shifts A and B by that many elements."""
    import torch
    from paper_2604_01489_amd import binding, inputs as gen
    A = gen.to_bf16_bits(gen.uniform(seed, gen.STREAM_A, M * K, -1.0, 1.0).reshape(M, K))
    B = gen.to_bf16_bits(gen.uniform(seed, gen.STREAM_B, K * N, -1.0, 1.0).reshape(K, N))
    bias = gen.uniform(seed, gen.STREAM_BIAS, N, -1.0, 1.0) if with_bias else None
    rowsB, colsB = (N, K) if transB else (K, N)
    lda, ldb = K + pad[0], colsB + pad[1]
    junk = np.uint16(0x7F00)                                   # a large finite bf16 in every padding element
    As = np.full((M, lda), junk, dtype=np.uint16)
    As[:, :K] = A
    Bs = np.full((rowsB, ldb), junk, dtype=np.uint16)
    Bs[:, :colsB] = B.T if transB else B

    def shifted(flat):
        buf = np.full(flat.size + misalign, junk, dtype=np.uint16)
        buf[misalign:] = flat
        t = to_device(buf)
        return t, t[misalign:]

    keepA, dA = shifted(As.ravel())
    keepB, dB = shifted(Bs.ravel())
    dbias = to_device(bias)
    params = torch.full((K + 2,), -7.0e30, dtype=torch.float32, device="cuda:0")
    y = torch.full((M + 1,), -7.0e30, dtype=torch.float32, device="cuda:0")
    print(f"rowsum case M={M} N={N} K={K} transB={transB} alpha={alpha} bias={with_bias} pad={pad} misalign={misalign}",
          flush=True)
    binding.gemm_rowsum_params_bf16(N, K, dB, ldb, transB, dbias, params)
    cfg_p = binding.last_config()
    binding.gemm_rowsum_bf16(M, K, dA, lda, params, alpha, y)
    cfg_y = binding.last_config()
    torch.cuda.synchronize()
    canary = float(np.float32(-7.0e30))
    assert float(params[K + 1]) == canary and float(y[M]) == canary, "wrote past an output"
    got = y[:M].cpu().numpy().astype(np.float64)
    ref = oracle.gemm_rowsum(A, B, bias, alpha)
    # the parameter sums against numpy in fp64 (their own check: an error there would be averaged away in y)
    Bf = gen.bf16_bits_to_f32(B).astype(np.float64)
    s_ref = Bf.sum(axis=1)
    s_got = params[:K].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(s_got - s_ref) <= 1e-5 * np.abs(Bf).sum(axis=1) + 1e-30), f"{cfg_p}: parameter sums"
    t_ref = 0.0 if bias is None else float(bias.astype(np.float64).sum())
    assert abs(float(params[K]) - t_ref) <= 1e-5 * (1.0 + (0.0 if bias is None else float(np.abs(bias).sum())))
    err = np.abs(got - ref)
    assert np.all(np.isfinite(got))
    assert np.all(err <= ELEM_TOL * np.maximum(1.0, np.abs(ref))), f"{cfg_y}: element {int(np.argmax(err))}"
    rel = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
    assert rel <= REL_FRO_TOL, f"{cfg_y}: relative Frobenius error {rel:.3e}"
    assert rel <= 1e-5, f"{cfg_y}: error {rel:.3e} is far above fp32 accumulation noise"
    del keepA, keepB
    return got, cfg_p, cfg_y


@pytest.mark.parametrize("transB", [False, True])
def test_rowsum_shapes(oracle, transB):
    cols = "rowsum_params_cols" if transB else "rowsum_params_rows"
    for M, N, K, pad in [(64, 48, 32, (0, 0)), (300, 520, 264, (8, 16)), (1024, 1032, 2048, (0, 0)), (33, 7, 13000, (0, 8))]:
        _, cfg_p, cfg_y = run_rowsum_case(oracle, M, N, K, transB=transB, alpha=0.5, pad=pad, seed=M + N)
        assert cfg_p == cols and cfg_y == ("rowsum_rows_wide" if K >= 384 else "rowsum_rows_vec8")


@pytest.mark.parametrize("transB", [False, True])
def test_rowsum_wide_rows(oracle, transB):
    """Rows of 384 columns and more take the kernel in which a group of waves owns 8 rows and a block of
    1024 threads 8 to 128 of them: every group width (sweeps of 512 ... 8192 columns), sweeps partly filled,
    exactly one, two with a ragged second one, row counts that are no multiple of a block's rows, padded
    leading dimensions; with B stored K x N and N wide the parameter pass takes it too (with no vector to
    multiply by)."""
    for M, N, K, pad in [(77, 40, 4096, (0, 0)), (8, 24, 8192, (16, 8)), (21, 16, 8192 + 520, (8, 0)), (16, 4104, 56, (0, 8)),
                         (133, 8, 392, (0, 0)), (259, 8, 1016, (8, 0)), (70, 8, 2048, (0, 0)), (300, 8, 1032, (0, 0))]:
        _, _, cfg_y = run_rowsum_case(oracle, M, N, K, transB=transB, alpha=0.5, pad=pad, seed=M + N + K)
        assert cfg_y == ("rowsum_rows_wide" if K >= 384 else "rowsum_rows_vec8")


@pytest.mark.parametrize("transB", [False, True])
def test_rowsum_odd_and_unaligned(oracle, transB):
    """Sizes that are no multiple of 8, odd leading dimensions, pointers shifted by one element."""
    for M, N, K, pad, mis in [(45, 67, 33, (0, 0), 0), (130, 129, 257, (3, 5), 0), (64, 64, 64, (0, 0), 1), (5, 3, 1, (0, 0), 3)]:
        _, _, cfg_y = run_rowsum_case(oracle, M, N, K, transB=transB, alpha=-0.75, pad=pad, misalign=mis, seed=7 * M + K)
        assert cfg_y == ("rowsum_rows_vec8" if (mis == 0 and (K + pad[0]) % 8 == 0) else "rowsum_rows_generic")


def test_rowsum_no_bias_and_repeatable(oracle):
    a, _, _ = run_rowsum_case(oracle, 512, 384, 1024, transB=True, with_bias=False, seed=3)
    b, _, _ = run_rowsum_case(oracle, 512, 384, 1024, transB=True, with_bias=False, seed=3)
    assert np.array_equal(a, b)


def test_rowsum_equals_the_layer_then_the_sum(oracle):
    """The same quantity the long way round on the GPU: the fused operator's fp32 output summed over n
    (torch, fp64) agrees with the collapsed form to fp32 accumulation noise."""
    import torch
    from paper_2604_01489_amd import binding, inputs as gen
    M, N, K = 512, 768, 1024
    A = gen.to_bf16_bits(gen.uniform(11, gen.STREAM_A, M * K, -1.0, 1.0).reshape(M, K))
    W = gen.to_bf16_bits(gen.uniform(11, gen.STREAM_B, N * K, -1.0, 1.0).reshape(N, K))      # weights as stored: N x K
    bias = gen.uniform(11, gen.STREAM_BIAS, N, -1.0, 1.0)
    dA, dW, dbias = to_device(A), to_device(W), to_device(bias)
    C = torch.empty(M, N, dtype=torch.float32, device="cuda:0")
    binding.gemm_epilogue_bf16_fused(M, N, K, dA, K, dW, K, C, N, transB=True, alpha=0.25, bias=dbias)
    params = torch.empty(K + 1, dtype=torch.float32, device="cuda:0")
    y = torch.empty(M, dtype=torch.float32, device="cuda:0")
    binding.gemm_rowsum_params_bf16(N, K, dW, K, True, dbias, params)
    binding.gemm_rowsum_bf16(M, K, dA, K, params, 0.25, y)
    torch.cuda.synchronize()
    long_way = C.double().sum(dim=1).cpu().numpy()
    short_way = y.double().cpu().numpy()
    assert np.linalg.norm(long_way - short_way) <= 1e-5 * np.linalg.norm(long_way)
