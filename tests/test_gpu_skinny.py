"""GPU parity of the tall-skinny kernel (many rows, at most 32 columns: a workgroup owns 32 rows and
every column, K walked in stages of 128) against the CPU oracle, through the C-ABI: ragged M, N of 8 to
32, K from less than one stage to many with a ragged last one, padded leading dimensions, batches,
every activation, K slices (planner's own, caller's, caller's workspace), bitwise repeatability; and
the full-size shapes on sampled rows."""
import numpy as np
import pytest

from paper_2604_01489_amd import binding, inputs as gen

from gpu_util import compare, run_case, to_device

pytestmark = pytest.mark.gpu

DIRECT, SPLIT = "bf16_skinny_32xN_k128", "bf16_skinny_32xN_k128_splitk"


def test_skinny_shapes(oracle):
    for M, N, K, kw in [(1024, 32, 256, {}), (1056, 16, 1024, dict(act="gelu_tanh", alpha=0.125)),
                        (2000, 8, 72, dict(act="relu")), (1500, 24, 1288, dict(lda=1296, ldb=40, ldc=27, alpha=0.0625)),
                        (4096, 32, 520, dict(with_bias=False)), (2048, 16, 2048, dict(batch=3, act="relu", alpha=0.03))]:
        _, _, _, cfg = run_case(oracle, "bf16", M, N, K, seed=M + N + K, **kw)
        assert cfg == DIRECT, cfg
    # three batches of 1024 rows are 96 workgroups: the planner slices K in two
    _, _, _, cfg = run_case(oracle, "bf16", 1024, 16, 2048, batch=3, act="relu", alpha=0.03, seed=5)
    assert cfg == SPLIT, cfg


def test_skinny_k_slices(oracle):
    """Few rows and a long K: the planner slices K (1024 rows: 32 workgroups, 8 slices of 2048 at K = 16384);
    a caller's slice count and workspace; a ragged last slice."""
    assert binding.auto_split_k(1024, 32, 16384, 1) == 8
    _, _, _, cfg = run_case(oracle, "bf16", 1024, 32, 16384, alpha=1 / 128, seed=3)
    assert cfg == SPLIT, cfg
    for s in (2, 3, 5):
        _, _, _, cfg = run_case(oracle, "bf16", 1100, 16, 3000, alpha=1 / 64, act="gelu_tanh", seed=4 + s, plan="splitk",
                                split_k=s, workspace="caller")
        assert cfg == SPLIT, cfg
    _, _, _, cfg = run_case(oracle, "bf16", 1024, 32, 16384, alpha=1 / 128, seed=3, plan="direct")
    assert cfg == DIRECT, cfg


def test_skinny_is_repeatable_and_leaves_other_shapes_alone(oracle):
    a = run_case(oracle, "bf16", 2048, 32, 4096, alpha=1 / 64, seed=9)[0]
    b = run_case(oracle, "bf16", 2048, 32, 4096, alpha=1 / 64, seed=9)[0]
    assert np.array_equal(a, b)
    # more than 32 columns, few rows, a column count that is no multiple of 8, an unaligned pointer: other kernels
    for M, N, K, kw in [(2048, 40, 512, {}), (512, 32, 512, {}), (2048, 20, 512, {}), (2048, 32, 512, dict(misalign=1))]:
        cfg = run_case(oracle, "bf16", M, N, K, seed=M + N, **kw)[3]
        assert not cfg.startswith("bf16_skinny"), cfg


@pytest.mark.parametrize("M,N,K", [(8192, 32, 8192), (65536, 16, 1024), (16384, 8, 4096)])
def test_skinny_full_size_on_sampled_rows(oracle, M, N, K):
    """The tall-skinny shapes the measurements quote, at full size, in the launch configuration the library
    picks for them: 64 blocks of 32 rows spread over M (first and last included) against the oracle."""
    import torch
    A = gen.to_bf16_bits(gen.normal(77, gen.STREAM_A, M * K, K ** -0.5).reshape(M, K))
    B = gen.to_bf16_bits(gen.normal(77, gen.STREAM_B, K * N, 1.0).reshape(K, N))
    bias = gen.uniform(77, gen.STREAM_BIAS, N, -0.1, 0.1)
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
    print(f"skinny full size {M}x{N}x{K}", flush=True)
    binding.gemm_epilogue_bf16(M, N, K, to_device(A), K, to_device(B), N, to_device(bias), 0.5, "gelu_tanh", C, N)
    torch.cuda.synchronize()
    assert binding.last_config() == DIRECT
    got = C.cpu().numpy()
    assert np.all(np.isfinite(got))
    starts = np.unique(np.round(np.linspace(0, M - 32, 64)).astype(np.int64))
    rows = np.unique((starts[:, None] + np.arange(32)[None, :]).ravel())
    ref = oracle.gemm_epilogue(np.ascontiguousarray(A[rows]), B, bias, 0.5, "gelu_tanh")
    compare(got[rows], ref, f"skinny {M}x{N}x{K}")
