"""GPU parity of the widened operator (gemm_epilogue_bf16_fused) against its CPU oracle:
operands stored either way round, row scale, residual, clamp, fp32 and bf16 output, on the
direct-to-LDS kernels (256 and 128 tiles), the guarded kernel and the split-K path."""
import itertools
import os

import numpy as np
import pytest

from paper_2604_01489_amd import binding

from gpu_util import run_case, run_fused_case

pytestmark = pytest.mark.gpu

LAYOUTS = list(itertools.product([False, True], repeat=2))
NAME = {(False, False): "nn", (False, True): "nt", (True, False): "tn", (True, True): "tt"}


def stage_k(transA, transB, shared_cu=True):
    """k per load phase the library picks for a layout (64 where both operands' rows run along k; with
    128 x 128 blocks only when more than 256 blocks are launched, so that blocks share a CU);
    GE_STAGE_K=32 switches that off for timing runs."""
    if os.environ.get("GE_STAGE_K") == "32":
        return 32
    return 64 if (not transA and transB and shared_cu) else 32


@pytest.mark.parametrize("transA,transB", LAYOUTS)
def test_layouts_tile_256(oracle, transA, transB, monkeypatch):
    """Full and ragged tiles, several K tiles (ring) and few (one load phase); leading dimensions padded.
    (The 256 x 256 kernel is forced: by the planning rule so few tiles go to the 128 x 128 kernel.)"""
    binding.set_option("force_config", "256x256")
    binding.set_option("waves", "8")         # the four-wave kernel has its own tests
    for M, N, K, pad in [(256, 256, 64, (0, 0, 0, 0)), (512, 768, 256, (8, 16, 0, 4)), (520, 776, 328, (24, 8, 0, 0))]:
        _, _, _, cfg = run_fused_case(oracle, M, N, K, transA=transA, transB=transB, alpha=0.5, act="gelu_tanh",
                                      with_row_scale=True, pad=pad, seed=M + K + 2 * transA + transB)
        assert cfg == f"bf16_fused_256x256x{stage_k(transA, transB)}_w8_{NAME[transA, transB]}"


@pytest.mark.parametrize("transA,transB", LAYOUTS)
def test_layouts_tile_128(oracle, transA, transB):
    for M, N, K in [(128, 128, 192), (136, 248, 200), (8, 8, 8), (64, 384, 40)]:
        _, _, _, cfg = run_fused_case(oracle, M, N, K, transA=transA, transB=transB, act="relu", with_row_scale=True,
                                      seed=3 * M + K)
        assert cfg == f"bf16_fused_128x128x{stage_k(transA, transB, shared_cu=False)}_w4_{NAME[transA, transB]}"
    # more blocks than CUs (17 x 17 full and ragged tiles): 64 k per load phase where both operands run along k
    for M, N, K in [(2176, 2176, 192), (2184, 2168, 200)]:
        _, _, _, cfg = run_fused_case(oracle, M, N, K, transA=transA, transB=transB, act="relu", with_row_scale=True,
                                      out="bf16", seed=3 * M + K, plan="direct")
        assert cfg == f"bf16_fused_128x128x{stage_k(transA, transB)}_w4_{NAME[transA, transB]}"


@pytest.mark.parametrize("transA,transB", LAYOUTS)
def test_layouts_guarded_kernel(oracle, transA, transB):
    for M, N, K, mis in [(67, 45, 33, 0), (130, 70, 100, 0), (1, 1, 1, 0), (128, 128, 64, 1)]:
        _, _, _, cfg = run_fused_case(oracle, M, N, K, transA=transA, transB=transB, act="gelu_tanh", alpha=1.5,
                                      with_row_scale=True, residual="f32", beta=0.5, clamp=(-0.1, 2.0),
                                      pad=(1, 3, 2, 5), misalign=mis, seed=M + N)
        assert cfg == f"bf16_fused_generic_64x64x32_{NAME[transA, transB]}"


@pytest.mark.parametrize("out", ["f32", "bf16"])
@pytest.mark.parametrize("residual", [None, "f32", "bf16"])
def test_epilogue_chain(oracle, out, residual):
    """Row scale, bias, residual with beta, activation and a clamp that bites on both sides."""
    for (M, N, K), (tA, tB) in [((520, 264, 136), (False, True)), ((128, 136, 72), (True, False))]:
        got, _, _, cfg = run_fused_case(oracle, M, N, K, transA=tA, transB=tB, alpha=0.75, with_row_scale=True,
                                        residual=residual, beta=-0.5, act="gelu_tanh", clamp=(-0.05, 1.25), out=out,
                                        pad=(0, 0, 8, 8), seed=11 + M)
        assert "generic" not in cfg
        assert (got == np.float32(-0.05)).any() or out == "bf16"
        assert got.max() <= 1.25 + 1e-6


@pytest.mark.parametrize("out", ["f32", "bf16"])
@pytest.mark.parametrize("clamp", [(-0.5, 0.75), (0.25, 0.75), (-0.75, -0.25), (0.0, 0.0), None])
def test_relu_then_clamp(oracle, out, clamp):
    """relu followed by a clamp whose interval lies across, above or below zero (the kernels fold the
    relu into the bounds: below zero the result is the constant upper bound)."""
    got, ref, _, cfg = run_fused_case(oracle, 264, 264, 72, act="relu", clamp=clamp, residual="bf16", out=out,
                                      seed=31)
    assert "generic" not in cfg
    if clamp == (-0.75, -0.25):
        assert (got == np.float32(-0.25)).all()
    if clamp == (0.25, 0.75):
        assert got.min() == np.float32(0.25) and got.max() == np.float32(0.75)
    run_fused_case(oracle, 45, 67, 33, act="relu", clamp=clamp, out=out, seed=32)       # guarded kernel


@pytest.mark.parametrize("structure", ["lower", "upper"])
@pytest.mark.parametrize("transA,transB", LAYOUTS)
def test_triangular_a(oracle, structure, transA, transB):
    """A promised triangular: the library skips the K ranges in which a whole tile row of A is zero.
    Same result as the oracle on that A (which is told nothing), and bit for bit the result of the
    same call without the promise (the skipped terms are exact zeros)."""
    cases = [(768, 520, 768, "f32", {}),                      # 256 tiles, square A, ragged N
             (520, 264, 1032, "bf16", {}),                    # K > M, ragged everything
             (1032, 256, 520, "f32", {}),                     # M > K: tile rows past the last column
             (392, 136, 392, "bf16", dict(pad=(8, 8, 0, 8))), # 128 tiles (N < 256)
             (200, 67, 131, "f32", {})]                       # guarded kernel
    for M, N, K, out, extra in cases:
        kw = dict(transA=transA, transB=transB, alpha=0.5, act="relu", with_row_scale=True, out=out,
                  seed=50 + M + K, a_structure=structure, plan="direct", **extra)      # one pass, the same order of sums
        got, _, _, cfg = run_fused_case(oracle, M, N, K, **kw)
        plain, _, _, cfg2 = run_fused_case(oracle, M, N, K, hint=False, **kw)
        assert cfg == cfg2
        assert np.array_equal(got, plain), f"{cfg}: the promise changed the result"
    # batched, and the promise is not compatible with K slices
    run_fused_case(oracle, 512, 256, 512, batch=3, transA=transA, transB=transB, residual="bf16", out="bf16",
                   seed=60, a_structure=structure)
    with pytest.raises(Exception):
        run_fused_case(oracle, 256, 256, 2048, transA=transA, transB=transB, plan="splitk", split_k=4,
                       a_structure=structure)


def test_bf16_output_all_paths(oracle):
    run_fused_case(oracle, 512, 512, 128, out="bf16", act="relu", seed=21)                       # 256 tile, full
    run_fused_case(oracle, 264, 520, 72, out="bf16", act="none", pad=(0, 0, 0, 6), seed=22)      # 256 tile, ragged, ldc even
    run_fused_case(oracle, 72, 136, 40, out="bf16", act="gelu_tanh", seed=23)                    # 128 tile
    _, _, _, cfg = run_fused_case(oracle, 72, 136, 40, out="bf16", pad=(0, 0, 0, 3), seed=24)    # odd ldc -> guarded
    assert "generic" in cfg
    _, _, _, cfg = run_fused_case(oracle, 45, 67, 33, out="bf16", act="relu", seed=25)
    assert "generic" in cfg


def test_batched(oracle):
    run_fused_case(oracle, 256, 256, 64, batch=5, transB=True, act="relu", residual="bf16", out="bf16", seed=31)
    run_fused_case(oracle, 136, 72, 48, batch=4, transA=True, with_row_scale=True, pad=(8, 8, 0, 4), seed=32)
    run_fused_case(oracle, 33, 65, 17, batch=3, transA=True, transB=True, residual="f32", seed=33)


@pytest.mark.parametrize("transA,transB", LAYOUTS)
def test_split_k(oracle, transA, transB, monkeypatch):
    _, _, _, cfg = run_fused_case(oracle, 256, 256, 4096, transA=transA, transB=transB, alpha=1.0 / 64, act="gelu_tanh",
                                  with_row_scale=True, residual="f32", clamp=(-1.0, 1.0), out="bf16",
                                  plan="splitk", split_k=0, seed=41)
    assert cfg == f"bf16_fused_128x128x{stage_k(transA, transB, shared_cu=False)}_w4_{NAME[transA, transB]}_splitk"
    binding.set_option("force_config", "256x256")
    binding.set_option("waves", "8")         # the four-wave kernel has its own tests
    _, _, _, cfg = run_fused_case(oracle, 256, 256, 4096, transA=transA, transB=transB, alpha=1.0 / 64, act="gelu_tanh",
                                  with_row_scale=True, residual="f32", clamp=(-1.0, 1.0), out="bf16",
                                  plan="splitk", split_k=0, seed=41)
    assert cfg == f"bf16_fused_256x256x{stage_k(transA, transB)}_w8_{NAME[transA, transB]}_splitk"
    binding.set_option("waves", None)
    _, _, _, cfg = run_fused_case(oracle, 130, 70, 1500, transA=transA, transB=transB, alpha=1.0 / 32,
                                  with_row_scale=True, plan="splitk", split_k=3, seed=42)
    assert cfg == f"bf16_fused_generic_64x64x32_{NAME[transA, transB]}_splitk"
    binding.set_option("force_config", None)


def test_plain_operator_is_the_special_case(oracle):
    """Extras off, fp32 output, both operands as stored by the plain entry point: the call is routed to
    the plain operator's kernels (same bits); one extra switched on keeps the fused kernel."""
    for M, N, K in [(512, 512, 256), (200, 136, 72), (67, 45, 33)]:
        got_f, _, _, cfg_f = run_fused_case(oracle, M, N, K, alpha=0.5, act="gelu_tanh", seed=5)
        got_p, _, _, cfg_p = run_case(oracle, "bf16", M, N, K, alpha=0.5, act="gelu_tanh", seed=5)
        assert cfg_f == cfg_p and not cfg_f.startswith("bf16_fused")
        assert np.array_equal(got_f, got_p)
    _, _, _, cfg = run_fused_case(oracle, 512, 512, 256, alpha=0.5, act="gelu_tanh", clamp=(-1.0, 1.0), seed=5)
    assert cfg == f"bf16_fused_128x128x{stage_k(False, False)}_w4_nn"


def test_diagonal_times_dense(oracle):
    """A = identity with a row scale: the row scaling diag(d) @ B as a special case of the operator."""
    import torch
    from paper_2604_01489_amd import inputs as gen
    M, N = 256, 512
    dev = torch.device("cuda:0")
    B32 = gen.uniform(9, 1, M * N, -1.0, 1.0).reshape(M, N)
    Bb = gen.to_bf16_bits(B32)
    d = gen.uniform(9, 7, M, -2.0, 2.0)
    eye = gen.to_bf16_bits(np.eye(M, dtype=np.float32))
    dA = torch.from_numpy(eye.view(np.int16)).to(dev)
    dB = torch.from_numpy(Bb.view(np.int16)).to(dev)
    dd = torch.from_numpy(d).to(dev)
    C = torch.empty(M, N, dtype=torch.float32, device=dev)
    binding.gemm_epilogue_bf16_fused(M, N, M, dA, M, dB, N, C, N, row_scale=dd)
    torch.cuda.synchronize()
    want = d.astype(np.float64)[:, None] * gen.bf16_bits_to_f32(Bb).astype(np.float64)
    assert np.allclose(C.cpu().numpy(), want, rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("M,N,batch,pad,act", [
    (256, 512, 1, (0, 0), "none"),          # 16-byte row pieces
    (300, 1000, 3, (8, 4), "relu"),         # padded leading dimensions, still in pieces
    (67, 45, 2, (3, 1), "gelu_tanh"),       # odd sizes: element-wise kernel
    (1, 1, 1, (0, 0), "relu"),
])
def test_diag_entry_point(oracle, M, N, batch, pad, act):
    """gemm_epilogue_diag_bf16 against the operator's definition with the dense matrix diag(d) as A
    (the fused oracle with A = I and row_scale = d, pinned to d[:, None] * B on the CPU)."""
    import torch
    from paper_2604_01489_amd import inputs as gen
    dev = torch.device("cuda:0")
    ldb, ldc = N + pad[0], N + pad[1]
    Bb = gen.to_bf16_bits(gen.normal(50 + M, 1, batch * M * N, 1.0).reshape(batch, M, N))
    d = gen.uniform(50 + M, 7, M, -2.0, 2.0)
    bias = gen.uniform(50 + M, 2, N, -1.0, 1.0)
    Bs = np.full((batch, M, ldb), np.uint16(0x7F00), dtype=np.uint16)
    Bs[:, :, :N] = Bb
    dB = torch.from_numpy(Bs.view(np.int16)).to(dev)
    dd, dbias = torch.from_numpy(d).to(dev), torch.from_numpy(bias).to(dev)
    C = torch.full((batch, M, ldc), -7.0e30, dtype=torch.float32, device=dev)
    print(f"diag case M={M} N={N} batch={batch} pad={pad} act={act}", flush=True)
    binding.gemm_epilogue_diag_bf16(M, N, dd, dB, ldb, dbias, 0.75, act, C, ldc, batch)
    torch.cuda.synchronize()
    cfg = binding.last_config()
    assert cfg == ("diag_rows_vec4" if N % 4 == 0 and ldb % 4 == 0 and ldc % 4 == 0 else "diag_rows_generic")
    out = C.cpu().numpy()
    assert np.all(out[:, :, N:] == np.float32(-7.0e30)), "wrote into the padding of C"
    eye = gen.to_bf16_bits(np.broadcast_to(np.eye(M, dtype=np.float32), (batch, M, M)).copy())
    ref = oracle.gemm_fused(M, N, M, eye, Bs, batch=batch, ldb=ldb, alpha=0.75, row_scale=d, bias=bias, act=act)
    from gpu_util import compare
    compare(out[:, :, :N], ref, f"{cfg} diag {M}x{N}x{batch}")
