"""GPU parity of the four-wave 256 x 256 kernel (full or ragged tiles, K ranges of 256 or more)
against the CPU oracles, through the C-ABI: the plain operator with each activation, the widened
operator in all four operand storages with fp32 and bf16 output, residual and row scale, padded
leading dimensions, batches, K slices and a triangular A.  The 256 x 256 tile is forced, since at
sizes the oracle finishes in seconds the planner would hand these shapes to the 128 x 128 kernel;
each case is also run on the eight-wave kernel (GE_WAVES=8), which must agree within the bar too."""
import itertools

import numpy as np
import pytest

from paper_2604_01489_amd import binding

from gpu_util import run_case, run_fused_case

pytestmark = pytest.mark.gpu

LAYOUTS = list(itertools.product([False, True], repeat=2))
NAME = {(False, False): "nn", (False, True): "nt", (True, False): "tn", (True, True): "tt"}


@pytest.mark.parametrize("M,N,K", [
    (256, 256, 256),     # one tile, one pass of the four-step loop body
    (512, 768, 384),     # 2 x 3 tiles, three passes
    (256, 512, 1152),    # nine passes: every stage refilled several times
])
@pytest.mark.parametrize("act", ["none", "relu", "gelu_tanh"])
def test_plain_operator(oracle, M, N, K, act, monkeypatch):
    binding.set_option("force_config", "256x256")
    got4, _, _, cfg = run_case(oracle, "bf16", M, N, K, alpha=0.5, act=act, seed=M + N + K, plan="direct")
    assert cfg == "bf16_256x256x64_w4"
    binding.set_option("waves", "8")
    got8, _, _, cfg = run_case(oracle, "bf16", M, N, K, alpha=0.5, act=act, seed=M + N + K, plan="direct")
    assert cfg == "bf16_256x256x32_w8"
    # same products, same order of the k steps within an accumulator: the two kernels agree closely
    np.testing.assert_allclose(got4, got8, rtol=1e-4, atol=1e-5)


def test_plain_padded_batched_no_bias(oracle, monkeypatch):
    binding.set_option("force_config", "256x256")
    _, _, _, cfg = run_case(oracle, "bf16", 256, 512, 256, batch=3, lda=264, ldb=520, ldc=516, act="relu", seed=31,
                            plan="direct")
    assert cfg == "bf16_256x256x64_w4"
    _, _, _, cfg = run_case(oracle, "bf16", 512, 256, 512, with_bias=False, alpha=-1.25, seed=32, dist="normal",
                            plan="direct")
    assert cfg == "bf16_256x256x64_w4"


def test_not_taken_when_k_is_short(oracle, monkeypatch):
    """K ranges below 256 stay on the eight-wave kernel (one load phase, or a ring that barely turns)."""
    binding.set_option("force_config", "256x256")
    for M, N, K in [(256, 256, 128), (520, 264, 248), (256, 256, 64)]:
        _, _, _, cfg = run_case(oracle, "bf16", M, N, K, act="relu", seed=M + K, plan="direct")
        assert cfg == "bf16_256x256x32_w8", (M, N, K, cfg)


@pytest.mark.parametrize("K", [264, 320, 328, 392, 1000])
def test_ragged_k(oracle, K, monkeypatch):
    """K ranges that are not multiples of 128, of 64, of 32: the chunks beyond the end are masked, the loop
    runs on over zero-filled stages to the next multiple of four steps."""
    binding.set_option("force_config", "256x256")
    _, _, _, cfg = run_case(oracle, "bf16", 256, 512, K, alpha=0.5, act="gelu_tanh", seed=K, lda=K + 8, plan="direct")
    assert cfg == "bf16_256x256x64_w4"
    _, _, _, cfg = run_case(oracle, "bf16", 264, 248, K, alpha=-0.5, seed=K + 1, plan="direct")
    assert cfg == "bf16_256x256x64_w4"
    for transA, transB in LAYOUTS:
        if transA and not transB:
            continue
        _, _, _, cfg = run_fused_case(oracle, 256, 264, K, transA=transA, transB=transB, with_row_scale=True, act="relu",
                                      out="bf16", pad=(8, 0, 0, 8), plan="direct", seed=K + 2 * transA + transB)
        assert cfg == f"bf16_fused_256x256x64_w4_{NAME[transA, transB]}"


@pytest.mark.parametrize("M,N", [(520, 256), (256, 264), (328, 776), (8, 8), (249, 505)])
def test_plain_operator_ragged_tiles(oracle, M, N, monkeypatch):
    """Tiles hanging over M, N or both (rows and column chunks beyond are never fetched, never stored):
    padded leading dimensions hold garbage and a canary that must survive."""
    binding.set_option("force_config", "256x256")
    M8, N8 = (M + 7) // 8 * 8, (N + 7) // 8 * 8         # the direct-to-LDS kernels want N a multiple of 8; M is free
    for act, K in [("gelu_tanh", 256), ("relu", 640)]:
        _, _, _, cfg = run_case(oracle, "bf16", M, N8, K, alpha=0.5, act=act, seed=M + N + K, lda=K + 8, ldb=N8 + 16,
                                ldc=N8 + 4, plan="direct")
        assert cfg == "bf16_256x256x64_w4", (M, N8, K, cfg)
    _, _, _, cfg = run_case(oracle, "bf16", M, N8, 1024, alpha=0.25, seed=M + N, plan="splitk", split_k=2)
    assert cfg == "bf16_256x256x64_w4_splitk"


@pytest.mark.parametrize("transA,transB", [(False, False), (False, True), (True, True)])
@pytest.mark.parametrize("out", ["f32", "bf16"])
def test_widened_operator_ragged_tiles(oracle, transA, transB, out, monkeypatch):
    binding.set_option("force_config", "256x256")
    for M, N, K, pad in [(520, 264, 256, (8, 8, 8, 8)), (200, 776, 384, (0, 16, 0, 8)), (264, 8, 256, (0, 0, 0, 0))]:
        _, _, _, cfg = run_fused_case(oracle, M, N, K, transA=transA, transB=transB, alpha=0.5, with_row_scale=True,
                                      residual="bf16" if out == "f32" else "f32", beta=-0.5, act="relu", clamp=(0.0, 2.0),
                                      out=out, pad=pad, plan="direct", seed=M + N + K + 2 * transA + transB)
        assert cfg == f"bf16_fused_256x256x64_w4_{NAME[transA, transB]}", (M, N, K, cfg)


def test_split_k(oracle, monkeypatch):
    """Partial tiles from the four-wave kernel, reduced in slice order: matches the oracle, repeats
    bit for bit; slice lengths that are not multiples of 128 take the edge variant, short ones eight waves."""
    binding.set_option("force_config", "256x256")
    got1, _, _, cfg = run_case(oracle, "bf16", 256, 512, 2048, alpha=0.125, act="gelu_tanh", seed=41, plan="splitk", split_k=4)
    assert cfg == "bf16_256x256x64_w4_splitk"
    got2, _, _, _ = run_case(oracle, "bf16", 256, 512, 2048, alpha=0.125, act="gelu_tanh", seed=41, plan="splitk", split_k=4)
    assert np.array_equal(got1, got2)
    _, _, _, cfg = run_case(oracle, "bf16", 256, 256, 1152, alpha=0.125, seed=42, plan="splitk", split_k=4)  # slices of 288
    assert cfg == "bf16_256x256x64_w4_splitk"
    _, _, _, cfg = run_case(oracle, "bf16", 256, 256, 1096, alpha=0.125, seed=43, plan="splitk", split_k=3)  # 384, 384, 328
    assert cfg == "bf16_256x256x64_w4_splitk"
    _, _, _, cfg = run_case(oracle, "bf16", 256, 256, 800, alpha=0.125, seed=44, plan="splitk", split_k=4)   # slices of 224: too short
    assert cfg == "bf16_256x256x32_w8_splitk"


@pytest.mark.parametrize("transA,transB", LAYOUTS)
@pytest.mark.parametrize("out", ["f32", "bf16"])
def test_widened_operator_layouts(oracle, transA, transB, out, monkeypatch):
    binding.set_option("force_config", "256x256")
    name = f"bf16_fused_256x256x64_w4_{NAME[transA, transB]}"
    if transA and not transB:       # both operands in whole lines already: stays on eight waves
        name = "bf16_fused_256x256x32_w8_tn"
    for M, N, K, pad in [(256, 256, 256, (0, 0, 0, 0)), (512, 768, 384, (8, 16, 8, 8))]:
        _, _, _, cfg = run_fused_case(oracle, M, N, K, transA=transA, transB=transB, alpha=0.5, act="gelu_tanh",
                                      with_row_scale=True, out=out, pad=pad, plan="direct",
                                      seed=M + K + 2 * transA + transB)
        assert cfg == name


@pytest.mark.parametrize("residual,out", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32"), ("f32", "bf16")])
def test_widened_operator_chain(oracle, residual, out, monkeypatch):
    """Row scale, bias, residual (aligned and, with a padded ldr, unaligned rows), relu, clamp."""
    binding.set_option("force_config", "256x256")
    for pad in [(0, 0, 0, 0), (0, 8, 3 if out == "f32" else 8, 0)]:
        _, _, _, cfg = run_fused_case(oracle, 256, 512, 640, transB=True, alpha=0.25, with_row_scale=True,
                                      residual=residual, beta=-0.5, act="relu", clamp=(0.0, 1.5), out=out, pad=pad,
                                      plan="direct", seed=77)
        assert cfg == "bf16_fused_256x256x64_w4_nt"


def test_widened_operator_batched_and_split(oracle, monkeypatch):
    binding.set_option("force_config", "256x256")
    _, _, _, cfg = run_fused_case(oracle, 256, 256, 384, batch=3, transA=True, transB=True, act="relu", out="bf16",
                                  plan="direct", seed=51)
    assert cfg == "bf16_fused_256x256x64_w4_tt"
    _, _, _, cfg = run_fused_case(oracle, 256, 512, 2048, transB=True, alpha=0.125, with_row_scale=True, residual="f32",
                                  act="gelu_tanh", out="bf16", plan="splitk", split_k=4, seed=52)
    assert cfg == "bf16_fused_256x256x64_w4_nt_splitk"


@pytest.mark.parametrize("structure", ["lower", "upper"])
def test_triangular_a(oracle, structure, monkeypatch):
    """Per-tile-row K ranges (multiples of 256): the shortest is one pass of the loop body."""
    binding.set_option("force_config", "256x256")
    got_h, _, _, cfg = run_fused_case(oracle, 768, 256, 768, act="relu", a_structure=structure, hint=True, plan="direct", seed=61)
    assert cfg == "bf16_fused_256x256x64_w4_nn"
    got_g, _, _, _ = run_fused_case(oracle, 768, 256, 768, act="relu", a_structure=structure, hint=False, plan="direct", seed=61)
    assert np.array_equal(got_h, got_g)         # the skipped steps only ever added exact zeros
