"""Seeded random sweeps of argument combinations through the C-ABI against the CPU oracles: shapes around
the tile sizes (full, ragged, tiny), every operand storage, output and residual type, activations, clamps,
padded leading dimensions, misaligned pointers, batches and K slices.  The draws are fixed by the seed, so
a failure names a reproducible case (each case prints its arguments before it runs)."""
import numpy as np
import pytest

from paper_2604_01489_amd import binding

from gpu_util import run_case, run_fused_case
from test_gpu_conv import run_conv_case

pytestmark = pytest.mark.gpu

DIMS = [1, 7, 16, 33, 64, 72, 127, 128, 136, 200, 255, 256, 264, 328, 392, 512, 520]
KDIMS = [1, 8, 24, 32, 40, 64, 72, 96, 128, 136, 200, 256, 328, 512, 1032]


def _pick(rng, seq):
    return seq[int(rng.integers(len(seq)))]


@pytest.mark.parametrize("chunk", range(8))
def test_fused_operator_sweep(oracle, chunk):
    rng = np.random.default_rng(1000 + chunk)
    for i in range(12):
        M, N, K = _pick(rng, DIMS), _pick(rng, DIMS), _pick(rng, KDIMS)
        aligned = rng.random() < 0.7                      # mostly shapes the direct-to-LDS kernels take
        if aligned:
            M, N, K = max(8, M // 8 * 8), max(8, N // 8 * 8), max(8, K // 8 * 8)
        batch = int(_pick(rng, [1, 1, 1, 2, 3]))
        pad = tuple(int(8 * rng.integers(0, 3)) if aligned else int(rng.integers(0, 5)) for _ in range(4))
        clamp = _pick(rng, [None, None, (-0.25, 0.5), (0.0, 6.0), (-1.0, -0.5)])
        splitk = K >= 256 and rng.random() < 0.3
        run_fused_case(oracle, M, N, K, batch=batch, transA=bool(rng.integers(2)), transB=bool(rng.integers(2)),
                       alpha=float(_pick(rng, [1.0, 0.5, -0.75])), with_row_scale=bool(rng.integers(2)),
                       with_bias=bool(rng.integers(2)), residual=_pick(rng, [None, "f32", "bf16"]),
                       beta=float(_pick(rng, [1.0, -0.5])), act=_pick(rng, ["none", "relu", "gelu_tanh"]), clamp=clamp,
                       out=_pick(rng, ["f32", "bf16"]), pad=pad, seed=2000 + 100 * chunk + i,
                       misalign=0 if aligned else int(rng.integers(0, 4)),
                       plan="splitk" if splitk else "auto", split_k=int(_pick(rng, [0, 2, 3])) if splitk else 0)


@pytest.mark.parametrize("chunk", range(4))
def test_plain_operator_sweep(oracle, chunk):
    rng = np.random.default_rng(3000 + chunk)
    for i in range(12):
        dtype = _pick(rng, ["bf16", "bf16", "f32"])
        M, N, K = _pick(rng, DIMS), _pick(rng, DIMS), _pick(rng, KDIMS)
        if rng.random() < 0.7:
            M, N, K = max(8, M // 8 * 8), max(8, N // 8 * 8), max(8, K // 8 * 8)
        run_case(oracle, dtype, M, N, K, batch=int(_pick(rng, [1, 1, 2, 3])), alpha=float(_pick(rng, [1.0, 0.5, -2.0])),
                 act=_pick(rng, ["none", "relu", "gelu_tanh"]), seed=4000 + 100 * chunk + i)


@pytest.mark.parametrize("chunk", range(4))
def test_convolution_sweep(oracle, chunk):
    rng = np.random.default_rng(5000 + chunk)
    for i in range(8):
        KH, KW = int(_pick(rng, [1, 2, 3, 5])), int(_pick(rng, [1, 3, 4]))
        dil = (int(_pick(rng, [1, 1, 2])), int(_pick(rng, [1, 1, 2])))
        H = int(rng.integers(dil[0] * (KH - 1) + 1, 24))
        W = int(rng.integers(dil[1] * (KW - 1) + 1, 24))
        Cin = int(_pick(rng, [3, 32, 32, 64, 96, 40]))
        Cout = int(_pick(rng, [8, 24, 64, 72, 256, 264, 10]))
        run_conv_case(oracle, (int(_pick(rng, [1, 2, 5])), H, W, Cin, Cout, KH, KW),
                      stride=(int(_pick(rng, [1, 1, 2, 3])), int(_pick(rng, [1, 2]))),
                      pad=(int(rng.integers(0, 4)), int(rng.integers(0, 4))), dil=dil,
                      alpha=float(_pick(rng, [1.0, 0.5])), with_bias=bool(rng.integers(2)),
                      residual=_pick(rng, [None, "f32", "bf16"]), beta=float(_pick(rng, [1.0, -0.5])),
                      act=_pick(rng, ["none", "relu", "gelu_tanh"]), clamp=_pick(rng, [None, (0.0, 1.5), (-0.5, 0.5)]),
                      out=_pick(rng, ["f32", "bf16"]), seed=6000 + 100 * chunk + i)


@pytest.mark.parametrize("chunk", range(4))
def test_four_wave_sweep(oracle, chunk, monkeypatch):
    """256 x 256 tiles, full or ragged, over K ranges of 256 and more, the tile forced: the shapes the four-wave
    kernel takes, with every storage, consumer chain, output type, padding, batch and K slicing drawn at random."""
    binding.set_option("force_config", "256x256")
    rng = np.random.default_rng(7000 + chunk)
    seen = set()
    for i in range(8):
        M, N = 256 * int(_pick(rng, [1, 1, 2, 3])), 256 * int(_pick(rng, [1, 2, 3]))
        K = 128 * int(_pick(rng, [2, 3, 4, 5, 8, 9]))
        if rng.random() < 0.4:                            # ragged in every direction: the edge variant
            M, N, K = M - 8 * int(rng.integers(0, 20)), N - 8 * int(rng.integers(0, 20)), K + 8 * int(rng.integers(0, 16))
        splitk = K >= 1024 and rng.random() < 0.5         # 1024 or 1152 in 2 slices: 512 (four waves) or 576 (eight)
        pad = tuple(int(8 * rng.integers(0, 3)) for _ in range(4))
        _, _, _, cfg = run_fused_case(
            oracle, M, N, K, batch=int(_pick(rng, [1, 1, 2])), transA=bool(rng.integers(2)), transB=bool(rng.integers(2)),
            alpha=float(_pick(rng, [1.0, 0.5, -0.75])), with_row_scale=bool(rng.integers(2)),
            with_bias=bool(rng.integers(2)), residual=_pick(rng, [None, "f32", "bf16"]),
            beta=float(_pick(rng, [1.0, -0.5])), act=_pick(rng, ["none", "relu", "gelu_tanh"]),
            clamp=_pick(rng, [None, None, (-0.25, 0.5), (0.0, 6.0)]), out=_pick(rng, ["f32", "bf16"]), pad=pad,
            seed=8000 + 100 * chunk + i, plan="splitk" if splitk else "direct", split_k=2 if splitk else 0)
        seen.add("w4" if "_w4" in cfg else "w8")
    assert "w4" in seen, seen
