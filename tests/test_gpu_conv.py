"""GPU parity of the convolution front-end (conv2d_epilogue_bf16) against the direct-convolution
oracle: the gathering implicit-GEMM kernel on both tile shapes, full and ragged tiles, strides,
paddings, dilations, the consumer chain with fp32 and bf16 output, and the guarded kernel."""
import numpy as np
import pytest

from paper_2604_01489_amd import binding

from gpu_util import compare, to_device, torch_device

pytestmark = pytest.mark.gpu


def run_conv_case(oracle, shape, *, stride=(1, 1), pad=(0, 0), dil=(1, 1), alpha=1.0, with_bias=True,
                  residual=None, beta=1.0, act="none", clamp=None, out="f32", seed=0, expect=None):
    import torch
    from paper_2604_01489_amd import inputs as gen
    Nb, H, W, Cin, Cout, KH, KW = shape
    OH = oracle.conv_out_size(H, KH, stride[0], pad[0], dil[0])
    OW = oracle.conv_out_size(W, KW, stride[1], pad[1], dil[1])
    X = gen.to_bf16_bits(gen.normal(seed, gen.STREAM_A, Nb * H * W * Cin, 1.0).reshape(Nb, H, W, Cin))
    Wt = gen.to_bf16_bits(gen.normal(seed, gen.STREAM_B, Cout * KH * KW * Cin, (KH * KW * Cin) ** -0.5)
                          .reshape(Cout, KH, KW, Cin))
    bias = gen.uniform(seed, gen.STREAM_BIAS, Cout, -1.0, 1.0) if with_bias else None
    R = None
    if residual is not None:
        R = gen.uniform(seed, gen.STREAM_RESIDUAL, Nb * OH * OW * Cout, -1.0, 1.0).reshape(Nb, OH, OW, Cout)
        if residual == "bf16":
            R = gen.to_bf16_bits(R)
    dX, dW, dbias, dR = to_device(X), to_device(Wt), to_device(bias), to_device(R)
    if dR is not None and residual == "bf16":
        dR = dR.view(torch.bfloat16)
    ydtype = torch.float32 if out == "f32" else torch.bfloat16
    Y = torch.full((Nb, OH, OW, Cout), -7.0e30, dtype=ydtype, device=torch_device())
    print(f"conv case {shape} stride={stride} pad={pad} dil={dil} act={act} out={out} res={residual} clamp={clamp}",
          flush=True)
    binding.conv2d_epilogue_bf16(dX, dW, Y, stride=stride, pad=pad, dil=dil, alpha=alpha, bias=dbias, residual=dR,
                                 beta=beta, act=act, clamp=clamp)
    torch.cuda.synchronize()
    cfg = binding.last_config()
    if expect is not None:
        assert cfg == expect, cfg
    got = Y.to(torch.float32).cpu().numpy()
    ref = oracle.conv2d_nhwc(X, Wt, stride=stride, pad=pad, dil=dil, alpha=alpha, bias=bias, residual=R, beta=beta,
                             act=act, clamp=clamp, out=out)
    compare(got.reshape(1, -1, Cout), ref.reshape(1, -1, Cout), f"{cfg} conv {shape}", bf16_out=(out == "bf16"))
    return cfg


def test_conv_3x3_tiles_128(oracle):
    run_conv_case(oracle, (2, 20, 20, 64, 64, 3, 3), pad=(1, 1), act="relu", seed=1, expect="conv_bf16_128x128x32_w4")
    run_conv_case(oracle, (1, 16, 16, 32, 128, 3, 3), pad=(1, 1), seed=2, expect="conv_bf16_128x128x32_w4")   # 256 x 128: full tiles


def test_conv_3x3_tiles_256(oracle, monkeypatch):
    """The 256 x 256 gathering kernel on shapes the oracle finishes quickly (forced: the planning rule gives so
    few tiles to the 128 x 128 kernel)."""
    binding.set_option("force_config", "256x256")
    run_conv_case(oracle, (4, 16, 16, 32, 256, 3, 3), pad=(1, 1), act="gelu_tanh", alpha=0.5, seed=3,
                  expect="conv_bf16_256x256x32_w8")                                                      # 1024 x 256: full tiles
    run_conv_case(oracle, (1, 18, 19, 64, 264, 3, 3), pad=(1, 1), act="relu", seed=4, expect="conv_bf16_256x256x32_w8")
    run_conv_case(oracle, (2, 16, 16, 256, 256, 3, 3), pad=(1, 1), act="relu", residual="bf16", out="bf16", seed=5,
                  expect="conv_bf16_256x256x32_w8_splitk")                                # 512 x 256: two full tiles, K = 2304


@pytest.mark.parametrize("stride,pad,dil,k", [
    ((2, 2), (1, 1), (1, 1), (3, 3)),
    ((2, 1), (0, 2), (1, 1), (3, 5)),
    ((1, 2), (2, 0), (2, 1), (3, 2)),
    ((3, 2), (0, 3), (1, 2), (1, 4)),
    ((1, 1), (0, 0), (1, 1), (1, 1)),
    ((1, 1), (3, 3), (2, 2), (3, 3)),
])
def test_conv_geometry(oracle, stride, pad, dil, k):
    run_conv_case(oracle, (2, 17, 23, 32, 72, k[0], k[1]), stride=stride, pad=pad, dil=dil, act="relu",
                  seed=10 + k[0] + 3 * k[1], expect="conv_bf16_128x128x32_w4")
    cfg = run_conv_case(oracle, (1, 17, 23, 128, 40, k[0], k[1]), stride=stride, pad=pad, dil=dil, out="bf16",
                        seed=12 + k[0] + 3 * k[1])
    assert cfg in ("conv_bf16_128x128x32_w4", "conv_bf16_128x128x32_w4_splitk")     # K slices where K is long


@pytest.mark.parametrize("out", ["f32", "bf16"])
@pytest.mark.parametrize("residual", [None, "f32", "bf16"])
def test_conv_chain(oracle, out, residual):
    for shape in [(2, 14, 14, 64, 256, 3, 3), (1, 15, 13, 32, 64, 3, 3)]:
        run_conv_case(oracle, shape, pad=(1, 1), alpha=0.75, residual=residual, beta=0.5, act="relu",
                      clamp=(0.0, 1.5), out=out, seed=20)


def test_conv_guarded_kernel(oracle):
    run_conv_case(oracle, (2, 21, 19, 3, 10, 7, 7), stride=(2, 2), pad=(3, 3), act="relu", seed=30,
                  expect="conv_bf16_generic_64x64x32")                                    # Cin = 3 with 10 output channels
    run_conv_case(oracle, (1, 9, 9, 40, 24, 3, 3), pad=(1, 1), residual="f32", out="bf16", seed=31,
                  expect="conv_bf16_generic_64x64x32")                                    # Cin not a multiple of 32
    run_conv_case(oracle, (1, 8, 8, 32, 12, 1, 1), seed=32, expect="conv_bf16_generic_64x64x32")   # Cout not a multiple of 8


HALO_56 = "conv_bf16_halo_3x3_w4_14_11"
HALO_ANY = "conv_bf16_halo_3x3_w4_12_12"


def test_conv_halo_56_wide(oracle):
    """3 x 3, stride 1 on 56-wide images: tiles of 4 and of 3 output rows in one launch (8 + 8 per image), the
    channel slabs walked in pairs, bf16 and fp32 output, one and two tile columns of 256 channels.  (With so few
    images the plan would take the variant for shorter tiles, whose tiles all run at once: this one is asked for.)"""
    binding.set_option("conv_halo", "14_11")
    try:
        _halo_56_wide_cases(oracle)
    finally:
        binding.set_option("conv_halo", None)


def _halo_56_wide_cases(oracle):
    run_conv_case(oracle, (1, 56, 56, 64, 256, 3, 3), pad=(1, 1), act="relu", residual="bf16", out="bf16", seed=90, expect=HALO_56)
    run_conv_case(oracle, (2, 56, 56, 128, 256, 3, 3), pad=(1, 1), act="gelu_tanh", alpha=0.5, seed=91, expect=HALO_56)
    run_conv_case(oracle, (1, 56, 56, 64, 512, 3, 3), pad=(1, 1), residual="f32", beta=0.5, clamp=(-0.5, 0.5), out="bf16", seed=92,
                  expect=HALO_56)


@pytest.mark.parametrize("shape,pad,expect", [
    ((3, 12, 12, 64, 256, 3, 3), (1, 1), HALO_ANY),        # 5 + 5 + 2 rows of 12: ragged last row block
    ((2, 9, 62, 64, 256, 3, 3), (1, 1), HALO_ANY),         # the widest row: 62 + 2 halo columns = a staged row
    ((2, 20, 30, 128, 512, 3, 3), (0, 0), HALO_ANY),       # no padding: 18 x 28 outputs, four slabs, two tile columns
    ((2, 10, 17, 64, 256, 3, 3), (2, 2), HALO_ANY),        # padding 2: two halo rows above the image
    ((1, 7, 52, 192, 256, 3, 3), (1, 0), HALO_56),         # 50 outputs per row, 4 + 3 rows; six slabs
    ((3, 12, 12, 64, 256, 3, 3), (1, 1), HALO_56),         # short rows on the 14- and 11-block loops
    ((5, 1, 1, 64, 256, 3, 3), (1, 1), HALO_ANY),          # one position per image
])
def test_conv_halo_geometry(oracle, shape, pad, expect):
    binding.set_option("conv_halo", "14_11" if expect == HALO_56 else "12_12")
    try:
        run_conv_case(oracle, shape, pad=pad, act="relu", seed=sum(shape), expect=expect)
        run_conv_case(oracle, shape, pad=pad, with_bias=False, residual="bf16", out="bf16", seed=1 + sum(shape), expect=expect)
    finally:
        binding.set_option("conv_halo", None)


def test_conv_halo_taken_by_default_and_switched_off(oracle):
    """Tiles for half of the CUs, nearly all of their positions in use: the halo-staged kernel without being asked;
    "off" keeps the gathering one.  Short rows (a third of the loop's positions in use), few tiles: not taken."""
    assert "halo" not in run_conv_case(oracle, (32, 20, 12, 64, 256, 3, 3), pad=(1, 1), seed=94)
    assert "halo" not in run_conv_case(oracle, (8, 6, 62, 64, 256, 3, 3), pad=(1, 1), seed=94)
    shape = (64, 6, 62, 64, 256, 3, 3)                       # 64 images x 2 tiles of 3 rows of 62
    run_conv_case(oracle, shape, pad=(1, 1), act="relu", out="bf16", seed=95, expect=HALO_ANY)
    binding.set_option("conv_halo", "off")
    try:
        assert "halo" not in run_conv_case(oracle, shape, pad=(1, 1), act="relu", out="bf16", seed=95)
    finally:
        binding.set_option("conv_halo", None)
    # shapes it does not take: stride 2, 5 x 5, Cin not a multiple of 64, Cout not a multiple of 256, rows too wide
    binding.set_option("conv_halo", "on")
    try:
        for shape, kw in [((1, 16, 16, 64, 256, 3, 3), dict(stride=(2, 2), pad=(1, 1))), ((1, 16, 16, 64, 256, 5, 5), dict(pad=(2, 2))),
                          ((1, 16, 16, 96, 256, 3, 3), dict(pad=(1, 1))), ((1, 16, 16, 64, 128, 3, 3), dict(pad=(1, 1))),
                          ((1, 4, 70, 64, 256, 3, 3), dict(pad=(1, 1))), ((1, 16, 16, 64, 256, 3, 3), dict(pad=(1, 1), dil=(2, 2)))]:
            cfg = run_conv_case(oracle, shape, seed=96, **kw)
            assert "halo" not in cfg, cfg
    finally:
        binding.set_option("conv_halo", None)


def test_conv_halo_is_repeatable():
    import torch
    binding.set_option("conv_halo", "14_11")
    from paper_2604_01489_amd import inputs as gen
    X = torch.from_numpy(gen.to_bf16_bits(gen.normal(97, 0, 2 * 56 * 56 * 64, 1.0).reshape(2, 56, 56, 64)).view(np.int16)).cuda()
    Wt = torch.from_numpy(gen.to_bf16_bits(gen.normal(97, 1, 256 * 9 * 64, 0.05).reshape(256, 3, 3, 64)).view(np.int16)).cuda()
    outs = []
    for _ in range(3):
        Y = torch.empty(2, 56, 56, 256, dtype=torch.bfloat16, device="cuda:0")
        binding.conv2d_epilogue_bf16(X, Wt, Y, pad=(1, 1), act="relu")
        torch.cuda.synchronize()
        assert binding.last_config() == HALO_56
        outs.append(Y.view(torch.int16).cpu().numpy().tobytes())
    binding.set_option("conv_halo", None)
    assert outs[0] == outs[1] == outs[2]


ROWS = "conv_bf16_rows_k32"


def test_conv_few_channels_first_layer(oracle):
    """Few input channels: the kernel whose K step is one filter row.  The first layer's geometry (7 x 7, stride 2,
    padding 3, 3 -> 64) on images whose rows are even and odd in length (staged dword by dword, or element by
    element), several tiles of 16 output columns and a ragged last one, rows above and below the image."""
    run_conv_case(oracle, (2, 40, 40, 3, 64, 7, 7), stride=(2, 2), pad=(3, 3), act="relu", out="bf16", seed=50, expect=ROWS)
    run_conv_case(oracle, (3, 23, 37, 3, 64, 7, 7), stride=(2, 2), pad=(3, 3), act="relu", seed=51, expect=ROWS)
    run_conv_case(oracle, (1, 70, 150, 3, 64, 7, 7), stride=(2, 2), pad=(3, 3), act="gelu_tanh", alpha=0.5, out="bf16", seed=52,
                  expect=ROWS)                                  # 75 output columns: five tiles, the last with 11


@pytest.mark.parametrize("shape,stride,pad,dil", [
    ((2, 12, 33, 1, 32, 7, 7), (2, 2), (3, 3), (1, 1)),       # one channel, 32 output channels
    ((2, 14, 19, 4, 64, 5, 7), (2, 3), (2, 2), (2, 1)),       # four channels, stride 3 along the row, dilated filter rows
    ((1, 9, 50, 2, 32, 1, 16), (1, 1), (0, 0), (1, 1)),       # a filter row of exactly 32 elements, no padding
    ((2, 10, 21, 3, 64, 3, 3), (1, 1), (1, 1), (1, 1)),       # 3 x 3, stride 1: windows begin at odd and even elements
    ((1, 6, 16, 3, 64, 2, 2), (1, 2), (0, 1), (1, 1)),        # even filter
    ((5, 3, 5, 3, 32, 7, 7), (2, 2), (3, 3), (1, 1)),         # an image smaller than the filter
])
def test_conv_few_channels_geometry(oracle, shape, stride, pad, dil):
    run_conv_case(oracle, shape, stride=stride, pad=pad, dil=dil, act="relu", seed=sum(shape), expect=ROWS)


@pytest.mark.parametrize("out", ["f32", "bf16"])
@pytest.mark.parametrize("residual", [None, "f32", "bf16"])
def test_conv_few_channels_chain(oracle, out, residual):
    for cout in (32, 64):
        run_conv_case(oracle, (2, 18, 26, 3, cout, 7, 7), stride=(2, 2), pad=(3, 3), alpha=0.75, residual=residual, beta=0.5,
                      act="relu", clamp=(0.0, 1.5), out=out, seed=60 + cout, expect=ROWS)
    run_conv_case(oracle, (1, 18, 26, 3, 64, 7, 7), stride=(2, 2), pad=(3, 3), with_bias=False, residual=residual, out=out,
                  seed=61, expect=ROWS)


def test_conv_few_channels_random_sweep(oracle):
    """Seeded random geometries and consumer chains on the row kernel: 1 to 4 input channels, filter rows of up to 32
    elements and up to 7 of them, strides 1 to 3, paddings 0 to 3, dilated filter rows, even and odd image rows
    (staged straight into LDS or through registers), both channel counts of the output."""
    rng = np.random.default_rng(2024)
    done = 0
    while done < 24:
        cin = int(rng.integers(1, 5))
        kw = int(rng.integers(1, 32 // cin + 1))
        kh = int(rng.integers(1, 8))
        sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        ph, pw = int(rng.integers(0, 4)), int(rng.integers(0, 4))
        dh = int(rng.integers(1, 3))
        H = int(rng.integers(dh * (kh - 1) + 1, dh * (kh - 1) + 14))
        W = int(rng.integers(kw, kw + 40))
        nb = int(rng.integers(1, 4))
        cout = int(rng.choice([32, 64]))
        out = str(rng.choice(["f32", "bf16"]))
        residual = [None, "f32", "bf16"][int(rng.integers(0, 3))]
        act = str(rng.choice(["none", "relu", "gelu_tanh"]))
        clamp = None if rng.integers(0, 2) else (-0.5, 0.75)
        if nb * H * W * cout * kh * kw * cin > 3.0e8:       # keep the oracle quick
            continue
        run_conv_case(oracle, (nb, H, W, cin, cout, kh, kw), stride=(sh, sw), pad=(ph, pw), dil=(dh, 1), alpha=0.5 + 0.25 * done % 1.0,
                      with_bias=bool(rng.integers(0, 2)), residual=residual, beta=-0.5, act=act, clamp=clamp, out=out,
                      seed=100 + done, expect=ROWS)
        done += 1


def test_conv_few_channels_falls_back(oracle):
    """Shapes the row kernel does not take go to the guarded kernel: other channel counts of the output, a filter
    row longer than 32 elements, a dilated filter row, more than 7 filter rows."""
    g = "conv_bf16_generic_64x64x32"
    run_conv_case(oracle, (1, 12, 12, 3, 48, 3, 3), pad=(1, 1), seed=70, expect=g)
    run_conv_case(oracle, (1, 12, 20, 3, 64, 3, 11), pad=(1, 5), seed=71, expect=g)
    run_conv_case(oracle, (1, 12, 20, 3, 64, 3, 3), pad=(1, 2), dil=(1, 2), seed=72, expect=g)
    run_conv_case(oracle, (1, 20, 12, 3, 64, 9, 3), pad=(4, 1), seed=73, expect=g)


def test_conv_few_channels_is_repeatable(oracle):
    import torch
    from paper_2604_01489_amd import inputs as gen
    X = torch.from_numpy(gen.to_bf16_bits(gen.normal(80, 0, 4 * 64 * 64 * 3, 1.0).reshape(4, 64, 64, 3)).view(np.int16)).cuda()
    Wt = torch.from_numpy(gen.to_bf16_bits(gen.normal(80, 1, 64 * 49 * 3, 0.1).reshape(64, 7, 7, 3)).view(np.int16)).cuda()
    outs = []
    for _ in range(3):
        Y = torch.empty(4, 32, 32, 64, dtype=torch.bfloat16, device="cuda:0")
        binding.conv2d_epilogue_bf16(X, Wt, Y, stride=(2, 2), pad=(3, 3), act="relu")
        torch.cuda.synchronize()
        assert binding.last_config() == ROWS
        outs.append(Y.view(torch.int16).cpu().numpy().tobytes())
    assert outs[0] == outs[1] == outs[2]


def test_conv_split_k_for_few_tiles_and_long_k(oracle, monkeypatch):
    """Late-layer shapes: a handful of output tiles and K = KH*KW*Cin in the thousands -> K slices,
    summed in slice order by the second pass, which also runs the consumer chain."""
    cfg = run_conv_case(oracle, (1, 8, 8, 512, 256, 3, 3), pad=(1, 1), act="relu", residual="bf16", out="bf16", seed=40)
    assert cfg == "conv_bf16_128x128x32_w4_splitk"
    cfg = run_conv_case(oracle, (4, 9, 9, 256, 512, 3, 3), pad=(1, 1), act="gelu_tanh", alpha=0.5, seed=41)
    assert cfg == "conv_bf16_128x128x32_w4_splitk"
    cfg = run_conv_case(oracle, (1, 7, 7, 200, 100, 3, 3), pad=(1, 1), stride=(2, 2), act="relu", clamp=(0.0, 1.0), seed=42)
    assert cfg == "conv_bf16_generic_64x64x32_splitk"
    binding.set_option("force_config", "256x256")            # the 256 x 256 kernel's partial tiles
    cfg = run_conv_case(oracle, (4, 9, 9, 256, 512, 3, 3), pad=(1, 1), act="gelu_tanh", alpha=0.5, seed=41)
    assert cfg == "conv_bf16_256x256x32_w8_splitk"
    binding.set_option("force_config", None)
    # repeatable bit for bit
    import torch
    from paper_2604_01489_amd import inputs as gen
    X = torch.from_numpy(gen.to_bf16_bits(gen.normal(43, 0, 8 * 8 * 512, 1.0).reshape(1, 8, 8, 512)).view(np.int16)).cuda()
    Wt = torch.from_numpy(gen.to_bf16_bits(gen.normal(43, 1, 256 * 9 * 512, 0.02).reshape(256, 3, 3, 512)).view(np.int16)).cuda()
    Y1 = torch.empty(1, 8, 8, 256, device="cuda")
    Y2 = torch.empty_like(Y1)
    binding.conv2d_epilogue_bf16(X, Wt, Y1, pad=(1, 1))
    binding.conv2d_epilogue_bf16(X, Wt, Y2, pad=(1, 1))
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)
