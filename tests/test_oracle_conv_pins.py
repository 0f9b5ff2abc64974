"""Pins for the convolution oracle (oracle/conv_oracle.c): every check compares it with something
other than itself -- a library convolution in fp64, exact rational brute force, the pinned GEMM
oracle on the 1x1 case, a one-hot kernel, zero padding, the output-size formula.  Shapes are
asymmetric in every pair of dimensions that could be confused (H/W, KH/KW, strides, paddings)."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2604_01489_amd import inputs as gen


def _rng(seed):
    return np.random.default_rng(seed)


def _torch_conv(X, Wt, stride, pad, dil):
    import torch
    import torch.nn.functional as F
    x = torch.from_numpy(X).permute(0, 3, 1, 2)          # NHWC -> NCHW
    w = torch.from_numpy(Wt).permute(0, 3, 1, 2)         # [Cout,KH,KW,Cin] -> [Cout,Cin,KH,KW]
    y = F.conv2d(x, w, None, stride, pad, dil)
    return y.permute(0, 2, 3, 1).contiguous().numpy()


@pytest.mark.parametrize("stride,pad,dil,k", [
    ((1, 1), (0, 0), (1, 1), (3, 3)),
    ((1, 1), (1, 1), (1, 1), (3, 3)),
    ((2, 1), (1, 2), (1, 1), (3, 5)),
    ((1, 2), (2, 0), (2, 1), (3, 2)),
    ((3, 2), (0, 3), (1, 2), (1, 4)),
    ((1, 1), (0, 0), (1, 1), (1, 1)),
])
def test_against_library_convolution(oracle, stride, pad, dil, k):
    r = _rng(60 + k[0] * 7 + k[1])
    X = r.normal(size=(2, 9, 11, 5))
    Wt = r.normal(size=(4, k[0], k[1], 5))
    got = oracle.conv2d_nhwc(X, Wt, stride=stride, pad=pad, dil=dil)
    want = _torch_conv(X, Wt, stride, pad, dil)
    assert got.shape == want.shape
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_brute_force_exact_rationals_with_chain(oracle):
    r = _rng(61)
    Nb, H, W, Cin, Cout, KH, KW = 1, 4, 5, 2, 3, 2, 3
    sh, sw, ph, pw, dh, dw = 2, 1, 1, 2, 1, 2
    X = r.uniform(-1, 1, (Nb, H, W, Cin)).astype(np.float32)
    Wt = r.uniform(-1, 1, (Cout, KH, KW, Cin)).astype(np.float32)
    bias = r.uniform(-1, 1, Cout).astype(np.float32)
    OH, OW = oracle.conv_out_size(H, KH, sh, ph, dh), oracle.conv_out_size(W, KW, sw, pw, dw)
    R = r.uniform(-1, 1, (Nb, OH, OW, Cout)).astype(np.float32)
    alpha, beta, lo, hi = 0.75, -0.5, 0.05, 0.6
    got = oracle.conv2d_nhwc(X, Wt, stride=(sh, sw), pad=(ph, pw), dil=(dh, dw), alpha=alpha, bias=bias,
                             residual=R, beta=beta, act="relu", clamp=(lo, hi))
    F = lambda x: Fraction(float(x))
    for co in range(Cout):
        for ow in range(OW):
            for oh in range(OH):
                s = Fraction(0)
                for c in range(Cin):
                    for kw in range(KW):
                        for kh in range(KH):
                            ih, iw = oh * sh - ph + kh * dh, ow * sw - pw + kw * dw
                            if 0 <= ih < H and 0 <= iw < W:
                                s += F(X[0, ih, iw, c]) * F(Wt[co, kh, kw, c])
                v = F(alpha) * s + F(bias[co]) + F(beta) * F(R[0, oh, ow, co])
                y = min(max(max(v, Fraction(0)), F(lo)), F(hi))
                assert abs(got[0, oh, ow, co] - float(y)) <= 4 * np.spacing(max(abs(float(y)), 1e-3)), (oh, ow, co)
    assert (got == lo).any() and (got == hi).any() and ((got > lo) & (got < hi)).any()


@pytest.mark.parametrize("dtype", ["f64", "bf16"])
def test_one_by_one_is_the_pinned_gemm(oracle, dtype):
    """1x1, stride 1: Y[pos, co] = sum_c X[pos, c] Wt[co, c] -- the plain oracle with B = Wt^T."""
    r = _rng(62)
    Nb, H, W, Cin, Cout = 2, 3, 5, 7, 4
    X = r.normal(size=(Nb, H, W, Cin))
    Wt = r.normal(size=(Cout, 1, 1, Cin))
    bias = r.normal(size=Cout)
    if dtype == "bf16":
        X, Wt = gen.to_bf16_bits(X.astype(np.float32)), gen.to_bf16_bits(Wt.astype(np.float32))
    got = oracle.conv2d_nhwc(X, Wt, alpha=1.5, bias=bias, act="gelu_tanh")
    A = X.reshape(Nb * H * W, Cin)
    B = np.ascontiguousarray(Wt.reshape(Cout, Cin).T)
    want = oracle.gemm_epilogue(A, B, bias, 1.5, "gelu_tanh").reshape(Nb, H, W, Cout)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)


def test_one_hot_kernel_shifts_the_input(oracle):
    """A kernel that is 1 at tap (kh0, kw0), channel c0 -> output channel 0 copies the shifted input
    plane, zero where the tap falls into the padding."""
    r = _rng(63)
    H, W, Cin, KH, KW, ph, pw = 6, 7, 3, 3, 4, 1, 2
    X = r.normal(size=(1, H, W, Cin))
    kh0, kw0, c0 = 2, 1, 1
    Wt = np.zeros((2, KH, KW, Cin))
    Wt[0, kh0, kw0, c0] = 1.0
    got = oracle.conv2d_nhwc(X, Wt, pad=(ph, pw))
    OH, OW = H + 2 * ph - KH + 1, W + 2 * pw - KW + 1
    assert got.shape == (1, OH, OW, 2)
    want = np.zeros((OH, OW))
    for oh in range(OH):
        for ow in range(OW):
            ih, iw = oh - ph + kh0, ow - pw + kw0
            if 0 <= ih < H and 0 <= iw < W:
                want[oh, ow] = X[0, ih, iw, c0]
    assert np.array_equal(got[0, :, :, 0], want)
    assert np.all(got[0, :, :, 1] == 0.0)
    assert (want == 0.0).any()              # some taps did fall into the padding


def test_output_size_formula(oracle):
    for size, k, s, p, d in [(7, 3, 1, 0, 1), (7, 3, 2, 1, 1), (8, 3, 2, 1, 1), (10, 3, 1, 2, 2), (5, 5, 3, 0, 1), (4, 3, 1, 0, 2)]:
        want = len([o for o in range(100) if o * s - p + d * (k - 1) <= size - 1 + p])
        assert oracle.conv_out_size(size, k, s, p, d) == want, (size, k, s, p, d)
    with pytest.raises(ValueError):
        oracle.conv2d_nhwc(np.zeros((1, 2, 2, 1)), np.zeros((1, 3, 3, 1)))        # kernel larger than the input


def test_rounded_outputs_and_bias_axis(oracle):
    import torch
    r = _rng(64)
    X = r.normal(size=(1, 5, 6, 4))
    Wt = r.normal(size=(3, 2, 2, 4))
    bias = np.array([10.0, 20.0, 30.0])
    base = oracle.conv2d_nhwc(X, Wt)
    withb = oracle.conv2d_nhwc(X, Wt, bias=bias)
    assert np.allclose(withb - base, bias[None, None, None, :], rtol=1e-12)      # per output channel
    full = oracle.conv2d_nhwc(X, Wt, bias=bias, act="gelu_tanh")
    b16 = oracle.conv2d_nhwc(X, Wt, bias=bias, act="gelu_tanh", out="bf16")
    want = torch.from_numpy(full.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(b16, want)
    f32 = oracle.conv2d_nhwc(X, Wt, bias=bias, act="gelu_tanh", out="f32")
    assert np.array_equal(f32, full.astype(np.float32).astype(np.float64))


def test_clamp_follows_activation(oracle):
    r = _rng(65)
    X = r.normal(size=(1, 5, 6, 4))
    Wt = r.normal(size=(3, 2, 2, 4))
    pre = oracle.conv2d_nhwc(X, Wt, act="gelu_tanh")
    got = oracle.conv2d_nhwc(X, Wt, act="gelu_tanh", clamp=(-0.1, 1.5))
    assert np.array_equal(got, np.clip(pre, -0.1, 1.5))
    assert (got == -0.1).any() and (got == 1.5).any()
    lin = np.clip(oracle.conv2d_nhwc(X, Wt), -0.1, 1.5)
    wrong = 0.5 * lin * (1 + np.tanh(0.7978845608028654 * (lin + 0.044715 * lin ** 3)))
    assert not np.allclose(got, wrong)
    with pytest.raises(ValueError):
        oracle.conv2d_nhwc(X, Wt, clamp=(1.0, -1.0))
