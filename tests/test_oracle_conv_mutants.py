"""Each planted mistake in a copy of the convolution oracle must fail one of its pins (CPU only)."""
import inspect
import itertools
import os

import pytest

import oracle as oracle_mod
import test_oracle_conv_pins as pins

_SRC = os.path.join(os.path.dirname(oracle_mod.__file__), "conv_oracle.c")

MUTANTS = {
    "stride_h_w_swapped": ("const int ih = oh * sh - ph + kh * dh;", "const int ih = oh * sw - ph + kh * dh;"),
    "pad_h_w_swapped": ("const int iw = ow * sw - pw + kw * dw;", "const int iw = ow * sw - ph + kw * dw;"),
    "dilation_ignored": ("const int ih = oh * sh - ph + kh * dh;", "const int ih = oh * sh - ph + kh;"),
    "dilation_w_ignored": ("const int iw = ow * sw - pw + kw * dw;", "const int iw = ow * sw - pw + kw;"),
    "pad_sign": ("const int ih = oh * sh - ph + kh * dh;", "const int ih = oh * sh + ph + kh * dh;"),
    "kernel_flipped": ("const size_t wi = (((size_t)co * KH + kh) * KW + kw) * Cin;",
                       "const size_t wi = (((size_t)co * KH + (KH - 1 - kh)) * KW + (KW - 1 - kw)) * Cin;"),
    "weight_kh_kw_swapped": ("const size_t wi = (((size_t)co * KH + kh) * KW + kw) * Cin;",
                             "const size_t wi = (((size_t)co * KW + kw) * KH + kh) * Cin;"),
    "input_h_w_swapped": ("const size_t xi = (((size_t)n * H + ih) * W + iw) * Cin;",
                          "const size_t xi = (((size_t)n * W + iw) * H + ih) * Cin;"),
    "batch_ignored": ("const size_t xi = (((size_t)n * H + ih) * W + iw) * Cin;",
                      "const size_t xi = (((size_t)0 * H + ih) * W + iw) * Cin;"),
    "upper_bound_h_off": ("if (ih < 0 || ih >= H) continue;", "if (ih < 0 || ih >= H - 1) continue;"),
    "lower_bound_w_off": ("if (iw < 0 || iw >= W) continue;", "if (iw < 1 || iw >= W) continue;"),
    "channel_loop_short": ("for (int c = 0; c < Cin; ++c)", "for (int c = 0; c < Cin - 1; ++c)"),
    "out_size_no_dilation": ("int span = in + 2 * pad - dil * (k - 1) - 1;", "int span = in + 2 * pad - (k - 1) - 1;"),
    "out_size_pad_once": ("int span = in + 2 * pad - dil * (k - 1) - 1;", "int span = in + pad - dil * (k - 1) - 1;"),
    "out_size_round_up": ("return span < 0 ? 0 : span / stride + 1;", "return span < 0 ? 0 : (span + stride - 1) / stride + 1;"),
    "bias_per_position": ("if (bias) v = v + bias[co];", "if (bias) v = v + bias[ow % Cout];"),
    "bias_dropped": ("if (bias) v = v + bias[co];", ""),
    "alpha_on_bias": ("double v = alpha * s;\n                    if (bias) v = v + bias[co];",
                      "double v = s;\n                    if (bias) v = v + bias[co];\n                    v = alpha * v;"),
    "beta_dropped": ("v = v + beta * conv_element(R, r_kind, yi);", "v = v + conv_element(R, r_kind, yi);"),
    "residual_after_act": ("double y = conv_act(v, act);",
                           "double y = conv_act(R ? v - beta * conv_element(R, r_kind, yi) : v, act); if (R) y += beta * conv_element(R, r_kind, yi);"),
    "clamp_before_act": ("double y = conv_act(v, act);", "if (v < lo) v = lo; if (v > hi) v = hi; double y = conv_act(v, act);"),
    "clamp_high_dropped": ("if (y > hi) y = hi;", ""),
    "round_truncates": ("if (lower > 0x8000u || (lower == 0x8000u && (w & 0x10000u))) w += 0x10000u;", ""),
    "f32_rounding_skipped": ("if (out_kind == CONV_F32) y = (double)(float)y;", ""),
    "relu_sign": ("return v > 0.0 ? v : 0.0;", "return v < 0.0 ? v : 0.0;"),
    "gelu_constant": ("0.7978845608028654", "0.7978845608028654 * 1.01"),
    "output_channel_stride": ("const size_t yi = (((size_t)n * OH + oh) * OW + ow) * Cout + co;",
                              "const size_t yi = (((size_t)n * OH + oh) * OW + ow) + (size_t)co * Nb * OH * OW;"),
}


def _pin_functions():
    return [f for name, f in inspect.getmembers(pins, inspect.isfunction) if name.startswith("test_")]


def _run_pin(f):
    marks = [m.args for m in getattr(f, "pytestmark", []) if m.name == "parametrize"]
    if not marks:
        f(oracle_mod)
        return
    axes = []
    for names, values in marks:
        names = [n.strip() for n in names.split(",")]
        axes.append([dict(zip(names, v if (isinstance(v, (tuple, list)) and len(names) > 1) else (v,))) for v in values])
    for combo in itertools.product(*axes):
        kw = {}
        for d in combo:
            kw.update(d)
        f(oracle_mod, **kw)


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(_SRC).read()
    assert src.count(old) >= 1, f"mutation site for {name} not found"
    mutated = src.replace(old, new, 1)
    assert mutated != src
    c = tmp_path / "mutant.c"
    c.write_text(mutated)
    so = oracle_mod.compile_source(str(c), str(tmp_path / "mutant.so"))
    caught = []
    try:
        oracle_mod.use_conv_library(so)
        for f in _pin_functions():
            try:
                _run_pin(f)
            except (AssertionError, ValueError, FloatingPointError, pytest.fail.Exception):
                caught.append(f.__name__)
    finally:
        oracle_mod.use_conv_library(None)
    assert caught, f"no pin noticed the planted mistake '{name}'"
