"""Each planted mistake in a copy of the widened operator's oracle must fail one of its pins.

The mistakes are planted on the CPU, in copies of ``oracle/gemm_fused_oracle.c`` compiled to a
temporary directory; the real oracle and the GPU library are not touched.
"""
import inspect
import os

import pytest

import oracle as oracle_mod
import test_oracle_fused_pins as pins

_SRC = os.path.join(os.path.dirname(oracle_mod.__file__), "gemm_fused_oracle.c")

MUTANTS = {
    "transA_ignored": ("(transA ? (size_t)k * lda + m : (size_t)m * lda + k)", "((size_t)m * lda + k)"),
    "transB_ignored": ("(transB ? (size_t)n * ldb + k : (size_t)k * ldb + n)", "((size_t)k * ldb + n)"),
    "transA_swapped": ("(transA ? (size_t)k * lda + m : (size_t)m * lda + k)",
                       "(transA ? (size_t)m * lda + k : (size_t)k * lda + m)"),
    "transB_wrong_ld": ("(transB ? (size_t)n * ldb + k :", "(transB ? (size_t)n * K + k :"),
    "batch_stride_transA": ("const size_t batchA = (size_t)(transA ? K : M) * (size_t)lda;",
                            "const size_t batchA = (size_t)M * (size_t)lda;"),
    "batch_stride_transB": ("const size_t batchB = (size_t)(transB ? N : K) * (size_t)ldb;",
                            "const size_t batchB = (size_t)K * (size_t)ldb;"),
    "row_scale_per_column": ("v = row_scale[m] * v;", "v = row_scale[n % M] * v;"),
    "row_scale_after_bias": ("if (row_scale) v = row_scale[m] * v;\n                if (bias) v = v + bias[n];",
                             "if (bias) v = v + bias[n];\n                if (row_scale) v = row_scale[m] * v;"),
    "row_scale_dropped": ("if (row_scale) v = row_scale[m] * v;", ""),
    "bias_dropped": ("if (bias) v = v + bias[n];", ""),
    "bias_per_row": ("if (bias) v = v + bias[n];", "if (bias) v = v + bias[m % N];"),
    "alpha_dropped": ("double v = alpha * p;", "double v = p;"),
    "beta_dropped": ("v = v + beta * element(R,", "v = v + element(R,"),
    "residual_scaled_by_alpha": ("v + beta * element(R,", "v + alpha * beta * element(R,"),
    "residual_after_activation": ("double y = act_apply(v, act);",
                                  "double y = act_apply(R ? v - beta * element(R, r_kind, ((size_t)b * M + m) * (size_t)ldr + n) : v, act);"
                                  " if (R) y += beta * element(R, r_kind, ((size_t)b * M + m) * (size_t)ldr + n);"),
    "residual_wrong_ld": ("((size_t)b * M + m) * (size_t)ldr + n);\n                double y",
                          "((size_t)b * M + m) * (size_t)N + n);\n                double y"),
    "residual_no_batch": ("element(R, r_kind, ((size_t)b * M + m) * (size_t)ldr + n);\n                double y",
                          "element(R, r_kind, ((size_t)m) * (size_t)ldr + n);\n                double y"),
    "clamp_before_activation": ("double y = act_apply(v, act);",
                                "if (v < lo) v = lo; if (v > hi) v = hi; double y = act_apply(v, act);"),
    "clamp_low_dropped": ("if (y < lo) y = lo;", ""),
    "clamp_high_dropped": ("if (y > hi) y = hi;", ""),
    "round_truncates": ("if (lower > 0x8000u || (lower == 0x8000u && (w & 0x10000u))) w += 0x10000u;", ""),
    "round_ties_away": ("(lower == 0x8000u && (w & 0x10000u))", "(lower == 0x8000u)"),
    "round_ties_down": ("if (lower > 0x8000u || (lower == 0x8000u && (w & 0x10000u))) w += 0x10000u;",
                        "if (lower > 0x8000u) w += 0x10000u;"),
    "round_from_double": ("y = (double)oracle_round_f32_to_bf16((float)y);",
                          "{ float f = (float)y; uint32_t q; memcpy(&q, &f, 4); q &= 0xFFFF0000u; memcpy(&f, &q, 4); y = f; }"),
    "f32_rounding_skipped": ("if (out_kind == FUSED_OUT_F32) y = (double)(float)y;", ""),
    "k_loop_short": ("for (int k = 0; k < K; ++k) {", "for (int k = 0; k < K - 1; ++k) {"),
    "relu_sign": ("return v > 0.0 ? v : 0.0;", "return v < 0.0 ? v : 0.0;"),
    "gelu_cubic_coeff": ("0.044715 * v * v * v", "0.044715 * v * v"),
    "bf16_shift": ("((uint32_t)bits) << 16", "((uint32_t)bits) << 15"),
    "lo_hi_check_dropped": ("if (!(lo <= hi)) return -1;", ""),
}


def _pin_functions():
    return [f for name, f in inspect.getmembers(pins, inspect.isfunction) if name.startswith("test_")]


def _run_pin(f):
    marks = [m.args for m in getattr(f, "pytestmark", []) if m.name == "parametrize"]
    if not marks:
        f(oracle_mod)
        return
    # stacked parametrize marks: the full product
    import itertools
    axes = []
    for names, values in marks:
        names = [n.strip() for n in names.split(",")]
        axes.append([dict(zip(names, v if isinstance(v, (tuple, list)) else (v,))) for v in values])
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
        oracle_mod.use_fused_library(so)
        for f in _pin_functions():
            try:
                f_name = f.__name__
                _run_pin(f)
            except (AssertionError, ValueError, FloatingPointError, pytest.fail.Exception):
                caught.append(f_name)         # pytest.fail.Exception: a pytest.raises that did not raise
    finally:
        oracle_mod.use_fused_library(None)
    assert caught, f"no pin noticed the planted mistake '{name}'"
