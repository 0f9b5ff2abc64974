"""Each planted mistake in a copy of the oracle's source must fail a pin.

The mistakes are planted on the CPU, in copies of ``oracle/gemm_epilogue_oracle.c``
compiled to a temporary directory; the real oracle and the GPU library are not
touched.  This shows the pins of test_oracle_pins.py would notice a dropped
term, a wrong sign or index, a transposed operand or a narrowed accumulator.
"""
import inspect
import os

import pytest

import oracle as oracle_mod
import test_oracle_pins as pins

_SRC = os.path.join(os.path.dirname(oracle_mod.__file__), "gemm_epilogue_oracle.c")

MUTANTS = {
    "bias_dropped": ("double v = alpha * acc[n] + (bias ? bias[n] : 0.0);", "double v = alpha * acc[n];"),
    "bias_scaled_by_alpha": ("double v = alpha * acc[n] + (bias ? bias[n] : 0.0);",
                             "double v = alpha * (acc[n] + (bias ? bias[n] : 0.0));"),
    "bias_per_row": ("(bias ? bias[n] : 0.0)", "(bias ? bias[m % N] : 0.0)"),
    "alpha_dropped": ("double v = alpha * acc[n]", "double v = acc[n]"),
    "k_loop_short": ("for (int k = 0; k < K; ++k) {", "for (int k = 0; k < K - 1; ++k) {"),
    "k_loop_starts_at_1": ("for (int k = 0; k < K; ++k) {", "for (int k = 1; k < K; ++k) {"),
    "b_transposed": ("const T *b_row = b_mat + (size_t)k * ldb;  ", "const T *b_row = b_mat + (size_t)k;"),
    "a_wrong_ld": ("size_t a_off = (size_t)b * M * lda + (size_t)m * lda;",
                   "size_t a_off = (size_t)b * M * lda + (size_t)m * K;"),
    "batch_stride_b": ("size_t b_off = (size_t)b * K * ldb;", "size_t b_off = 0;"),
    "c_wrong_ld": ("double *c_row = C + (size_t)b * M * ldc + (size_t)m * ldc;",
                   "double *c_row = C + (size_t)b * M * ldc + (size_t)m * N;"),
    "float_accumulator": ("acc[n] += a * WIDEN(b_row[n]);", "acc[n] = (float)(acc[n] + a * WIDEN(b_row[n]));"),
    "bf16_shift": ("((uint32_t)bits) << 16", "((uint32_t)bits) << 15"),
    "relu_sign": ("return v > 0.0 ? v : 0.0;", "return v < 0.0 ? v : 0.0;"),
    "gelu_cubic_coeff": ("0.044715 * v * v * v", "0.044715 * v * v"),
    "gelu_constant": ("0.7978845608028654", "0.7978845608028654 * 1.01"),
    "gelu_erf_form": ("return 0.5 * v * (1.0 + tanh(u));", "return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));"),
    "gelu_missing_half": ("return 0.5 * v * (1.0 + tanh(u));", "return v * (1.0 + tanh(u));"),
}


def _pin_functions():
    return [f for name, f in inspect.getmembers(pins, inspect.isfunction)
            if name.startswith("test_") and name != "test_thread_count_does_not_change_bits"]


def _run_pin(f):
    params = [m.args for m in getattr(f, "pytestmark", []) if m.name == "parametrize"]
    if not params:
        f(oracle_mod)
        return
    names, values = params[0]
    names = [n.strip() for n in names.split(",")]
    for v in values:
        v = v if isinstance(v, (tuple, list)) else (v,)
        f(oracle_mod, **dict(zip(names, v)))


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(_SRC).read()
    # the macro body carries trailing spaces and a backslash; match on the code only
    old_key = old.rstrip()
    assert src.count(old_key) >= 1, f"mutation site for {name} not found"
    mutated = src.replace(old_key, new.rstrip(), 1)
    assert mutated != src
    c = tmp_path / "mutant.c"
    c.write_text(mutated)
    so = oracle_mod.compile_source(str(c), str(tmp_path / "mutant.so"))
    caught = []
    try:
        oracle_mod.use_library(so)
        for f in _pin_functions():
            try:
                _run_pin(f)
            except (AssertionError, ValueError, FloatingPointError):
                caught.append(f.__name__)
    finally:
        oracle_mod.use_library(None)
    assert caught, f"no pin noticed the planted mistake '{name}'"
