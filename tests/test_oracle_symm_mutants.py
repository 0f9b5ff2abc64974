"""Each planted mistake in a copy of the symmetric-operand oracle must fail one of its pins.

The mistakes are planted on the CPU, in copies of ``oracle/gemm_symm_oracle.c`` compiled to a
temporary directory; the real oracle and the GPU library are not touched."""
import inspect
import itertools
import os

import pytest

import oracle as oracle_mod
import test_oracle_symm_pins as pins

_SRC = os.path.join(os.path.dirname(oracle_mod.__file__), "gemm_symm_oracle.c")

MUTANTS = {
    "no_mirror": ("const size_t row = stored ? (size_t)m : (size_t)k, col = stored ? (size_t)k : (size_t)m;",
                  "const size_t row = (size_t)m, col = (size_t)k;"),
    "always_mirrored": ("const size_t row = stored ? (size_t)m : (size_t)k, col = stored ? (size_t)k : (size_t)m;",
                        "const size_t row = (size_t)k, col = (size_t)m;"),
    "wrong_triangle": ("uplo == SYMM_LOWER ? (k <= m) : (k >= m)", "uplo == SYMM_LOWER ? (k >= m) : (k <= m)"),
    "uplo_ignored": ("uplo == SYMM_LOWER ? (k <= m) : (k >= m)", "(k <= m)"),
    "mirror_reads_a_neighbour": ("col = stored ? (size_t)k : (size_t)m;", "col = stored ? (size_t)k : (size_t)m + (m + 1 < M && !stored ? 1 : 0);"),
    "unread_triangle_zero": ("p += value_at(A, in_kind, b * batchA + row * lda + col) *", "p += (stored ? value_at(A, in_kind, b * batchA + row * lda + col) : 0.0) *"),
    "diagonal_twice": ("p += value_at(A, in_kind, b * batchA + row * lda + col) *", "p += (k == m ? 2.0 : 1.0) * value_at(A, in_kind, b * batchA + row * lda + col) *"),
    "wrong_lda": ("b * batchA + row * lda + col)", "b * batchA + row * M + col)"),
    "batch_stride_A": ("const size_t batchA = (size_t)M * (size_t)lda;", "const size_t batchA = (size_t)M * (size_t)M;"),
    "batch_ignored_A": ("value_at(A, in_kind, b * batchA + row", "value_at(A, in_kind, row"),
    "transB_ignored": ("(transB ? (size_t)n * ldb + k : (size_t)k * ldb + n)", "((size_t)k * ldb + n)"),
    "k_loop_short": ("for (int k = 0; k < M; ++k) {", "for (int k = 0; k < M - 1; ++k) {"),
    "alpha_dropped": ("double v = alpha * p;", "double v = p;"),
    "bias_per_row": ("if (bias) v = v + bias[n];", "if (bias) v = v + bias[m % N];"),
    "row_scale_after_bias": ("if (row_scale) v = row_scale[m] * v;\n                if (bias) v = v + bias[n];",
                             "if (bias) v = v + bias[n];\n                if (row_scale) v = row_scale[m] * v;"),
    "beta_dropped": ("v = v + beta * value_at(R,", "v = v + value_at(R,"),
    "clamp_before_activation": ("double y = v;", "if (v < lo) v = lo; if (v > hi) v = hi; double y = v;"),
    "relu_sign": ("y = v > 0.0 ? v : 0.0;", "y = v < 0.0 ? v : 0.0;"),
    "gelu_cubic_coeff": ("0.044715 * v * v * v", "0.044715 * v * v"),
    "round_truncates": ("if (lower > 0x8000u || (lower == 0x8000u && (w & 0x10000u))) w += 0x10000u;", ""),
    "bf16_shift": ("((const uint16_t *)base)[index]) << 16", "((const uint16_t *)base)[index]) << 15"),
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
        oracle_mod.use_symm_library(so)
        for f in _pin_functions():
            try:
                f_name = f.__name__
                _run_pin(f)
            except (AssertionError, ValueError, FloatingPointError, pytest.fail.Exception):
                caught.append(f_name)
    finally:
        oracle_mod.use_symm_library(None)
    assert caught, f"no pin noticed the planted mistake '{name}'"
