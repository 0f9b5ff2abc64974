"""Planted mistakes in copies of oracle.gemm_rowsum: every one must be caught by the pins."""
import numpy as np
import pytest

import oracle
import test_oracle_rowsum_pins as pins


MUTANTS = {
    "sum_over_rows": lambda A, B, bias=None, alpha=1.0: np.sum(np.atleast_2d(oracle.gemm_epilogue(A, B, bias, alpha, "none")), axis=0),
    "bias_forgotten": lambda A, B, bias=None, alpha=1.0: np.sum(oracle.gemm_epilogue(A, B, None, alpha, "none"), axis=1),
    "bias_once_per_row": lambda A, B, bias=None, alpha=1.0: np.sum(oracle.gemm_epilogue(A, B, None, alpha, "none"), axis=1)
    + (0.0 if bias is None else float(np.asarray(bias, dtype=np.float64)[0])),
    "bias_scaled_by_alpha": lambda A, B, bias=None, alpha=1.0: alpha * np.sum(
        oracle.gemm_epilogue(A, B, bias, 1.0, "none"), axis=1),
    "alpha_forgotten": lambda A, B, bias=None, alpha=1.0: np.sum(oracle.gemm_epilogue(A, B, bias, 1.0, "none"), axis=1),
    "mean_instead_of_sum": lambda A, B, bias=None, alpha=1.0: np.mean(oracle.gemm_epilogue(A, B, bias, alpha, "none"), axis=1),
    "relu_sneaked_in": lambda A, B, bias=None, alpha=1.0: np.sum(oracle.gemm_epilogue(A, B, bias, alpha, "relu"), axis=1),
}

PINS = [pins.test_exact_rational_brute_force, pins.test_closed_form_ones, pins.test_bias_enters_once_per_column_unscaled,
        pins.test_alpha_scales_the_product_only, pins.test_collapsed_form_in_a_library_routine,
        pins.test_rows_are_independent_and_ordered]


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, monkeypatch):
    oracle.build()
    monkeypatch.setattr(oracle, "gemm_rowsum", MUTANTS[name])
    caught = []
    for pin in PINS:
        try:
            pin()
        except (AssertionError, ValueError, IndexError) as exc:
            caught.append(pin.__name__)
        except pytest.fail.Exception:
            caught.append(pin.__name__)
    assert caught, f"planted mistake '{name}' passed every pin"
