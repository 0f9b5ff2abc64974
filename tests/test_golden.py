"""The oracles still return, bit for bit, the values frozen under tests/golden/ (written by
tests/golden/make_golden.py from oracle/ alone).  A change to an oracle's arithmetic must come with
regenerated files and a stated reason."""
import importlib.util
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def _load_maker():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_oracles_match_frozen_values(oracle):
    maker = _load_maker()
    for name, arr in maker.cases().items():
        path = os.path.join(HERE, "golden", name + ".txt")
        rows = [[float.fromhex(t) for t in line.split()] for line in open(path) if not line.startswith("#")]
        want = np.array(rows, dtype=np.float64)
        got = np.atleast_2d(arr)
        assert got.shape == want.shape, name
        assert np.array_equal(got, want), name
