"""The oracle against its stored values (tests/golden/tiny_oracle.json, written by tests/golden/make_golden.py
from the oracle alone): a regression pin, CPU only."""
import importlib.util
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_reproduces_its_golden_values(oracle):
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    ref = json.load(open(os.path.join(HERE, "golden", "tiny_oracle.json")))
    assert set(now) == set(ref)
    for k, v in ref.items():
        if isinstance(v, str) or (isinstance(v, list) and v and not isinstance(np.asarray(v).flat[0], (float, np.floating))):
            assert now[k] == v, k
        elif isinstance(v, (int,)):
            assert now[k] == v, k
        else:
            a, b = np.asarray(now[k], np.float64), np.asarray(v, np.float64)
            assert a.shape == b.shape and np.all(np.abs(a - b) <= 1e-12 * np.maximum(1.0, np.abs(b))), k
