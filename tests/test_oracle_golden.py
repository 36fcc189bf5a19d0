"""Regression pin of the oracle against values written earlier by tests/golden/make_golden.py
(which calls only oracle/).  The paper prints no model outputs, so there is no paper fixture."""
import importlib.util
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_matches_its_stored_samples():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.sample()
    stored = {}
    for line in open(os.path.join(HERE, "golden", "tiny_vit_oracle.txt")):
        if line.startswith("#"):
            continue
        name, *vals = line.split()
        stored[name] = np.array([float(v) for v in vals])
    assert set(stored) == set(now)
    for k in stored:
        assert np.allclose(now[k], stored[k], rtol=1e-12, atol=1e-14), k
