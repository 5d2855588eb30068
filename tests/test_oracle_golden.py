"""The oracle still reproduces the stored Tiny-workload figures (drift guard)."""
import importlib.util
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_tiny_golden_unchanged():
    spec = importlib.util.spec_from_file_location("make_tiny_golden", os.path.join(HERE, "golden", "make_tiny_golden.py"))
    mod = importlib.util.module_from_spec(spec); spec.loader.exec_module(mod)
    got = [r.split() for r in mod.rows(mod.tiny_outputs())]
    with open(os.path.join(HERE, "golden", "tiny_oracle.txt")) as f:
        want = [l.split() for l in f if not l.startswith("#")]
    assert len(got) == len(want) == 7
    for g, w in zip(got, want):
        assert np.allclose([float(v) for v in g], [float(v) for v in w], rtol=1e-9, atol=1e-12)


def test_tree_golden_unchanged():
    spec = importlib.util.spec_from_file_location("make_tree_golden", os.path.join(HERE, "golden", "make_tree_golden.py"))
    mod = importlib.util.module_from_spec(spec); spec.loader.exec_module(mod)
    got = [r.split() for r in mod.rows(mod.tree_outputs())]
    with open(os.path.join(HERE, "golden", "tree_oracle.txt")) as f:
        want = [l.split() for l in f if not l.startswith("#")]
    assert len(got) == len(want) == 3
    for g, w in zip(got, want):
        assert np.allclose([float(v) for v in g], [float(v) for v in w], rtol=1e-9, atol=1e-12)
