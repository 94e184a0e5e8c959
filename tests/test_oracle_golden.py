"""The oracle still returns what it returned when the fixture was written (tests/golden/make_golden.py)."""
import os

import numpy as np

import oracle
from workloads import get_config, make_problem

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_forward_seed0.txt")


def test_tiny_forward_matches_stored_oracle_values():
    rows = [l.split() for l in open(GOLDEN) if not l.startswith("#")]
    cfg = get_config("tiny")
    pr = make_problem(cfg)
    out = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    assert len(rows) == 20
    for b, n, d, v in rows:
        np.testing.assert_allclose(out[int(b), int(n), int(d)], float(v), rtol=1e-13, atol=1e-13)


def test_tiny_backward_matches_stored_oracle_values():
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(os.path.dirname(GOLDEN), "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    cfg = get_config("tiny")
    pr = make_problem(cfg)
    g = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, mg.upstream(cfg))
    rows = [l.split() for l in open(os.path.join(os.path.dirname(GOLDEN), "tiny_backward_seed0.txt"))
            if not l.startswith("#")]
    assert len(rows) == len(mg.GRAD_ENTRIES)
    for row in rows:
        name, idx, v = row[0], tuple(int(i) for i in row[1:-1]), float(row[-1])
        np.testing.assert_allclose(mg.grad_entry(g, name, idx), v, rtol=1e-12, atol=1e-13)
