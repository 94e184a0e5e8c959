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
