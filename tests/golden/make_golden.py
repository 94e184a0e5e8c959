"""Writes tests/golden/tiny_forward_seed0.txt from the CPU oracle alone.

The paper prints no numerical example of the tokenize + aggregate path, so this
fixture is NOT a paper value: it freezes what the pinned oracle returns on the
tiny configuration (8 channels, two groups of four, then one top layer: the
two-layer sketch of Section 3.2), so that a later change to the oracle's
arithmetic or to the input generator shows up as a diff.

Run from the repository root:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from workloads import get_config, make_problem  # noqa: E402

PATCHES = [(0, 0), (0, 1), (0, 63), (0, 127)]


def main():
    cfg = get_config("tiny")
    pr = make_problem(cfg)
    bs = np.array([b for b, _ in PATCHES], dtype=np.int32)
    ns = np.array([n for _, n in PATCHES], dtype=np.int32)
    out = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, sample=(bs, ns))
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_forward_seed0.txt")
    with open(path, "w") as f:
        f.write("# oracle.forward on the tiny configuration, seed 0; columns: b n d value (fp64, %.17g)\n")
        f.write("# written by tests/golden/make_golden.py from oracle/ alone; not a value printed in the paper\n")
        for i, (b, n) in enumerate(PATCHES):
            for d in (0, 1, 31, 64, 127):
                f.write(f"{b} {n} {d} {out[i, d]:.17g}\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
