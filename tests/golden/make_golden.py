"""Writes tests/golden/tiny_forward_seed0.txt and tiny_backward_seed0.txt from the CPU oracle alone.

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
    write_backward(cfg, pr)


# entries of the gradient tensors that are stored: (tensor, index)
GRAD_ENTRIES = [("dWe", (0, 0, 0)), ("dWe", (7, 127, 15)), ("dtok_bias", (3, 64)),
                ("l0.dWq", (0, 1, 2)), ("l0.dWk", (1, 31, 7)), ("l0.dWv", (1, 127, 127)), ("l0.dWo", (0, 5, 99)),
                ("l0.dquery", (1, 17)), ("l0.dbv", (0, 3)), ("l1.dWk", (0, 64, 64)), ("l1.dWv", (0, 0, 127)),
                ("l1.dbo", (0, 126)), ("dx", (5, 3, 9))]


def upstream(cfg):
    """The seeded upstream gradient of the fixture: N(0, 1), PCG64(123), [B*N, D]."""
    return np.random.Generator(np.random.PCG64(123)).standard_normal((cfg.B * cfg.N, cfg.D))


def grad_entry(g, name, idx):
    if name.startswith("l"):
        lvl, key = name.split(".")
        return g["levels"][int(lvl[1:])][key][idx]
    return g[name][idx]


def write_backward(cfg, pr):
    g = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, upstream(cfg))
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_backward_seed0.txt")
    with open(path, "w") as f:
        f.write("# oracle.backward on the tiny configuration, seed 0, upstream gradient N(0,1) from PCG64(123);\n")
        f.write("# columns: tensor index... value (fp64, %.17g); dx is indexed [sample = b*N + n, channel, pixel]\n")
        f.write("# written by tests/golden/make_golden.py from oracle/ alone; not a value printed in the paper\n")
        for name, idx in GRAD_ENTRIES:
            f.write(f"{name} {' '.join(str(i) for i in idx)} {grad_entry(g, name, idx):.17g}\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
