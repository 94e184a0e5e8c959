"""Pins of the oracle's linear partial-aggregation level (D-CHAG-L, paper Sections 3.2 and 3.3).

The paper only says that intermediate cross-attention layers can be replaced by lightweight linear
layers with fewer parameters while the final layer stays cross-attention; the reading pinned here is
y = sum_c w[c] * z[c] + b along the channel axis, elementwise in the feature.
"""
import numpy as np
import pytest

import oracle
from workloads import ShapeCfg, make_level, make_linear_level, make_problem, n_groups

TOL = 1e-12


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def f64(a):
    return np.asarray(a, dtype=np.float64)


@pytest.mark.parametrize("c_in,g,D", [(6, 3, 8), (7, 3, 4), (5, 8, 6), (4, 1, 8)])
def test_linear_level_matches_numpy_and_brute_force(c_in, g, D):
    G = n_groups(c_in, g)
    lv = make_linear_level(rng(c_in), G, g, D, "f32")
    z = rng(1).standard_normal((5, c_in, D))
    y = oracle.aggregate_level(z, lv, 2 if D % 2 == 0 else 1)
    assert y.shape == (5, G, D)
    for k in range(G):
        mem = range(k * g, min((k + 1) * g, c_in))
        want = sum(f64(lv.Wv[k, c - k * g])[None, :] * z[:, c, :] for c in mem) + f64(lv.bv[k])[None, :]
        np.testing.assert_allclose(y[:, k], want, rtol=0, atol=TOL)
    # explicit scalar loops on one patch
    s = 3
    for k in range(G):
        for d in range(D):
            acc = float(lv.bv[k, d])
            for c in range(k * g, min((k + 1) * g, c_in)):
                acc += float(lv.Wv[k, c - k * g, d]) * z[s, c, d]
            assert abs(y[s, k, d] - acc) < 1e-12


def test_uniform_weights_give_the_mean_and_unit_weight_the_identity():
    g, D = 4, 8
    lv = make_linear_level(rng(2), 2, g, D, "f32", biases=False)
    lv.Wv = np.full_like(lv.Wv, 1.0 / g)
    z = rng(3).standard_normal((3, 2 * g, D))
    y = oracle.aggregate_level(z, lv, 2)
    np.testing.assert_allclose(y[:, 0], z[:, :g].mean(axis=1), rtol=0, atol=1e-7)   # 0.25 is exact in float32
    one = make_linear_level(rng(4), 5, 1, D, "f32")
    y1 = oracle.aggregate_level(z[:, :5], one, 2)
    np.testing.assert_allclose(y1, f64(one.Wv[:, 0])[None] * z[:, :5] + f64(one.bv)[None], rtol=0, atol=TOL)


def test_linear_level_is_linear_and_permutation_covariant():
    g, D = 3, 4
    lv = make_linear_level(rng(5), 1, g, D, "f32", biases=False)
    za, zb = rng(6).standard_normal((2, g, D)), rng(7).standard_normal((2, g, D))
    ya, yb, yc = (oracle.aggregate_level(v, lv, 1) for v in (za, zb, 2.0 * za - 3.0 * zb))
    np.testing.assert_allclose(yc, 2.0 * ya - 3.0 * yb, rtol=0, atol=1e-12)
    perm = [2, 0, 1]
    lv2 = make_linear_level(rng(5), 1, g, D, "f32", biases=False)
    lv2.Wv = np.ascontiguousarray(lv.Wv[:, perm])
    np.testing.assert_allclose(oracle.aggregate_level(za[:, perm], lv2, 1), ya, rtol=0, atol=1e-12)


def test_forward_with_linear_partial_levels_is_the_composition():
    cfg = ShapeCfg("l", "f32", 2, 7, 4, 6, 2, 8, 2, (3, 3), "gauss", 9, ("linear", "attention"))
    pr = make_problem(cfg)
    assert pr.levels[0].kind == "linear" and pr.levels[1].kind == "attention"
    t = oracle.tokenize(pr.x, pr.We, pr.be, pr.ce, cfg.p)
    z1 = oracle.aggregate_level(t, pr.levels[0], cfg.heads)
    z2 = oracle.aggregate_level(z1, pr.levels[1], cfg.heads)
    out = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads)
    np.testing.assert_array_equal(out, z2[:, 0])
    # the linear level by hand, groups (3, 3, 1)
    lv = pr.levels[0]
    want = np.stack([sum(f64(lv.Wv[k, c - 3 * k]) * t[:, c] for c in range(3 * k, min(3 * k + 3, 7))) + f64(lv.bv[k])
                     for k in range(3)], axis=1)
    np.testing.assert_allclose(z1, want, rtol=0, atol=TOL)


def test_last_level_must_be_cross_attention():
    cfg = ShapeCfg("l", "f32", 1, 4, 4, 4, 2, 8, 2, (4,), "gauss", 9, ("linear",))
    pr = make_problem(cfg)
    with pytest.raises(ValueError):
        oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads)
    with pytest.raises(ValueError):
        oracle.aggregate_level(np.zeros((1, 4, 8)), pr.levels[0], 2, want_alpha=True)


@pytest.mark.parametrize("old,new", [
    ("acc += (double)lv->Wv[((size_t)k * g + (c - c0)) * D + d] * z[(size_t)c * D + d];",
     "acc += (double)lv->Wv[((size_t)k * g + (c - c0)) * D + d] * z[(size_t)c0 * D + d];"),      # always the first member
    ("acc += (double)lv->Wv[((size_t)k * g + (c - c0)) * D + d] * z[(size_t)c * D + d];",
     "acc += (double)lv->Wv[((size_t)0 * g + (c - c0)) * D + d] * z[(size_t)c * D + d];"),       # group 0's weights
    ("y[(size_t)k * D + d] = acc + (lv->bv ? (double)lv->bv[(size_t)k * D + d] : 0.0);",
     "y[(size_t)k * D + d] = acc;"),                                                             # bias dropped
])
def test_planted_mistakes_in_the_linear_level_are_caught(old, new, tmp_path):
    import os
    src = os.path.join(os.path.dirname(oracle.__file__), "dchag_oracle.c")
    text = open(src).read()
    assert text.count(old) == 1
    bad = tmp_path / "bad.c"
    bad.write_text(text.replace(old, new))
    lib = str(tmp_path / "libbad.so")
    oracle.compile_source(str(bad), lib)
    oracle.use_library(lib)
    try:
        with pytest.raises(AssertionError):
            test_linear_level_matches_numpy_and_brute_force(7, 3, 4)
    finally:
        oracle.use_library(None)
