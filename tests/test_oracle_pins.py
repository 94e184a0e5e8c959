"""Pins of the fp64 CPU oracle to things other than itself (no GPU needed).

The paper (Sections 2.1, 3.2, 3.3) describes the method in prose and prints no
worked numerical example, so the oracle is pinned to: library routines for the
special cases that have one (grouped conv2d, multi-head attention with a
length-1 query), a pure-Python brute force in a different loop order, the
invariants the definition fixes, and algebraic identities in numpy fp64.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from workloads import Level, ShapeCfg, get_config, make_problem, n_groups

TOL = 1e-11


def small_cfg(**kw):
    base = dict(name="s", dtype="f32", B=2, C=6, H=4, W=6, p=2, D=8, heads=2, group_sizes=(3, 2),
                x_kind="gauss_mu_sigma", seed=11)
    base.update(kw)
    return ShapeCfg(**base)


def f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def level_slice(lv: Level, k: int, g: int) -> Level:
    """Group k of a level as a one-group level of its own."""
    def s(a):
        return None if a is None else a[k:k + 1]
    return Level(g, s(lv.query), s(lv.Wq), s(lv.Wk), s(lv.Wv), s(lv.Wo), s(lv.bq), s(lv.bk), s(lv.bv), s(lv.bo))


# ---------------------------------------------------------------------------
# library special cases
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("p,H,W", [(2, 4, 6), (4, 8, 12), (1, 3, 5)])
def test_tokenizer_is_a_grouped_conv2d(p, H, W):
    """Section 2.1: each channel's patches go through that channel's own conv (kernel = stride = p)."""
    cfg = small_cfg(p=p, H=H, W=W, C=5, D=7, heads=1, group_sizes=(5,))
    pr = make_problem(cfg)
    t = oracle.tokenize(pr.x, pr.We, pr.be, pr.ce, p)                        # [B*N, C, D]
    w = torch.from_numpy(f64(pr.We)).reshape(cfg.C * cfg.D, 1, p, p)
    y = torch.nn.functional.conv2d(torch.from_numpy(f64(pr.x)), w, bias=torch.from_numpy(f64(pr.be)).reshape(-1),
                                   stride=p, groups=cfg.C)                  # [B, C*D, H/p, W/p]
    y = y.reshape(cfg.B, cfg.C, cfg.D, cfg.N).permute(0, 3, 1, 2)            # [B, N, C, D]
    y = y + torch.from_numpy(f64(pr.ce))[None, None]
    np.testing.assert_allclose(t.reshape(cfg.B, cfg.N, cfg.C, cfg.D), y.numpy(), rtol=0, atol=TOL)


@pytest.mark.parametrize("heads,D,g", [(1, 8, 5), (2, 8, 3), (4, 16, 7)])
def test_one_group_is_library_multihead_attention(heads, D, g):
    """Section 2.1: a cross-attention layer reduces the channels to one representation;
    with one learned query this is a library MHA call with query length 1."""
    cfg = small_cfg(C=g, D=D, heads=heads, group_sizes=(g,))
    pr = make_problem(cfg)
    lv = pr.levels[0]
    rng = np.random.default_rng(5)
    S = 9
    z = rng.standard_normal((S, g, D))
    y = oracle.aggregate_level(z, lv, heads)                                  # [S, 1, D]
    q = torch.from_numpy(f64(lv.query[0])).reshape(1, 1, D).expand(1, S, D)
    kv = torch.from_numpy(z).permute(1, 0, 2).contiguous()                    # [g, S, D]
    in_w = torch.from_numpy(np.concatenate([f64(lv.Wq[0]), f64(lv.Wk[0]), f64(lv.Wv[0])], axis=0))
    in_b = torch.from_numpy(np.concatenate([f64(lv.bq[0]), f64(lv.bk[0]), f64(lv.bv[0])], axis=0))
    out, _ = torch.nn.functional.multi_head_attention_forward(
        q, kv, kv, D, heads, in_w, in_b, None, None, False, 0.0,
        torch.from_numpy(f64(lv.Wo[0])), torch.from_numpy(f64(lv.bo[0])), training=False, need_weights=False)
    np.testing.assert_allclose(y[:, 0, :], out[0].numpy(), rtol=0, atol=TOL)


# ---------------------------------------------------------------------------
# brute force, explicit scalar loops, another loop order (heads outermost,
# scores through an explicit double sum over both projections)
# ---------------------------------------------------------------------------

def brute_forward(pr, b, n):
    cfg = pr.cfg
    p, D, h = cfg.p, cfg.D, cfg.heads
    dh = D // h
    pw = cfg.W // p
    pi, pj = divmod(n, pw)
    toks = []
    for c in range(cfg.C):
        t = []
        for d in range(D):
            acc = float(pr.ce[c, d]) if pr.ce is not None else 0.0
            if pr.be is not None:
                acc += float(pr.be[c, d])
            for s in range(p):              # columns first, then rows: another order than the oracle
                for r in range(p):
                    acc += float(pr.We[c, d, r * p + s]) * float(pr.x[b, c, pi * p + r, pj * p + s])
            t.append(acc)
        toks.append(t)
    z = toks
    for lv in pr.levels:
        g = lv.group_size
        G = (len(z) + g - 1) // g
        heads_out = [[0.0] * D for _ in range(G)]
        for a in range(h):
            for k in range(G):
                members = list(range(k * g, min((k + 1) * g, len(z))))
                Qa = []
                for i in range(a * dh, (a + 1) * dh):
                    acc = float(lv.bq[k, i]) if lv.bq is not None else 0.0
                    for j in range(D):
                        acc += float(lv.Wq[k, i, j]) * float(lv.query[k, j])
                    Qa.append(acc)
                sc = []
                for c in members:
                    acc = 0.0
                    for ii, i in enumerate(range(a * dh, (a + 1) * dh)):
                        kij = float(lv.bk[k, i]) if lv.bk is not None else 0.0
                        for j in range(D):
                            kij += float(lv.Wk[k, i, j]) * z[c][j]
                        acc += Qa[ii] * kij
                    sc.append(acc / math.sqrt(dh))
                mx = max(sc)
                ex = [math.exp(v - mx) for v in sc]
                den = sum(ex)
                for i in range(a * dh, (a + 1) * dh):
                    acc = 0.0
                    for w, c in zip(ex, members):
                        v = float(lv.bv[k, i]) if lv.bv is not None else 0.0
                        for j in range(D):
                            v += float(lv.Wv[k, i, j]) * z[c][j]
                        acc += (w / den) * v
                    heads_out[k][i] = acc
        nz = []
        for k in range(G):
            row = []
            for i in range(D):
                acc = float(lv.bo[k, i]) if lv.bo is not None else 0.0
                for j in range(D):
                    acc += float(lv.Wo[k, i, j]) * heads_out[k][j]
                row.append(acc)
            nz.append(row)
        z = nz
    assert len(z) == 1
    return np.asarray(z[0])


@pytest.mark.parametrize("kw", [
    dict(C=6, D=8, heads=2, group_sizes=(3, 2), p=2),
    dict(C=5, D=6, heads=1, group_sizes=(2, 3), p=1, H=3, W=4),          # uneven last group: 2,2,1
    dict(C=4, D=4, heads=2, group_sizes=(4,), p=2),                      # flat single layer
    dict(C=6, D=4, heads=4, group_sizes=(2, 2, 2), p=2),                 # three levels, 3 -> 2 (2+1) -> 1
])
@pytest.mark.parametrize("biases", [True, False])
def test_forward_matches_brute_force_micro(kw, biases):
    cfg = small_cfg(**kw)
    pr = make_problem(cfg, biases=biases)
    out = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    for b, n in [(0, 0), (cfg.B - 1, cfg.N - 1), (0, cfg.N // 2)]:
        np.testing.assert_allclose(out[b, n], brute_forward(pr, b, n), rtol=0, atol=TOL)


def test_forward_matches_brute_force_on_tiny_config():
    """The tiny configuration (8 channels -> 2 groups of 4 -> 1): the two-layer sketch of Section 3.2."""
    cfg = get_config("tiny")
    pr = make_problem(cfg)
    bs = np.array([0, 0, 0], dtype=np.int32)
    ns = np.array([0, 77, cfg.N - 1], dtype=np.int32)
    out = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, sample=(bs, ns))
    for i in range(3):
        np.testing.assert_allclose(out[i], brute_forward(pr, int(bs[i]), int(ns[i])), rtol=0, atol=1e-10)


# ---------------------------------------------------------------------------
# invariants of the definition
# ---------------------------------------------------------------------------

def rand_level(G, g, D, seed, biases=True):
    from workloads import make_level
    return make_level(np.random.Generator(np.random.PCG64(seed)), G, g, D, "f32", biases)


def test_group_of_one_is_value_then_output_projection():
    D, h, c_in = 8, 2, 4
    lv = rand_level(c_in, 1, D, 1)
    z = np.random.default_rng(0).standard_normal((5, c_in, D))
    y = oracle.aggregate_level(z, lv, h)
    for k in range(c_in):
        want = (z[:, k] @ f64(lv.Wv[k]).T + f64(lv.bv[k])) @ f64(lv.Wo[k]).T + f64(lv.bo[k])
        np.testing.assert_allclose(y[:, k], want, rtol=0, atol=TOL)


@pytest.mark.parametrize("how", ["zero_wk", "zero_query_proj", "identical_tokens"])
def test_identical_keys_give_the_mean_of_values(how):
    D, h, g = 8, 2, 5
    lv = rand_level(1, g, D, 2)
    z = np.random.default_rng(1).standard_normal((4, g, D))
    if how == "zero_wk":
        lv.Wk = np.zeros_like(lv.Wk)
    elif how == "zero_query_proj":
        lv.Wq = np.zeros_like(lv.Wq)
        lv.bq = None
    else:
        z[:] = z[:, :1]
    y, alpha = oracle.aggregate_level(z, lv, h, want_alpha=True)
    np.testing.assert_allclose(alpha, 1.0 / g, rtol=0, atol=1e-14)
    vmean = (z @ f64(lv.Wv[0]).T + f64(lv.bv[0])).mean(axis=1)
    np.testing.assert_allclose(y[:, 0], vmean @ f64(lv.Wo[0]).T + f64(lv.bo[0]), rtol=0, atol=TOL)


def permute_channels(pr, perm):
    pr.x = np.ascontiguousarray(pr.x[:, perm])
    pr.We = np.ascontiguousarray(pr.We[perm])
    pr.be = np.ascontiguousarray(pr.be[perm])
    pr.ce = np.ascontiguousarray(pr.ce[perm])


def test_permutation_inside_groups_is_invisible_across_groups_is_not():
    cfg = small_cfg(C=6, group_sizes=(3, 2))
    pr = make_problem(cfg)
    ref = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads)
    pr2 = make_problem(cfg)
    permute_channels(pr2, [2, 0, 1, 4, 5, 3])          # stays inside {0,1,2} and {3,4,5}
    same = oracle.forward(pr2.x, pr2.We, pr2.be, pr2.ce, pr2.levels, cfg.p, cfg.heads)
    np.testing.assert_allclose(same, ref, rtol=0, atol=TOL)
    pr3 = make_problem(cfg)
    permute_channels(pr3, [0, 1, 3, 2, 4, 5])          # swaps a channel across the two groups
    diff = oracle.forward(pr3.x, pr3.We, pr3.be, pr3.ce, pr3.levels, cfg.p, cfg.heads)
    assert np.abs(diff - ref).max() > 1e-3


def test_one_group_then_top_level_is_the_composed_flat_computation():
    cfg = small_cfg(C=5, group_sizes=(5, 1))
    pr = make_problem(cfg)
    out = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads)
    flat = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels[:1], cfg.p, cfg.heads)   # single layer
    l2 = pr.levels[1]
    want = (flat @ f64(l2.Wv[0]).T + f64(l2.bv[0])) @ f64(l2.Wo[0]).T + f64(l2.bo[0])
    np.testing.assert_allclose(out, want, rtol=0, atol=TOL)


def test_forward_is_tokenize_then_levels():
    cfg = small_cfg(C=7, group_sizes=(3, 2, 2))
    pr = make_problem(cfg)
    z = oracle.tokenize(pr.x, pr.We, pr.be, pr.ce, cfg.p)
    for lv in pr.levels:
        z = oracle.aggregate_level(z, lv, cfg.heads)
    out = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads)
    np.testing.assert_array_equal(z[:, 0], out)


def test_key_bias_and_score_shift_do_not_matter():
    D, h, g = 8, 2, 4
    lv = rand_level(2, g, D, 3)
    z = np.random.default_rng(2).standard_normal((3, 2 * g, D))
    y0 = oracle.aggregate_level(z, lv, h)
    lv.bk = None
    y1 = oracle.aggregate_level(z, lv, h)
    np.testing.assert_allclose(y1, y0, rtol=0, atol=TOL)
    lv.bk = np.full((2, D), 3.5, dtype=np.float32)
    np.testing.assert_allclose(oracle.aggregate_level(z, lv, h), y0, rtol=0, atol=TOL)


def test_duplicating_every_member_changes_nothing():
    D, h, g = 8, 4, 3
    lv = rand_level(1, g, D, 4)
    z = np.random.default_rng(3).standard_normal((4, g, D))
    y0 = oracle.aggregate_level(z, lv, h)
    lv2 = level_slice(lv, 0, 2 * g)
    y1 = oracle.aggregate_level(np.concatenate([z, z], axis=1), lv2, h)
    np.testing.assert_allclose(y1, y0, rtol=0, atol=TOL)


def test_softmax_weights_are_a_convex_combination():
    D, h, g, c_in = 8, 2, 3, 8                          # groups 3, 3, 2
    lv = rand_level(n_groups(c_in, g), g, D, 5)
    z = np.random.default_rng(4).standard_normal((6, c_in, D))
    y, alpha, pre = oracle.aggregate_level(z, lv, h, want_alpha=True, want_pre=True)
    assert (alpha > 0).all()
    dh = D // h
    for k in range(n_groups(c_in, g)):
        mem = slice(k * g, min((k + 1) * g, c_in))
        np.testing.assert_allclose(alpha[:, mem].sum(axis=1), 1.0, rtol=0, atol=1e-14)
        V = z[:, mem] @ f64(lv.Wv[k]).T + f64(lv.bv[k])                          # [S, m, D]
        assert (pre[:, k] <= V.max(axis=1) + 1e-12).all() and (pre[:, k] >= V.min(axis=1) - 1e-12).all()
        for a in range(h):
            want = np.einsum("sm,smd->sd", alpha[:, mem, a], V[:, :, a * dh:(a + 1) * dh])
            np.testing.assert_allclose(pre[:, k, a * dh:(a + 1) * dh], want, rtol=0, atol=TOL)
        np.testing.assert_allclose(y[:, k], pre[:, k] @ f64(lv.Wo[k]).T + f64(lv.bo[k]), rtol=0, atol=TOL)


def test_output_depends_only_on_its_own_patch():
    cfg = small_cfg(B=2, H=4, W=6, p=2)
    pr = make_problem(cfg)
    ref = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    x2 = pr.x.copy()
    x2[0, :, 0:2, 2:4] += 1.0                           # batch 0, patch (0,1) = n 1, all channels
    out = oracle.forward(x2, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    changed = np.abs(out - ref).max(axis=-1) > 0
    want = np.zeros((cfg.B, cfg.N), dtype=bool)
    want[0, 1] = True
    np.testing.assert_array_equal(changed, want)


def test_query_scale_limits():
    """A huge query picks the arg-max member per head; a zero query (no q bias) gives the mean."""
    D, h, g = 8, 2, 4
    dh = D // h
    lv = rand_level(1, g, D, 6)
    lv.bq = None
    z = np.random.default_rng(5).standard_normal((5, g, D))
    V = z @ f64(lv.Wv[0]).T + f64(lv.bv[0])
    K = z @ f64(lv.Wk[0]).T + f64(lv.bk[0])
    Q = f64(lv.Wq[0]) @ f64(lv.query[0])
    big = level_slice(lv, 0, g)
    big.query = (lv.query * 1e4).astype(np.float32)
    _, pre = oracle.aggregate_level(z, big, h, want_pre=True)
    for a in range(h):
        sl = slice(a * dh, (a + 1) * dh)
        win = (K[:, :, sl] @ Q[sl]).argmax(axis=1)
        np.testing.assert_allclose(pre[:, 0, sl], V[np.arange(5), win][:, sl], rtol=0, atol=1e-9)
    zero = level_slice(lv, 0, g)
    zero.query = np.zeros_like(lv.query)
    _, pre0 = oracle.aggregate_level(z, zero, h, want_pre=True)
    np.testing.assert_allclose(pre0[:, 0], V.mean(axis=1), rtol=0, atol=TOL)


def test_linear_in_value_and_output_weights():
    D, h, g = 8, 2, 3
    la, lb = rand_level(1, g, D, 7), rand_level(1, g, D, 8)
    z = np.random.default_rng(6).standard_normal((3, g, D))
    # same q/k side, W_o = identity, no b_o: the result is linear in (W_v, b_v)
    for l in (la, lb):
        l.query, l.Wq, l.bq, l.Wk, l.bk = la.query, la.Wq, la.bq, la.Wk, la.bk
        l.Wo = np.eye(D, dtype=np.float32)[None]
        l.bo = None
    lc = level_slice(la, 0, g)
    lc.Wv = (2.0 * la.Wv - 0.5 * lb.Wv).astype(np.float32)
    lc.bv = (2.0 * la.bv - 0.5 * lb.bv).astype(np.float32)
    ya, yb, yc = (oracle.aggregate_level(z, l, h) for l in (la, lb, lc))
    np.testing.assert_allclose(yc, 2.0 * ya - 0.5 * yb, rtol=0, atol=1e-6)   # float32 weights were combined


# ---------------------------------------------------------------------------
# algebraic identities a fast implementation may rely on (numpy fp64)
# ---------------------------------------------------------------------------

def test_identity_query_folded_into_key_weights():
    """s[c,a] = z[c] . M[:,a] + const,  M[:,a] = W_k[a rows]^T Q_a / sqrt(d_h)."""
    D, h, g = 8, 2, 5
    dh = D // h
    lv = rand_level(1, g, D, 9)
    z = np.random.default_rng(7).standard_normal((4, g, D))
    _, alpha = oracle.aggregate_level(z, lv, h, want_alpha=True)
    Q = f64(lv.Wq[0]) @ f64(lv.query[0]) + f64(lv.bq[0])
    for a in range(h):
        sl = slice(a * dh, (a + 1) * dh)
        M = f64(lv.Wk[0])[sl].T @ Q[sl] / math.sqrt(dh)
        s = z @ M
        e = np.exp(s - s.max(axis=1, keepdims=True))
        np.testing.assert_allclose(alpha[:, :, a], e / e.sum(axis=1, keepdims=True), rtol=0, atol=1e-13)


def test_identity_aggregate_then_project():
    """sum_c alpha[c] V_a[c] = W_v[a rows] (sum_c alpha[c] z[c]) + b_v,a  because the weights sum to one."""
    D, h, g = 8, 2, 4
    dh = D // h
    lv = rand_level(1, g, D, 10)
    z = np.random.default_rng(8).standard_normal((4, g, D))
    _, alpha, pre = oracle.aggregate_level(z, lv, h, want_alpha=True, want_pre=True)
    for a in range(h):
        sl = slice(a * dh, (a + 1) * dh)
        zbar = np.einsum("sc,scd->sd", alpha[:, :, a], z)
        np.testing.assert_allclose(pre[:, 0, sl], zbar @ f64(lv.Wv[0])[sl].T + f64(lv.bv[0])[sl], rtol=0, atol=TOL)


def test_identity_projection_folded_into_the_tokenizer():
    """At level 1, V[c] = (W_v W_e[c]) u[c] + W_v (b_e[c] + e[c]) + b_v."""
    cfg = small_cfg(C=3, group_sizes=(3,), B=1)
    pr = make_problem(cfg)
    lv = pr.levels[0]
    t = oracle.tokenize(pr.x, pr.We, pr.be, pr.ce, cfg.p)                          # [N, C, D]
    V = t @ f64(lv.Wv[0]).T + f64(lv.bv[0])
    p, pw = cfg.p, cfg.W // cfg.p
    for n in range(cfg.N):
        pi, pj = divmod(n, pw)
        for c in range(cfg.C):
            u = f64(pr.x[0, c, pi * p:(pi + 1) * p, pj * p:(pj + 1) * p]).reshape(-1)
            want = (f64(lv.Wv[0]) @ f64(pr.We[c])) @ u + f64(lv.Wv[0]) @ (f64(pr.be[c]) + f64(pr.ce[c])) + f64(lv.bv[0])
            np.testing.assert_allclose(V[n, c], want, rtol=0, atol=TOL)


def test_identity_first_level_output_from_the_pixels():
    """The two identities above together, as the inference path uses them at level 1: per head a,
    o_a = sum_c alpha[c,a] ((W_v W_e[c]) u[c] + W_v (b_e[c] + e[c]))_a + b_v,a  (the weights sum to one over the group),
    with a short last group (5 channels in groups of 3 + 2)."""
    cfg = small_cfg(C=5, group_sizes=(3, 2), B=2)
    pr = make_problem(cfg)
    lv = pr.levels[0]
    h, dh = cfg.heads, cfg.D // cfg.heads
    t = oracle.tokenize(pr.x, pr.We, pr.be, pr.ce, cfg.p)                          # [B*N, C, D]
    _, alpha, pre = oracle.aggregate_level(t, lv, h, want_alpha=True, want_pre=True)
    p, pw, g = cfg.p, cfg.W // cfg.p, cfg.group_sizes[0]
    for row in range(cfg.B * cfg.N):
        b, n = divmod(row, cfg.N)
        pi, pj = divmod(n, pw)
        for k in range(n_groups(cfg.C, g)):
            want = f64(lv.bv[k]).copy()
            for c in range(k * g, min((k + 1) * g, cfg.C)):
                u = f64(pr.x[b, c, pi * p:(pi + 1) * p, pj * p:(pj + 1) * p]).reshape(-1)
                v = (f64(lv.Wv[k]) @ f64(pr.We[c])) @ u + f64(lv.Wv[k]) @ (f64(pr.be[c]) + f64(pr.ce[c]))
                for a in range(h):
                    sl = slice(a * dh, (a + 1) * dh)
                    want[sl] += alpha[row, c, a] * v[sl]
            np.testing.assert_allclose(pre[row, k], want, rtol=0, atol=TOL)


# ---------------------------------------------------------------------------
# hierarchy bookkeeping and argument checks
# ---------------------------------------------------------------------------

def test_group_partitions():
    assert n_groups(1000, 16) == 63 and 1000 - 62 * 16 == 8
    assert n_groups(63, 8) == 8 and 63 - 7 * 8 == 7
    assert n_groups(8, 8) == 1
    # Section 4.5: 512 channels on two GPUs; Tree2 -> at most 128 per layer, Tree8 -> at most 32
    per_rank = 512 // 2
    assert per_rank // 2 == 128 and per_rank // 8 == 32
    assert n_groups(512, 32) == 16 == 2 * 8


def test_short_last_group_attends_only_over_real_members():
    D, h, g, c_in = 8, 2, 4, 6                           # groups {0..3}, {4,5}
    lv = rand_level(2, g, D, 12)
    z = np.random.default_rng(9).standard_normal((3, c_in, D))
    y = oracle.aggregate_level(z, lv, h)
    y_last = oracle.aggregate_level(z[:, 4:], level_slice(lv, 1, 2), h)
    np.testing.assert_allclose(y[:, 1], y_last[:, 0], rtol=0, atol=TOL)


def test_oracle_rejects_bad_shapes():
    cfg = small_cfg()
    pr = make_problem(cfg)
    with pytest.raises(ValueError):
        oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels[:1], cfg.p, cfg.heads)       # leaves 2 groups
    with pytest.raises(ValueError):
        oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, 3)                   # D % heads
    with pytest.raises(ValueError):
        oracle.tokenize(pr.x[:, :, :3], pr.We, pr.be, pr.ce, cfg.p)                      # H % p


def test_positional_embedding_is_added_per_patch_and_shared_by_the_batch():
    """Section 2.1: the aggregated token of a patch receives that patch's positional embedding."""
    cfg = small_cfg()
    pr = make_problem(cfg)
    pos = np.random.default_rng(3).standard_normal((cfg.N, cfg.D)).astype(np.float32)
    plain = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads)
    withp = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, pos=pos)
    want = plain.reshape(cfg.B, cfg.N, cfg.D) + f64(pos)[None]
    np.testing.assert_allclose(withp.reshape(cfg.B, cfg.N, cfg.D), want, rtol=0, atol=1e-15)
    # a sample in another order picks the rows of its own patches
    sb = np.array([1, 0, 1], dtype=np.int32)
    sn = np.array([cfg.N - 1, 2, 0], dtype=np.int32)
    some = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, sample=(sb, sn), pos=pos)
    np.testing.assert_allclose(some, want[sb, sn], rtol=0, atol=1e-15)
