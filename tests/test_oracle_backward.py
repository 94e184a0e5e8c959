"""Pins of the oracle's backward pass (no GPU needed).

The paper trains through the channel-aggregation module (Section 3.3 describes its backward
pass only as needing no communication) and prints no gradient values, so the oracle's backward
is pinned to things other than itself:
  * central finite differences of the oracle's (separately pinned) forward;
  * a library autograd through the library composition grouped conv2d -> multi-head attention
    with a length-1 query per group -> ... -> final attention layer;
  * identities the derivative fixes (zero key-bias gradient, linearity in the upstream gradient,
    additivity over patches, a group of one, uniform attention).
"""
import numpy as np
import pytest
import torch

import oracle
from workloads import ShapeCfg, make_problem, n_groups

def small_cfg(**kw):
    base = dict(name="s", dtype="f32", B=2, C=6, H=4, W=6, p=2, D=8, heads=2, group_sizes=(3, 2),
                x_kind="gauss_mu_sigma", seed=21)
    base.update(kw)
    return ShapeCfg(**base)


CASES = [
    dict(),                                                                       # 6 -> 2 -> 1
    dict(C=7, group_sizes=(3, 3), heads=4),                                       # uneven last group (3, 3, 1)
    dict(C=5, D=6, heads=1, group_sizes=(5,), p=1, H=3, W=4),                     # flat single layer, 1x1 patches
    dict(C=9, D=4, heads=2, group_sizes=(2, 3, 2), B=1),                          # three levels, 9 -> 5 -> 2 -> 1
    dict(C=7, group_sizes=(3, 3), level_kinds=("linear", "attention")),           # D-CHAG-L
    dict(C=9, D=4, heads=2, group_sizes=(2, 3, 2), level_kinds=("linear", "linear", "attention"), B=1),
]


def upstream(cfg, seed=3):
    return np.random.default_rng(seed).standard_normal((cfg.B * cfg.N, cfg.D))


def f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


# ---------------------------------------------------------------------------
# library autograd through library ops
# ---------------------------------------------------------------------------
def torch_forward(pr, leaves):
    """The path composed from library routines; `leaves` maps names to float64 tensors that require grad."""
    cfg = pr.cfg
    p, C, D, heads = cfg.p, cfg.C, cfg.D, cfg.heads
    w = leaves["We"].reshape(C * D, 1, p, p)
    t = torch.nn.functional.conv2d(leaves["x"], w, bias=leaves["be"].reshape(-1), stride=p, groups=C)
    z = t.reshape(cfg.B, C, D, cfg.N).permute(0, 3, 1, 2) + leaves["ce"][None, None]          # [B, N, C, D]
    z = z.reshape(cfg.B * cfg.N, C, D)
    for li, lv in enumerate(pr.levels):
        c_in, g = z.shape[1], lv.group_size
        outs = []
        for k in range(n_groups(c_in, g)):
            mem = z[:, k * g:min((k + 1) * g, c_in), :]                                        # [S, m, D]
            if lv.kind == "linear":
                wk = leaves[f"l{li}.Wv"][k, :mem.shape[1]]
                outs.append((mem * wk[None]).sum(dim=1) + leaves[f"l{li}.bv"][k][None])
                continue
            S = mem.shape[0]
            q = leaves[f"l{li}.query"][k].reshape(1, 1, D).expand(1, S, D)
            kv = mem.permute(1, 0, 2)
            in_w = torch.cat([leaves[f"l{li}.Wq"][k], leaves[f"l{li}.Wk"][k], leaves[f"l{li}.Wv"][k]], dim=0)
            in_b = torch.cat([leaves[f"l{li}.bq"][k], leaves[f"l{li}.bk"][k], leaves[f"l{li}.bv"][k]], dim=0)
            out, _ = torch.nn.functional.multi_head_attention_forward(
                q, kv, kv, D, heads, in_w, in_b, None, None, False, 0.0, leaves[f"l{li}.Wo"][k],
                leaves[f"l{li}.bo"][k], training=False, need_weights=False)
            outs.append(out[0])
        z = torch.stack(outs, dim=1)
    return z[:, 0, :]


def make_leaves(pr):
    leaves = {"x": f64(pr.x), "We": f64(pr.We), "be": f64(pr.be), "ce": f64(pr.ce)}
    for li, lv in enumerate(pr.levels):
        names = ("Wv", "bv") if lv.kind == "linear" else ("query", "Wq", "Wk", "Wv", "Wo", "bq", "bk", "bv", "bo")
        for n in names:
            leaves[f"l{li}.{n}"] = f64(getattr(lv, n))
    return {k: torch.from_numpy(v.copy()).requires_grad_(True) for k, v in leaves.items()}


def patches_of(dximg, cfg):
    """[B, C, H, W] -> [B*N, C, p*p], pixels of a patch row by row, patches row by row."""
    p = cfg.p
    a = dximg.reshape(cfg.B, cfg.C, cfg.H // p, p, cfg.W // p, p).transpose(0, 2, 4, 1, 3, 5)
    return a.reshape(cfg.B * cfg.N, cfg.C, p * p)


@pytest.mark.parametrize("kw", CASES)
def test_backward_matches_library_autograd(kw):
    cfg = small_cfg(**kw)
    pr = make_problem(cfg)
    dout = upstream(cfg)
    got = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, dout)
    leaves = make_leaves(pr)
    out = torch_forward(pr, leaves)
    np.testing.assert_allclose(out.detach().numpy(),
                               oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads), atol=1e-11)
    (out * torch.from_numpy(dout)).sum().backward()

    def check(name, a, b):
        scale = max(1.0, float(np.abs(b).max()))
        assert np.abs(a - b).max() < 1e-10 * scale, name

    check("dx", got["dx"], patches_of(leaves["x"].grad.numpy(), cfg))
    check("dWe", got["dWe"], leaves["We"].grad.numpy())
    check("dbe", got["dtok_bias"], leaves["be"].grad.numpy())
    check("dce", got["dtok_bias"], leaves["ce"].grad.numpy())
    for li, lv in enumerate(pr.levels):
        names = ("Wv", "bv") if lv.kind == "linear" else ("query", "Wq", "Wk", "Wv", "Wo", "bq", "bk", "bv", "bo")
        for n in names:
            want = leaves[f"l{li}.{n}"].grad.numpy()
            have = got["levels"][li]["d" + n]
            # (weights of members a short last linear group does not have receive no gradient on either side)
            check(f"l{li}.d{n}", have, want)


# ---------------------------------------------------------------------------
# central finite differences of the forward oracle
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kw", [CASES[1], CASES[3], CASES[4]])
def test_backward_matches_finite_differences_of_the_forward(kw):
    cfg = small_cfg(**kw)
    pr = make_problem(cfg)
    dout = upstream(cfg, seed=4)
    got = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, dout)

    def loss():
        return float((oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads) * dout).sum())

    rng = np.random.default_rng(8)
    h = np.float32(2.0 ** -8)

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = old + h
        hi_v, lp = arr[idx], loss()
        arr[idx] = old - h
        lo_v, lm = arr[idx], loss()
        arr[idx] = old
        return (lp - lm) / (float(hi_v) - float(lo_v))

    def probe(name, arr, grad, n=4):
        for _ in range(n):
            idx = tuple(int(rng.integers(0, s)) for s in arr.shape)
            want = fd(arr, idx)
            assert abs(grad[idx] - want) < 2e-4 * max(1.0, abs(want)), (name, idx, grad[idx], want)

    probe("We", pr.We, got["dWe"])
    probe("be", pr.be, got["dtok_bias"])
    probe("ce", pr.ce, got["dtok_bias"])
    p = cfg.p
    ximg = got["dx"].reshape(cfg.B, cfg.H // p, cfg.W // p, cfg.C, p, p).transpose(0, 3, 1, 4, 2, 5).reshape(pr.x.shape)
    probe("x", pr.x, ximg, n=6)
    for li, lv in enumerate(pr.levels):
        names = ("Wv", "bv") if lv.kind == "linear" else ("query", "Wq", "Wk", "Wv", "Wo", "bq", "bv", "bo")
        for n in names:
            arr = getattr(lv, n)
            if lv.kind == "linear" and n == "Wv":
                arr_probe = arr[:-1] if arr.shape[0] > 1 else arr      # stay off a short group's unused members
                probe(f"l{li}.{n}", arr_probe, got["levels"][li]["d" + n][:arr_probe.shape[0]])
            else:
                probe(f"l{li}.{n}", arr, got["levels"][li]["d" + n])


# ---------------------------------------------------------------------------
# identities of the derivative
# ---------------------------------------------------------------------------
def test_key_bias_has_zero_gradient_and_token_biases_share_theirs():
    """The key bias shifts every score of a softmax equally, so the loss does not depend on it."""
    cfg = small_cfg(C=7, group_sizes=(3, 3))
    pr = make_problem(cfg)
    got = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, upstream(cfg))
    for lg in got["levels"]:
        assert np.abs(lg["dbk"]).max() < 1e-12
        assert np.abs(lg["dbv"]).max() > 1e-3


def test_backward_is_linear_in_the_upstream_gradient_and_additive_over_patches():
    cfg = small_cfg()
    pr = make_problem(cfg)
    da, db = upstream(cfg, 1), upstream(cfg, 2)
    run = lambda d, s=None: oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, d, sample=s)
    ga, gb, gab = run(da), run(db), run(2.0 * da - 3.0 * db)
    np.testing.assert_allclose(gab["dWe"], 2.0 * ga["dWe"] - 3.0 * gb["dWe"], atol=1e-11)
    np.testing.assert_allclose(gab["levels"][0]["dWk"], 2.0 * ga["levels"][0]["dWk"] - 3.0 * gb["levels"][0]["dWk"],
                               atol=1e-11)
    # a sample of patches: the sum over its halves; a patch listed twice counts twice
    S = cfg.B * cfg.N
    sb = np.repeat(np.arange(cfg.B), cfg.N).astype(np.int32)
    sn = np.tile(np.arange(cfg.N), cfg.B).astype(np.int32)
    first, second = slice(0, S // 2), slice(S // 2, S)
    g1 = run(da[first], (sb[first], sn[first]))
    g2 = run(da[second], (sb[second], sn[second]))
    np.testing.assert_allclose(ga["levels"][1]["dWv"], g1["levels"][1]["dWv"] + g2["levels"][1]["dWv"], atol=1e-11)
    np.testing.assert_allclose(ga["dx"][second], g2["dx"], atol=1e-12)
    twice = run(np.concatenate([da[first], da[first]]), (np.concatenate([sb[first]] * 2), np.concatenate([sn[first]] * 2)))
    np.testing.assert_allclose(twice["dWe"], 2.0 * g1["dWe"], atol=1e-11)


def test_group_of_one_backward_is_the_two_projections():
    """With one member per group the softmax weight is 1: y = Wo (Wv z + bv) + bo, so
    dz = Wv^T Wo^T dy, the query path receives nothing."""
    cfg = small_cfg(C=3, group_sizes=(1, 3), heads=2)
    pr = make_problem(cfg)
    lv = pr.levels[0]
    got = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, upstream(cfg))
    l0 = got["levels"][0]
    for n in ("dquery", "dWq", "dWk", "dbq", "dbk"):
        assert np.abs(l0[n]).max() < 1e-12, n
    assert np.abs(l0["dWv"]).max() > 1e-3 and np.abs(l0["dWo"]).max() > 1e-3
    # y depends on bv only through Wo
    for k in range(3):
        np.testing.assert_allclose(l0["dbv"][k], f64(lv.Wo[k]).T @ l0["dbo"][k], atol=1e-10)


def test_value_bias_gradient_is_the_output_projection_of_the_output_bias_gradient():
    """Softmax weights sum to one, so bv reaches the output as Wo bv whatever the scores are."""
    cfg = small_cfg(C=7, group_sizes=(3, 3), heads=4)
    pr = make_problem(cfg)
    got = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, upstream(cfg))
    for li, lv in enumerate(pr.levels):
        for k in range(lv.Wo.shape[0]):
            np.testing.assert_allclose(got["levels"][li]["dbv"][k], f64(lv.Wo[k]).T @ got["levels"][li]["dbo"][k],
                                       atol=1e-10)
    # last level: dbo is the plain sum of the upstream gradient
    np.testing.assert_allclose(got["levels"][-1]["dbo"][0], upstream(cfg).sum(axis=0), atol=1e-11)
