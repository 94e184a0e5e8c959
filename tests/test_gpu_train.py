"""GPU parity of the weight-folded forward call and of the backward call, through the C ABI,
against the fp64 CPU oracle on the same seeded inputs.

Error measure, per tensor (output or gradient): max_i |y_i - y^_i| / max_i |y^_i|, below 2e-2 for bf16
(bf16 storage, fp32 accumulation) and 1e-4 for fp32.
"""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2506_21411_amd as dchag
from workloads import ShapeCfg, get_config, make_problem, n_groups, sample_patches, sample_patches_covering

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}
ATT = ("query", "Wq", "Wk", "Wv", "Wo", "bq", "bk", "bv", "bo")


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev(a, dtype):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(TDT[dtype]).contiguous()


def dev_level(lv, dtype):
    return dchag.LevelWeights(lv.group_size, dev(lv.query, dtype), dev(lv.Wq, dtype), dev(lv.Wk, dtype),
                              dev(lv.Wv, dtype), dev(lv.Wo, dtype), dev(lv.bq, dtype), dev(lv.bk, dtype),
                              dev(lv.bv, dtype), dev(lv.bo, dtype), kind=1 if lv.kind == "linear" else 0)


def host(t):
    return t.detach().to(torch.float64).cpu().numpy()


def rel_err(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all()
    return float(np.abs(got - want).max() / np.abs(want).max())


def cfg_of(**kw):
    base = dict(name="t", dtype="f32", B=2, C=6, H=8, W=12, p=2, D=32, heads=4, group_sizes=(3, 2),
                x_kind="gauss_mu_sigma", seed=3)
    base.update(kw)
    return ShapeCfg(**base)


SMALL = [
    dict(dtype="f32", B=2, C=7, H=8, W=12, p=2, D=32, heads=4, group_sizes=(3, 2, 2)),      # 7 -> 3 -> 2 -> 1
    dict(dtype="f32", B=1, C=5, H=4, W=4, p=2, D=24, heads=3, group_sizes=(5,)),            # flat single layer
    dict(dtype="f32", B=1, C=70, H=10, W=14, p=2, D=72, heads=2, group_sizes=(40, 2)),      # groups 40 + 30: two 32-member chunks
    dict(dtype="f32", B=2, C=7, H=8, W=12, p=2, D=32, heads=4, group_sizes=(3, 3), level_kinds=("linear", "attention")),
    dict(dtype="bf16", B=2, C=20, H=16, W=24, p=4, D=256, heads=4, group_sizes=(8, 3)),     # groups 8, 8, 4
    dict(dtype="bf16", B=1, C=9, H=24, W=40, p=8, D=512, heads=8, group_sizes=(4, 3)),      # groups 4, 4, 1
    dict(dtype="bf16", B=1, C=6, H=8, W=8, p=2, D=64, heads=2, group_sizes=(2, 2, 2)),      # three levels
    dict(dtype="bf16", B=1, C=10, H=80, W=72, p=8, D=320, heads=20, group_sizes=(5, 2)),    # 20 heads (two head passes), N = 90
    dict(dtype="bf16", B=2, C=12, H=16, W=16, p=4, D=256, heads=2, group_sizes=(3, 2, 2),
         level_kinds=("linear", "linear", "attention")),
    # N = 192 patches (a multiple of 64: the products over patches take the MFMA kernel, 1.5 row tiles of 128),
    # 16 heads of 16 (not a fast-level shape: generic scores, MFMA products), groups 5 + 5 + 3
    dict(dtype="bf16", B=2, C=13, H=32, W=96, p=4, D=256, heads=16, group_sizes=(5, 3)),
    # fast level: D = 512, 16 heads of 32, N = 128, groups of 20 + 20 + 3 (two member tiles, ragged last group)
    dict(dtype="bf16", B=1, C=43, H=64, W=128, p=8, D=512, heads=16, group_sizes=(20, 3)),
    # 32 heads of 32 (two blocks of 16 heads in the head-sum, token-gradient and key-path kernels), D = 1024
    dict(dtype="bf16", B=1, C=12, H=32, W=64, p=8, D=1024, heads=32, group_sizes=(6, 2)),
    # 24 heads: the second head block is half empty
    dict(dtype="bf16", B=1, C=7, H=16, W=32, p=4, D=768, heads=24, group_sizes=(4, 2)),
    # linear first level taken without tokens (its gradients and the tokenizer's from per-channel products with the
    # upstream gradient): 13 channels in groups of 4 (a short last group of one), 16 pixels per patch, N = 64
    dict(dtype="bf16", B=2, C=13, H=32, W=32, p=4, D=256, heads=4, group_sizes=(4, 4), level_kinds=("linear", "attention")),
    # the same route with 64 pixels per patch, N = 128, groups 2 + 2 + 1
    dict(dtype="bf16", B=2, C=5, H=64, W=128, p=8, D=512, heads=8, group_sizes=(2, 3), level_kinds=("linear", "attention")),
    # D = 2048: two blocks of 1024 columns per wavefront in the fused token kernel; groups 4 + 3, N = 6
    dict(dtype="bf16", B=1, C=7, H=16, W=24, p=8, D=2048, heads=16, group_sizes=(4, 2)),
    # 6 heads of 128 (not a multiple of 4 or 8: the head tables of the token kernels are zero-padded), groups 5 + 5 + 1
    dict(dtype="bf16", B=2, C=11, H=16, W=24, p=4, D=768, heads=6, group_sizes=(5, 3)),
    # groups of more than 64 channels (70 + 5): the d-alpha kernel for groups of any size, five member tiles
    dict(dtype="bf16", B=1, C=75, H=16, W=16, p=4, D=256, heads=4, group_sizes=(70, 2)),
    # one flat layer over 75 channels with 20 heads (two head passes of that kernel)
    dict(dtype="bf16", B=1, C=75, H=8, W=16, p=4, D=320, heads=20, group_sizes=(75,)),
]


# ------------------------------------------------------------------------------------------
# forward with the value projection behind the weighted sum
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("kw", SMALL)
def test_forward_folded_matches_oracle(kw):
    cfg = cfg_of(**kw)
    say(f"forward_folded {kw}")
    pr = make_problem(cfg)
    d = cfg.dtype
    out = dchag.dchag_forward_folded(dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d),
                                     [dev_level(lv, d) for lv in pr.levels], cfg.p, cfg.heads)
    torch.cuda.synchronize()
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    err = rel_err(host(out), want)
    say(f"  err={err:.3e}")
    assert err < TOL[d]


@pytest.mark.parametrize("name,per_batch", [("weather", 11), ("hyperspectral", 8), ("hyperspectral_linear", 8),
                                            ("hyperspectral_flat", 6), ("deep", 11), ("wide", 20), ("deep1000", 11)])
def test_forward_folded_full_size_on_sampled_patches(name, per_batch):
    """dchag_forward_folded at the benchmark's sizes and launch configuration, against the oracle on a seeded sample of
    patches; every output row is finite."""
    cfg = get_config(name)
    say(f"forward_folded full-size {name}: generating inputs")
    pr = make_problem(cfg)
    d = cfg.dtype
    out = dchag.dchag_forward_folded(dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d),
                                     [dev_level(lv, d) for lv in pr.levels], cfg.p, cfg.heads)
    torch.cuda.synchronize()
    bs, ns = sample_patches_covering(cfg.B, cfg.N, per_batch, seed=29)      # tile seams and both ends of the patch axis
    say(f"forward_folded full-size {name}: oracle on {bs.size} patches")
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, sample=(bs, ns))
    got = host(out[torch.from_numpy(bs).long().cuda(), torch.from_numpy(ns).long().cuda()])
    err = rel_err(got, want)
    say(f"forward_folded full-size {name}: err={err:.3e}")
    assert err < TOL[d]
    assert torch.isfinite(out.float()).all()


# Shapes whose first level takes its values from the pixels (8 x 8 patches, heads of 64 columns or a multiple).
PIXEL_VALUES = [
    # heads of 64: four heads per 256-column slice, two slices; N = 204 (two patch tiles, the second ragged); groups 4 + 4 + 3
    dict(dtype="bf16", B=2, C=11, H=96, W=136, p=8, D=512, heads=8, group_sizes=(4, 3)),
    # heads of 256: one head per slice; one flat layer over 3 channels
    dict(dtype="bf16", B=1, C=3, H=64, W=64, p=8, D=1024, heads=4, group_sizes=(3,)),
    # heads of 128: two per slice; groups 3 + 3
    dict(dtype="bf16", B=1, C=6, H=32, W=48, p=8, D=512, heads=4, group_sizes=(3, 2)),
    # a last group of one member, three batch elements, N = 45 (one ragged tile): 18 work items, not a multiple of the
    # eight ranges they are dealt to
    dict(dtype="bf16", B=3, C=9, H=40, W=72, p=8, D=256, heads=4, group_sizes=(4, 3)),
    # 4 x 4 patches (the kernel that passes the operands through registers): N = 156 (two tiles, the second ragged),
    # heads of 64, groups 4 + 4 + 1
    dict(dtype="bf16", B=2, C=9, H=48, W=52, p=4, D=512, heads=8, group_sizes=(4, 3)),
    # the same kernel on 8 x 8 patches: heads of 32 (eight per slice), N = 130, groups 5 + 2
    dict(dtype="bf16", B=1, C=7, H=80, W=104, p=8, D=256, heads=8, group_sizes=(5, 2)),
]


@pytest.mark.parametrize("kw", PIXEL_VALUES)
@pytest.mark.parametrize("route", ["folded_into_tokenizer", "ring_shape_1", "fold_by_general_product", "head_sums"])
def test_forward_folded_first_level_values_from_pixels(monkeypatch, kw, route):
    """The first attention level of dchag_forward_folded with the value projection folded into the tokenizer weights
    (one kernel from pixels and softmax weights to the level's pre-projection output; the weight-only fold by its own
    four-channel kernel or by the general product kernel), and, on the same shapes, the route through tokens and
    per-head token averages."""
    if route == "head_sums":
        monkeypatch.setenv("DCHAG_VALUE_UNFOLDED", "1")
    if route == "fold_by_general_product":
        monkeypatch.setenv("DCHAG_FOLD_VALUE_GEMM", "1")
    if route.startswith("ring_shape_"):
        monkeypatch.setenv("DCHAG_RING_SHAPE", route[-1])
    cfg = cfg_of(**kw)
    say(f"forward_folded pixel values {route} {kw}")
    pr = make_problem(cfg)
    d = cfg.dtype
    out = dchag.dchag_forward_folded(dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d),
                                     [dev_level(lv, d) for lv in pr.levels], cfg.p, cfg.heads)
    torch.cuda.synchronize()
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    err = rel_err(host(out), want)
    say(f"  err={err:.3e}")
    assert err < TOL[d]


@pytest.mark.parametrize("drop", ["be", "ce", "both"])
def test_forward_folded_first_level_values_from_pixels_without_token_biases(drop):
    cfg = cfg_of(**PIXEL_VALUES[0])
    say(f"forward_folded pixel values without {drop}")
    pr = make_problem(cfg)
    d = cfg.dtype
    be = None if drop in ("be", "both") else pr.be
    ce = None if drop in ("ce", "both") else pr.ce
    out = dchag.dchag_forward_folded(dev(pr.x, d), dev(pr.We, d), dev(be, d), dev(ce, d),
                                     [dev_level(lv, d) for lv in pr.levels], cfg.p, cfg.heads)
    torch.cuda.synchronize()
    want = oracle.forward(pr.x, pr.We, be, ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    err = rel_err(host(out), want)
    say(f"  err={err:.3e}")
    assert err < TOL[d]


@pytest.mark.parametrize("split", ["1", "3"])
def test_forward_folded_first_level_values_from_pixels_member_split(monkeypatch, split):
    """The members of a group in one workgroup per tile, and dealt to three (partial sums merged by a second kernel);
    by itself the library splits only when the tiles do not fill the chip."""
    monkeypatch.setenv("DCHAG_FIRST_LEVEL_SPLIT", split)
    cfg = cfg_of(**PIXEL_VALUES[0])
    say(f"forward_folded pixel values, members dealt to {split}")
    pr = make_problem(cfg)
    d = cfg.dtype
    out = dchag.dchag_forward_folded(dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d),
                                     [dev_level(lv, d) for lv in pr.levels], cfg.p, cfg.heads)
    torch.cuda.synchronize()
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    err = rel_err(host(out), want)
    say(f"  err={err:.3e}")
    assert err < TOL[d]


@pytest.mark.parametrize("kw", PIXEL_VALUES)
def test_forward_prefolded_equals_forward_folded(kw):
    """Everything that depends on the weights alone prepared once (dchag_fold_value) and two forward calls with it, the
    second on another input: bit for bit the results of dchag_forward_folded, which forms it in every call."""
    cfg = cfg_of(**kw)
    say(f"forward_prefolded {kw}")
    pr = make_problem(cfg)
    d = cfg.dtype
    x, We, be, ce = dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d)
    lv = [dev_level(l, d) for l in pr.levels]
    folded = dchag.dchag_fold_value(We, be, ce, lv, cfg.p, cfg.heads)
    assert folded is not None
    for scale in (1.0, -0.5):
        xs = (x.float() * scale).to(x.dtype)
        got = dchag.dchag_forward_prefolded(xs, We, be, ce, lv, cfg.p, cfg.heads, folded)
        want = dchag.dchag_forward_folded(xs, We, be, ce, lv, cfg.p, cfg.heads)
        torch.cuda.synchronize()
        assert torch.equal(got, want)
    ref = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    got = dchag.dchag_forward_prefolded(x, We, be, ce, lv, cfg.p, cfg.heads, folded)
    assert rel_err(host(got), ref) < TOL[d]


@pytest.mark.parametrize("name", ["hyperspectral", "weather", "hyperspectral_flat", "deep1000"])
def test_forward_prefolded_full_size_equals_forward_folded(name):
    """The same equality at the benchmark's sizes and launch configurations (the folded call itself is checked against
    the oracle on sampled patches above)."""
    cfg = get_config(name)
    say(f"forward_prefolded full-size {name}")
    pr = make_problem(cfg)
    d = cfg.dtype
    x, We, be, ce = dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d)
    lv = [dev_level(l, d) for l in pr.levels]
    folded = dchag.dchag_fold_value(We, be, ce, lv, cfg.p, cfg.heads)
    assert folded is not None
    got = dchag.dchag_forward_prefolded(x, We, be, ce, lv, cfg.p, cfg.heads, folded)
    want = dchag.dchag_forward_folded(x, We, be, ce, lv, cfg.p, cfg.heads)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    assert torch.isfinite(got.float()).all()


def test_forward_prefolded_rejects_shapes_without_a_fold():
    """fp32, and patches of 2 x 2, have no first level taken from the pixels: nothing to prepare, and the prepared
    call says so."""
    for kw in (SMALL[0], SMALL[6]):
        cfg = cfg_of(**kw)
        pr = make_problem(cfg)
        d = cfg.dtype
        x, We, be, ce = dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d)
        lv = [dev_level(l, d) for l in pr.levels]
        assert dchag.dchag_fold_value(We, be, ce, lv, cfg.p, cfg.heads) is None
        dummy = torch.zeros(4096, dtype=torch.uint8, device="cuda")
        with pytest.raises(dchag.DchagError):
            dchag.dchag_forward_prefolded(x, We, be, ce, lv, cfg.p, cfg.heads, dummy)


def test_forward_folded_without_biases_and_sharp_softmax():
    cfg = get_config("tiny")
    pr = make_problem(cfg, biases=False, query_scale=30.0)
    out = dchag.dchag_forward_folded(dev(pr.x, "f32"), dev(pr.We, "f32"), None, dev(pr.ce, "f32"),
                                     [dev_level(lv, "f32") for lv in pr.levels], cfg.p, cfg.heads)
    want = oracle.forward(pr.x, pr.We, None, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    assert rel_err(host(out), want) < TOL["f32"]


# ------------------------------------------------------------------------------------------
# backward
# ------------------------------------------------------------------------------------------
def run_backward(pr, dout_img, want_dx=True):
    """dout_img [B, N, D] float; returns (dx, dWe, dtok_bias, [LevelGrads]) as device tensors."""
    cfg = pr.cfg
    d = cfg.dtype
    tdt = TDT[d]
    lv_dev = [dev_level(lv, d) for lv in pr.levels]
    grads = []
    for lv in lv_dev:
        if lv.kind == 1:
            grads.append(dchag.LevelGrads(dWv=torch.full_like(lv.Wv, 7.0),
                                          dbv=None if lv.bv is None else torch.full_like(lv.bv, 7.0)))
        else:
            kw = {}
            for n in ATT:
                w = getattr(lv, n)
                kw["d" + n] = torch.full_like(w if w is not None else lv.query, 7.0)     # 7: must be overwritten
            grads.append(dchag.LevelGrads(**kw))
    x = dev(pr.x, d)
    dx = torch.full_like(x, 7.0) if want_dx else None
    dWe = torch.full((cfg.C, cfg.D, cfg.p * cfg.p), 7.0, dtype=tdt, device="cuda")
    dtb = torch.full((cfg.C, cfg.D), 7.0, dtype=tdt, device="cuda")
    dchag.dchag_backward(x, dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d), lv_dev, cfg.p, cfg.heads,
                         dev(dout_img, d), grads, dx=dx, dWe=dWe, dtok_bias=dtb)
    torch.cuda.synchronize()
    return dx, dWe, dtb, grads


def image_of_patches(dxp, cfg, bs, ns):
    """[S, C, p*p] patch gradients of the sampled patches -> [B, C, H, W] image (zero elsewhere)."""
    p = cfg.p
    img = np.zeros((cfg.B, cfg.C, cfg.H, cfg.W))
    pw = cfg.W // p
    for i, (b, n) in enumerate(zip(bs, ns)):
        r, c = (n // pw) * p, (n % pw) * p
        img[b, :, r:r + p, c:c + p] = dxp[i].reshape(cfg.C, p, p)
    return img


def compare_grads(cfg, pr, got, want, tol, bs, ns):
    dx, dWe, dtb, grads = got
    errs = {}
    if dx is not None:
        errs["dx"] = rel_err(host(dx), image_of_patches(want["dx"], cfg, bs, ns))
    errs["dWe"] = rel_err(host(dWe), want["dWe"])
    errs["dtok_bias"] = rel_err(host(dtb), want["dtok_bias"])
    for li, lv in enumerate(pr.levels):
        names = ("Wv", "bv") if lv.kind == "linear" else ATT
        for n in names:
            have = host(getattr(grads[li], "d" + n))
            ref = want["levels"][li]["d" + n]
            if n == "bk":
                assert np.abs(have).max() == 0.0                     # the key bias cannot matter
                continue
            errs[f"l{li}.d{n}"] = rel_err(have, ref)
    worst = max(errs, key=errs.get)
    say("  " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))
    assert errs[worst] < tol, (worst, errs[worst])


@pytest.mark.parametrize("kw", SMALL)
def test_backward_matches_oracle(kw):
    cfg = cfg_of(**kw)
    say(f"backward {kw}")
    pr = make_problem(cfg)
    rng = np.random.Generator(np.random.PCG64(41))
    dout = rng.standard_normal((cfg.B, cfg.N, cfg.D)).astype(np.float32)
    if cfg.dtype == "bf16":
        from workloads import round_to_bf16
        dout = round_to_bf16(dout)
    got = run_backward(pr, dout)
    want = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads,
                           dout.reshape(cfg.B * cfg.N, cfg.D).astype(np.float64))
    bs = np.repeat(np.arange(cfg.B), cfg.N)
    ns = np.tile(np.arange(cfg.N), cfg.B)
    compare_grads(cfg, pr, got, want, TOL[cfg.dtype], bs, ns)


@pytest.mark.parametrize("env", ["DCHAG_GENERIC_LEVEL", "DCHAG_GEMM_GENERIC", "DCHAG_DZ_VALU", "DCHAG_COLSUM",
                                 "DCHAG_GEMM_SCALAR_STORES", "DCHAG_TOKENS_UNFUSED", "DCHAG_RPART_VALU",
                                 "DCHAG_PIXEL_SCORES_TWO_KERNELS"])
def test_backward_generic_bf16_kernels_still_match(monkeypatch, env):
    """The shape-generic bf16 kernels (taken for shapes the MFMA and streaming kernels do not tile) on a shape
    the fast kernels would take, forced through the library's debug switches."""
    monkeypatch.setenv(env, "1")
    cfg = cfg_of(dtype="bf16", B=2, C=20, H=32, W=64, p=4, D=256, heads=4, group_sizes=(8, 3))
    pr = make_problem(cfg)
    from workloads import round_to_bf16
    dout = round_to_bf16(np.random.Generator(np.random.PCG64(47)).standard_normal((cfg.B, cfg.N, cfg.D)).astype(np.float32))
    got = run_backward(pr, dout)
    want = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads,
                           dout.reshape(cfg.B * cfg.N, cfg.D).astype(np.float64))
    compare_grads(cfg, pr, got, want, TOL["bf16"], np.repeat(np.arange(cfg.B), cfg.N), np.tile(np.arange(cfg.N), cfg.B))


def test_backward_linear_first_level_through_the_tokens_still_matches(monkeypatch):
    """The route of a linear first level that materialises tokens and token gradients (taken when the intermediates of
    the token-free route do not fit where the tokens would be), forced on a shape the token-free route takes."""
    monkeypatch.setenv("DCHAG_LINEAR_TOKENS", "1")
    cfg = cfg_of(dtype="bf16", B=2, C=13, H=32, W=32, p=4, D=256, heads=4, group_sizes=(4, 4),
                 level_kinds=("linear", "attention"))
    pr = make_problem(cfg)
    from workloads import round_to_bf16
    dout = round_to_bf16(np.random.Generator(np.random.PCG64(48)).standard_normal((cfg.B, cfg.N, cfg.D)).astype(np.float32))
    got = run_backward(pr, dout)
    want = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads,
                           dout.reshape(cfg.B * cfg.N, cfg.D).astype(np.float64))
    compare_grads(cfg, pr, got, want, TOL["bf16"], np.repeat(np.arange(cfg.B), cfg.N), np.tile(np.arange(cfg.N), cfg.B))


@pytest.mark.parametrize("kw", [SMALL[0], SMALL[3], SMALL[4], SMALL[10], SMALL[13]])
def test_forward_keep_and_backward_kept_equal_the_recomputing_calls(monkeypatch, kw):
    """A training step that keeps its activations: the output equals dchag_forward_folded's (on its route through the
    tokens at the first level, which the kept forward always takes) and every gradient equals dchag_backward's bit for
    bit (same kernels on the same buffers), for two upstream gradients in a row after one forward."""
    cfg = cfg_of(**kw)
    say(f"keep / kept {kw}")
    pr = make_problem(cfg)
    d = cfg.dtype
    x, We, be, ce = dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d)
    lv_dev = [dev_level(lv, d) for lv in pr.levels]
    dt = dchag.DCHAG_F32 if d == "f32" else dchag.DCHAG_BF16
    wsb = dchag.dchag_workspace_bytes(dt, cfg.B, cfg.C, cfg.H, cfg.W, cfg.p, cfg.D, cfg.heads, list(cfg.group_sizes), 3)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    out = dchag.dchag_forward_keep(x, We, be, ce, lv_dev, cfg.p, cfg.heads, ws)
    monkeypatch.setenv("DCHAG_VALUE_UNFOLDED", "1")
    ref = dchag.dchag_forward_folded(x, We, be, ce, lv_dev, cfg.p, cfg.heads)
    torch.cuda.synchronize()
    monkeypatch.delenv("DCHAG_VALUE_UNFOLDED")
    assert torch.equal(out, ref)
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    assert rel_err(host(out), want) < TOL[d]
    for seed in (51, 52):
        dout = np.random.Generator(np.random.PCG64(seed)).standard_normal((cfg.B, cfg.N, cfg.D)).astype(np.float32)
        a = run_backward(pr, dout)                                    # recomputes the forward
        grads = []
        for lv in lv_dev:
            if lv.kind == 1:
                grads.append(dchag.LevelGrads(dWv=torch.full_like(lv.Wv, 7.0), dbv=torch.full_like(lv.bv, 7.0)))
            else:
                grads.append(dchag.LevelGrads(**{"d" + n: torch.full_like(getattr(lv, n), 7.0) for n in ATT}))
        dx, dWe, dtb = torch.full_like(x, 7.0), torch.full_like(We, 7.0), torch.full_like(ce, 7.0)
        dchag.dchag_backward(x, We, be, ce, lv_dev, cfg.p, cfg.heads, dev(dout, d), grads, dx=dx, dWe=dWe, dtok_bias=dtb,
                             workspace=ws, kept=True)
        torch.cuda.synchronize()
        assert torch.equal(dx, a[0]) and torch.equal(dWe, a[1]) and torch.equal(dtb, a[2])
        for g, h in zip(grads, a[3]):
            for n in ("dquery", "dWq", "dWk", "dWv", "dWo", "dbq", "dbk", "dbv", "dbo"):
                if getattr(g, n) is not None:
                    assert torch.equal(getattr(g, n), getattr(h, n)), n


def test_backward_skips_gradients_that_are_not_asked_for():
    cfg = cfg_of(dtype="f32", B=1, C=6, H=8, W=8, p=2, D=32, heads=4, group_sizes=(3, 2))
    pr = make_problem(cfg)
    d = "f32"
    dout = np.random.Generator(np.random.PCG64(5)).standard_normal((cfg.B, cfg.N, cfg.D)).astype(np.float32)
    lv_dev = [dev_level(lv, d) for lv in pr.levels]
    grads = [dchag.LevelGrads(dWv=torch.zeros_like(lv.Wv)) for lv in lv_dev]
    dchag.dchag_backward(dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d), lv_dev, cfg.p, cfg.heads,
                         dev(dout, d), grads)
    torch.cuda.synchronize()
    want = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads,
                           dout.reshape(-1, cfg.D).astype(np.float64), want_dx=False)
    for li in range(2):
        assert rel_err(host(grads[li].dWv), want["levels"][li]["dWv"]) < TOL[d]


def test_backward_is_deterministic():
    cfg = cfg_of(dtype="bf16", B=2, C=20, H=16, W=24, p=4, D=256, heads=4, group_sizes=(8, 3))
    pr = make_problem(cfg)
    dout = np.random.Generator(np.random.PCG64(6)).standard_normal((cfg.B, cfg.N, cfg.D)).astype(np.float32)
    a = run_backward(pr, dout)
    b = run_backward(pr, dout)
    assert torch.equal(a[1], b[1]) and torch.equal(a[0], b[0])
    assert torch.equal(a[3][0].dWk, b[3][0].dWk) and torch.equal(a[3][1].dWv, b[3][1].dWv)


# 250 patches in tiles of 16 (the last tile holds 10), 250 channels in groups of 32 (the last holds 26), and enough
# blocks that the token-gradient kernels keep 16 patches per block as they do at the benchmark's sizes
RAGGED_TILES = dict(dtype="bf16", B=4, C=250, H=40, W=100, p=4, D=256, heads=8, group_sizes=(32, 8))


@pytest.mark.parametrize("name,per_batch", [("weather", 6), ("hyperspectral", 4), ("ragged_tiles", 12), ("deep", 4),
                                            ("wide", 6), ("hyperspectral_linear", 4), ("hyperspectral_flat", 3)])
def test_backward_full_size_with_upstream_gradient_on_sampled_patches(name, per_batch):
    """Full-size configurations in the launch configuration of the benchmark.  The upstream gradient is
    non-zero on a seeded sample of patches only; the path is independent per patch, so every other patch
    contributes exactly nothing and the oracle only has to visit the sample."""
    cfg = cfg_of(**RAGGED_TILES) if name == "ragged_tiles" else get_config(name)
    say(f"backward full-size {name}: generating inputs")
    pr = make_problem(cfg)
    bs, ns = sample_patches_covering(cfg.B, cfg.N, per_batch, seed=19)      # tile seams and both ends of the patch axis
    rng = np.random.Generator(np.random.PCG64(43))
    from workloads import round_to_bf16
    ds = round_to_bf16(rng.standard_normal((bs.size, cfg.D)).astype(np.float32))
    dout = np.zeros((cfg.B, cfg.N, cfg.D), dtype=np.float32)
    dout[bs, ns] = ds
    say(f"backward full-size {name}: GPU")
    got = run_backward(pr, dout)
    say(f"backward full-size {name}: oracle on {bs.size} patches")
    want = oracle.backward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, ds.astype(np.float64),
                           sample=(bs, ns))
    compare_grads(cfg, pr, got, want, TOL[cfg.dtype], bs, ns)


@pytest.mark.parametrize("name", ["weather", "wide", "deep", "deep1000", "hyperspectral_linear", "hyperspectral_flat"])
def test_backward_full_size_identities_with_a_dense_upstream_gradient(name):
    """Properties that hold at any size, with a dense upstream gradient, on every benchmark configuration:
    the last level's output-bias gradient is the plain sum of dout over all patches; the value-bias gradient
    of every attention level is Wo^T times its output-bias gradient (softmax weights sum to one, so bv
    reaches the output as Wo bv); the key-bias gradient is zero; everything is finite."""
    cfg = get_config(name)
    say(f"backward identities {name}: generating inputs")
    pr = make_problem(cfg)
    rng = np.random.Generator(np.random.PCG64(44))
    dout = rng.standard_normal((cfg.B, cfg.N, cfg.D)).astype(np.float32)
    say(f"backward identities {name}: GPU")
    got = run_backward(pr, dout, want_dx=False)
    from workloads import round_to_bf16
    want = round_to_bf16(dout).astype(np.float64).sum(axis=(0, 1))
    assert rel_err(host(got[3][-1].dbo)[0], want) < TOL["bf16"]
    for li, (lv, g) in enumerate(zip(pr.levels, got[3])):
        if lv.kind == "linear":
            assert torch.isfinite(g.dWv.float()).all() and torch.isfinite(g.dbv.float()).all()
            continue
        for n in ("dWq", "dWk", "dWv", "dWo", "dquery", "dbq", "dbv", "dbo"):
            assert torch.isfinite(getattr(g, n).float()).all(), (li, n)
        assert float(g.dbk.float().abs().max()) == 0.0
        Wo = torch.from_numpy(lv.Wo).to("cuda", torch.float64)
        ref = torch.einsum("kij,ki->kj", Wo, g.dbo.to(torch.float64))
        err = float((g.dbv.to(torch.float64) - ref).abs().max() / ref.abs().max())
        say(f"  level {li}: |dbv - Wo^T dbo| / max = {err:.2e}")
        assert err < TOL["bf16"]
    assert torch.isfinite(got[1].float()).all() and torch.isfinite(got[2].float()).all()
