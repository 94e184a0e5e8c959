"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs.

Error measure (the target gives only a number): for an output tensor y and the oracle's y^,
    err = max_i |y_i - y^_i| / max_i |y^_i|
must stay below 2e-2 for bf16 (bf16 storage, fp32 accumulation) and 1e-4 for fp32.  The full-size tests also print,
beside that gated figure, the element-wise error max_i |y_i - y^_i| / max(|y^_i|, rms y^) and the rms error
rms(y - y^) / rms(y^) (an element-wise relative error is unbounded where y^ is near zero, hence the rms floor).
"""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2506_21411_amd as dchag
from workloads import ShapeCfg, get_config, make_problem, make_tokens, n_groups, sample_patches
from workloads import sample_patches_covering
from workloads import make_level, make_linear_level

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev(a, dtype):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(TDT[dtype]).contiguous()


def dev_level(lv, dtype):
    return dchag.LevelWeights(lv.group_size, dev(lv.query, dtype), dev(lv.Wq, dtype), dev(lv.Wk, dtype),
                              dev(lv.Wv, dtype), dev(lv.Wo, dtype), dev(lv.bq, dtype), dev(lv.bk, dtype),
                              dev(lv.bv, dtype), dev(lv.bo, dtype), kind=1 if lv.kind == "linear" else 0)


def rel_err(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape
    assert np.isfinite(got).all()
    return float(np.abs(got - want).max() / np.abs(want).max())


def err_figures(got, want):
    """(max-normalised error: the gated one, element-wise error with an rms floor, rms error), see the module docstring."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    d = np.abs(got - want)
    rms = float(np.sqrt(np.mean(np.square(want))))
    return (float(d.max() / np.abs(want).max()), float((d / np.maximum(np.abs(want), rms)).max()),
            float(np.sqrt(np.mean(np.square(d))) / rms))


def host(t):
    return t.detach().to(torch.float64).cpu().numpy()


def run_forward(pr):
    cfg = pr.cfg
    d = cfg.dtype
    out = dchag.dchag_forward(dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d),
                              [dev_level(lv, d) for lv in pr.levels], cfg.p, cfg.heads)
    torch.cuda.synchronize()
    return out


def cfg_of(**kw):
    base = dict(name="t", dtype="f32", B=2, C=6, H=8, W=12, p=2, D=32, heads=4, group_sizes=(3, 2),
                x_kind="gauss_mu_sigma", seed=3)
    base.update(kw)
    return ShapeCfg(**base)


# ------------------------------------------------------------------------------------------
# tokenizer
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kw", [
    dict(B=2, C=5, H=8, W=12, p=2, D=40),                # N = 24: one full 16-patch tile and a ragged tail
    dict(B=1, C=3, H=20, W=28, p=4, D=256),              # N = 35
    dict(B=1, C=2, H=8, W=8, p=8, D=64),                 # N = 1
    dict(B=3, C=1, H=3, W=5, p=1, D=8),                  # 1x1 patches, one channel
    dict(B=2, C=3, H=48, W=52, p=4, D=320),              # MFMA tokenizer: N = 156 (two 128-patch tiles), 5 slices
    dict(B=1, C=2, H=80, W=136, p=8, D=1024),            # MFMA tokenizer: 8x8 patches, N = 170
    dict(B=1, C=2, H=32, W=48, p=16, D=128),             # 16x16 patches (k = 256), N = 6
    dict(B=2, C=2, H=48, W=52, p=4, D=512),              # two tiles, eight 64-column slices, N = 156
    dict(B=1, C=1, H=32, W=32, p=16, D=256),             # 16x16 patches with D = 256
])
def test_tokenize_matches_oracle(dtype, kw):
    cfg = cfg_of(dtype=dtype, heads=1, group_sizes=(kw["C"],), **kw)
    say(f"tokenize {dtype} {kw}")
    pr = make_problem(cfg)
    t = dchag.dchag_tokenize(dev(pr.x, dtype), dev(pr.We, dtype), dev(pr.be, dtype), dev(pr.ce, dtype), cfg.p)
    torch.cuda.synchronize()
    want = oracle.tokenize(pr.x, pr.We, pr.be, pr.ce, cfg.p).reshape(cfg.B, cfg.N, cfg.C, cfg.D).transpose(0, 2, 1, 3)
    assert rel_err(host(t), want) < TOL[dtype]


def test_tokenize_without_bias_and_embedding():
    cfg = cfg_of(B=1, C=3, H=8, W=8, p=4, D=16, heads=1, group_sizes=(3,))
    pr = make_problem(cfg)
    t = dchag.dchag_tokenize(dev(pr.x, "f32"), dev(pr.We, "f32"), None, None, cfg.p)
    want = oracle.tokenize(pr.x, pr.We, None, None, cfg.p).reshape(cfg.B, cfg.N, cfg.C, cfg.D).transpose(0, 2, 1, 3)
    assert rel_err(host(t), want) < 1e-5


# ------------------------------------------------------------------------------------------
# one aggregation level
# ------------------------------------------------------------------------------------------
LEVEL_CASES = [
    # dtype, B, Cin, N, D, heads, g
    ("f32", 2, 6, 10, 32, 4, 3),
    ("f32", 1, 7, 5, 24, 3, 3),          # uneven last group (3,3,1), D not a multiple of 64
    ("f32", 1, 4, 3, 16, 2, 1),          # groups of one
    ("f32", 1, 5, 1, 8, 1, 9),           # one short group, one patch, one head
    ("bf16", 2, 8, 24, 64, 4, 4),        # bf16 on the generic projection kernel (D % 256 != 0)
    ("bf16", 2, 12, 40, 256, 4, 8),      # MFMA projection: rows 320 and 160 per block -> ragged tiles
    ("bf16", 1, 33, 19, 512, 8, 16),     # MFMA, uneven last group of 1, rows 304 / 19
    ("bf16", 1, 70, 9, 256, 2, 70),      # one flat group of 70, head dim 128
    ("bf16", 1, 10, 50, 256, 8, 5),      # head dim 32: 8 heads per 256-column slice; N = 50 (pitch 64)
    ("bf16", 2, 6, 33, 512, 2, 3),       # head dim 256: one head per slice
    ("bf16", 1, 5, 20, 1024, 2, 5),      # head dim 512: a head spans two slices
    ("bf16", 1, 9, 17, 1024, 32, 9),     # 32 heads (two head blocks in the score kernel), 2 chunks of 8
]


@pytest.mark.parametrize("dtype,B,Cin,N,D,heads,g", LEVEL_CASES)
@pytest.mark.parametrize("biases", [True, False])
def test_aggregate_level_matches_oracle(dtype, B, Cin, N, D, heads, g, biases):
    say(f"aggregate_level {dtype} B={B} Cin={Cin} N={N} D={D} h={heads} g={g} biases={biases}")
    rng = np.random.Generator(np.random.PCG64(100 + Cin))
    lv = make_level(rng, n_groups(Cin, g), g, D, dtype, biases)
    z = make_tokens(B, Cin, N, D, dtype, seed=7)
    y = dchag.dchag_aggregate_level(dev(z, dtype), dev_level(lv, dtype), heads)
    torch.cuda.synchronize()
    zo = z.transpose(0, 2, 1, 3).reshape(B * N, Cin, D)
    want = oracle.aggregate_level(zo, lv, heads).reshape(B, N, -1, D).transpose(0, 2, 1, 3)
    err = rel_err(host(y), want)
    say(f"  err={err:.3e}")
    assert err < TOL[dtype]


@pytest.mark.parametrize("route", ["two_kernels", "one_kernel"])
@pytest.mark.parametrize("B,Cin,N,D,heads,g", [
    (2, 12, 40, 256, 4, 8),        # N = 40: second 32-patch tile holds 8 patches (pitch 64); short last group of 4
    (1, 33, 19, 512, 8, 16),       # last group of one member; fewer members than wavefronts in it
    (1, 70, 9, 256, 2, 70),        # one group of 70: wavefronts take 9 or 8 members each
    (1, 10, 50, 512, 16, 5),       # 16 heads: every key row of the 16-row fragment is a real head
    (1, 5, 20, 1024, 2, 5),        # D = 1024: 32 steps per token row
    (1, 9, 17, 1024, 32, 9),       # 32 heads: two head blocks; N = 17 (one full 16-patch tile and one patch)
    (2, 16, 48, 512, 8, 16),       # N = 48: the last 16-patch tile is full and the pitch (64) reaches beyond it
])
def test_aggregate_level_score_kernels(monkeypatch, route, B, Cin, N, D, heads, g):
    """The score routes of the bf16 MFMA path on the same small shapes: raw scores then a softmax kernel, and scores and
    softmax in one kernel over 32 patches and all members (taken by itself only on large inputs).  A route that does not
    tile a shape falls back to the two-kernel route."""
    monkeypatch.setenv("DCHAG_SCORES_ONE_KERNEL", "1" if route == "one_kernel" else "0")
    say(f"score route {route} B={B} Cin={Cin} N={N} D={D} h={heads} g={g}")
    rng = np.random.Generator(np.random.PCG64(400 + Cin))
    lv = make_level(rng, n_groups(Cin, g), g, D, "bf16", True)
    z = make_tokens(B, Cin, N, D, "bf16", seed=11)
    y = dchag.dchag_aggregate_level(dev(z, "bf16"), dev_level(lv, "bf16"), heads)
    torch.cuda.synchronize()
    want = oracle.aggregate_level(z.transpose(0, 2, 1, 3).reshape(B * N, Cin, D), lv, heads)
    err = rel_err(host(y), want.reshape(B, N, -1, D).transpose(0, 2, 1, 3))
    say(f"  err={err:.3e}")
    assert err < TOL["bf16"]


@pytest.mark.parametrize("regs", [False, True])
def test_aggregate_level_output_projection_of_few_tiles(monkeypatch, regs):
    """The output projection of a level with few tiles: the four-stage kernel that loads three slices ahead (taken by
    itself) and the register-staged one behind DCHAG_LINEAR_SMALL_REGS; 3 groups of 100 rows per batch item (a ragged 128-row
    tile each), D = 512 (eight slices, so the four stages wrap around twice), and a level of a single 16-row group."""
    if regs:
        monkeypatch.setenv("DCHAG_LINEAR_SMALL_REGS", "1")
    for (B, Cin, N, D, heads, g) in ((2, 9, 100, 512, 8, 3), (1, 4, 16, 256, 4, 4)):
        rng = np.random.Generator(np.random.PCG64(500 + Cin))
        lv = make_level(rng, n_groups(Cin, g), g, D, "bf16", True)
        z = make_tokens(B, Cin, N, D, "bf16", seed=21)
        y = dchag.dchag_aggregate_level(dev(z, "bf16"), dev_level(lv, "bf16"), heads)
        torch.cuda.synchronize()
        want = oracle.aggregate_level(z.transpose(0, 2, 1, 3).reshape(B * N, Cin, D), lv, heads)
        err = rel_err(host(y), want.reshape(B, N, -1, D).transpose(0, 2, 1, 3))
        say(f"few-tile output projection regs={regs} B={B} Cin={Cin} N={N} D={D}: err={err:.3e}")
        assert err < TOL["bf16"]


@pytest.mark.parametrize("Cin", [24, 48])
def test_aggregate_level_large_enough_for_the_one_kernel_score_route(Cin):
    """A level big enough that the library picks the one-kernel score route by itself (at least one
    32-patch block per compute unit), ragged in N, checked on sampled patches (tile seams among them); three and six groups."""
    B, N, D, heads, g = 2, 1500, 256, 4, 8
    rng = np.random.Generator(np.random.PCG64(77))
    lv = make_level(rng, n_groups(Cin, g), g, D, "bf16", True)
    z = make_tokens(B, Cin, N, D, "bf16", seed=12)
    y = dchag.dchag_aggregate_level(dev(z, "bf16"), dev_level(lv, "bf16"), heads)
    torch.cuda.synchronize()
    ns = np.array([0, 1, 31, 32, 33, 63, 64, 700, 1439, 1440, 1471, 1472, 1498, 1499])
    zo = z[:, :, ns, :].transpose(0, 2, 1, 3).reshape(B * ns.size, Cin, D)
    want = oracle.aggregate_level(zo, lv, heads).reshape(B, ns.size, -1, D).transpose(0, 2, 1, 3)
    err = rel_err(host(y)[:, :, ns, :], want)
    say(f"one-kernel route at scale: err={err:.3e}")
    assert err < TOL["bf16"]
    assert torch.isfinite(y.float()).all()


@pytest.mark.parametrize("split", ["1", "2", "4", "8"])
def test_aggregate_level_value_gemm_dealt_to_several_items(monkeypatch, split):
    """The value GEMM with a group's chunks of 8 channels dealt to 1, 2, 4 items (8 is cut back to 4: a group of 43
    has 6 chunks), partial sums merged by a second kernel: two groups of 43 channels, 40 patches (a ragged patch tile)."""
    monkeypatch.setenv("DCHAG_VAGG_SPLIT", split)
    B, Cin, N, D, heads, g = 2, 86, 40, 256, 4, 43
    rng = np.random.Generator(np.random.PCG64(431))
    lv = make_level(rng, n_groups(Cin, g), g, D, "bf16", True)
    z = make_tokens(B, Cin, N, D, "bf16", seed=13)
    y = dchag.dchag_aggregate_level(dev(z, "bf16"), dev_level(lv, "bf16"), heads)
    torch.cuda.synchronize()
    want = oracle.aggregate_level(z.transpose(0, 2, 1, 3).reshape(B * N, Cin, D), lv, heads)
    err = rel_err(host(y), want.reshape(B, N, -1, D).transpose(0, 2, 1, 3))
    say(f"value GEMM dealt to {split} items: err={err:.3e}")
    assert err < TOL["bf16"]


def test_aggregate_level_generic_bf16_kernels_still_match(monkeypatch):
    """The shape-generic bf16 kernels (taken for shapes the MFMA path does not tile) on a shape
    the MFMA path would take, forced through the library's DCHAG_GENERIC_LEVEL switch."""
    monkeypatch.setenv("DCHAG_GENERIC_LEVEL", "1")
    dtype, B, Cin, N, D, heads, g = "bf16", 2, 12, 40, 256, 4, 8
    rng = np.random.Generator(np.random.PCG64(5))
    lv = make_level(rng, n_groups(Cin, g), g, D, dtype, True)
    z = make_tokens(B, Cin, N, D, dtype, seed=8)
    y = dchag.dchag_aggregate_level(dev(z, dtype), dev_level(lv, dtype), heads)
    torch.cuda.synchronize()
    want = oracle.aggregate_level(z.transpose(0, 2, 1, 3).reshape(B * N, Cin, D), lv, heads)
    assert rel_err(host(y), want.reshape(B, N, -1, D).transpose(0, 2, 1, 3)) < TOL[dtype]


# ------------------------------------------------------------------------------------------
# linear partial-aggregation level (D-CHAG-L)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,B,Cin,N,D,g", [
    ("f32", 2, 6, 10, 32, 3),
    ("f32", 1, 7, 5, 24, 3),             # uneven last group (3,3,1); D / 4 = 6 vectors per row
    ("f32", 1, 4, 3, 16, 1),             # groups of one: a per-feature scale and shift
    ("bf16", 2, 12, 40, 256, 8),         # short last group of 4
    ("bf16", 1, 33, 19, 72, 16),         # D = 9 vectors of 8; last group of one
    ("bf16", 1, 70, 300, 1024, 70),      # one flat group; several blocks per (b, k)
])
@pytest.mark.parametrize("biases", [True, False])
def test_linear_level_matches_oracle(dtype, B, Cin, N, D, g, biases):
    say(f"linear level {dtype} B={B} Cin={Cin} N={N} D={D} g={g} biases={biases}")
    rng = np.random.Generator(np.random.PCG64(300 + Cin))
    lv = make_linear_level(rng, n_groups(Cin, g), g, D, dtype, biases)
    z = make_tokens(B, Cin, N, D, dtype, seed=9)
    y = dchag.dchag_aggregate_level(dev(z, dtype), dev_level(lv, dtype), heads=1)
    torch.cuda.synchronize()
    zo = z.transpose(0, 2, 1, 3).reshape(B * N, Cin, D)
    want = oracle.aggregate_level(zo, lv, 1).reshape(B, N, -1, D).transpose(0, 2, 1, 3)
    err = rel_err(host(y), want)
    say(f"  err={err:.3e}")
    assert err < TOL[dtype]


@pytest.mark.parametrize("kw", [
    dict(dtype="f32", B=2, C=7, H=8, W=12, p=2, D=32, heads=4, group_sizes=(3, 3), level_kinds=("linear", "attention")),
    dict(dtype="f32", B=1, C=9, H=8, W=8, p=2, D=16, heads=2, group_sizes=(2, 3, 2),
         level_kinds=("linear", "linear", "attention")),                                    # 9 -> 5 -> 2 -> 1
    # bf16, D % 256 == 0 and p*p % 16 == 0: tokenizer fused with the linear first level; groups 8, 8, 4;
    # N = 24 patches (one ragged 64-patch tile)
    dict(dtype="bf16", B=2, C=20, H=16, W=24, p=4, D=256, heads=4, group_sizes=(8, 3),
         level_kinds=("linear", "attention")),
    # fused, p = 8, N = 150 (three 64-patch tiles, the last ragged), two 256-column slices, groups 4, 4, 1
    dict(dtype="bf16", B=1, C=9, H=80, W=120, p=8, D=512, heads=8, group_sizes=(4, 3),
         level_kinds=("linear", "attention")),
    # fused first level followed by a second linear level and the attention top
    dict(dtype="bf16", B=1, C=12, H=16, W=16, p=4, D=256, heads=2, group_sizes=(3, 2, 2),
         level_kinds=("linear", "linear", "attention")),
    # bf16 shape the fused kernel does not take (D = 64): tokenizer, then the mixing kernel
    dict(dtype="bf16", B=1, C=6, H=8, W=8, p=2, D=64, heads=2, group_sizes=(2, 3),
         level_kinds=("linear", "attention")),
])
def test_forward_with_linear_levels_matches_oracle(kw):
    cfg = cfg_of(**kw)
    say(f"forward with linear levels {kw}")
    pr = make_problem(cfg)
    out = run_forward(pr)
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    err = rel_err(host(out), want)
    say(f"  err={err:.3e}")
    assert err < TOL[cfg.dtype]


def test_forward_linear_fused_and_unfused_agree(monkeypatch):
    """The fused tokenizer + linear level against the two-kernel route on the same inputs: equal up to the
    bf16 rounding of the per-channel tokens, which only the two-kernel route stores."""
    cfg = cfg_of(dtype="bf16", B=1, C=20, H=32, W=32, p=4, D=256, heads=4, group_sizes=(8, 3),
                 level_kinds=("linear", "attention"))
    pr = make_problem(cfg, biases=False)
    a = run_forward(pr)
    monkeypatch.setenv("DCHAG_GENERIC_TOKENIZE", "1")
    b = run_forward(pr)
    assert rel_err(host(a), host(b)) < TOL["bf16"]


def test_forward_rejects_linear_last_level():
    cfg = cfg_of(dtype="f32", C=6, group_sizes=(3, 2), level_kinds=("linear", "attention"))
    pr = make_problem(cfg)
    lvls = [dev_level(lv, "f32") for lv in pr.levels]
    lvls[1] = dchag.LevelWeights(2, None, None, None, torch.zeros(1, 2, cfg.D, device="cuda"), None, kind=1)
    with pytest.raises(dchag.DchagError) as e:
        dchag.dchag_forward(dev(pr.x, "f32"), dev(pr.We, "f32"), dev(pr.be, "f32"), dev(pr.ce, "f32"), lvls,
                            cfg.p, cfg.heads)
    assert e.value.status == -2


# ------------------------------------------------------------------------------------------
# whole path
# ------------------------------------------------------------------------------------------
def test_forward_tiny_config_fp32_full():
    cfg = get_config("tiny")
    pr = make_problem(cfg)
    out = run_forward(pr)
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    err = rel_err(host(out), want)
    say(f"tiny fp32 err={err:.3e}")
    assert err < TOL["f32"]


def test_forward_tiny_sharp_softmax_fp32():
    """Queries scaled by 30: near one-hot softmax weights and large scores."""
    cfg = get_config("tiny")
    pr = make_problem(cfg, query_scale=30.0)
    out = run_forward(pr)
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    err = rel_err(host(out), want)
    say(f"tiny sharp fp32 err={err:.3e}")
    assert err < TOL["f32"]


@pytest.mark.parametrize("kw", [
    dict(dtype="f32", B=2, C=7, H=8, W=12, p=2, D=32, heads=4, group_sizes=(3, 2, 2)),      # 7 -> 3 -> 2 -> 1
    dict(dtype="f32", B=1, C=5, H=4, W=4, p=2, D=16, heads=2, group_sizes=(5,)),            # flat single layer
    dict(dtype="bf16", B=2, C=20, H=16, W=24, p=4, D=256, heads=4, group_sizes=(8, 3)),     # groups 8, 8, 4
    dict(dtype="bf16", B=1, C=9, H=24, W=40, p=8, D=512, heads=8, group_sizes=(4, 3)),      # groups 4, 4, 1
    dict(dtype="bf16", B=1, C=6, H=8, W=8, p=2, D=64, heads=2, group_sizes=(2, 2, 2)),      # generic bf16 path
])
def test_forward_matches_oracle_small(kw):
    cfg = cfg_of(**kw)
    say(f"forward small {kw}")
    pr = make_problem(cfg)
    out = run_forward(pr)
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    err = rel_err(host(out), want)
    say(f"  err={err:.3e}")
    assert err < TOL[cfg.dtype]


@pytest.mark.parametrize("two", [False, True])
def test_forward_pixel_score_routes(monkeypatch, two):
    """Level-1 scores from the pixels with the softmax in the same kernel (default) and as two kernels."""
    if two:
        monkeypatch.setenv("DCHAG_PIXEL_SCORES_TWO_KERNELS", "1")
    for kw in (dict(dtype="bf16", B=2, C=20, H=16, W=24, p=4, D=256, heads=4, group_sizes=(8, 3)),
               dict(dtype="bf16", B=1, C=11, H=40, W=72, p=8, D=512, heads=16, group_sizes=(4, 3))):   # N = 45: ragged tile
        cfg = cfg_of(**kw)
        pr = make_problem(cfg)
        out = run_forward(pr)
        want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
        err = rel_err(host(out), want)
        say(f"pixel scores two_kernels={two} {kw}: err={err:.3e}")
        assert err < TOL[cfg.dtype]


@pytest.mark.parametrize("kw", [
    dict(dtype="bf16", B=2, C=20, H=16, W=24, p=4, D=256, heads=4, group_sizes=(8, 3)),     # 16 pixels: 8 channels per block
    dict(dtype="bf16", B=1, C=9, H=24, W=40, p=8, D=512, heads=8, group_sizes=(4, 3)),      # 64 pixels: 2 channels per block
    dict(dtype="bf16", B=1, C=6, H=16, W=32, p=8, D=768, heads=24, group_sizes=(3, 2)),     # odd groups: only the vector-ALU form
])
@pytest.mark.parametrize("valu", [False, True])
def test_forward_score_weight_composition_kernels(monkeypatch, kw, valu):
    """The level-1 scores come from the pixels through composed weights; both kernels that compose them (MFMA, and the
    vector-ALU one that shapes the MFMA form does not tile fall back to) against the oracle."""
    if valu:
        monkeypatch.setenv("DCHAG_COMPOSE_VALU", "1")
    cfg = cfg_of(**kw)
    pr = make_problem(cfg)
    out = run_forward(pr)
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads).reshape(cfg.B, cfg.N, cfg.D)
    err = rel_err(host(out), want)
    say(f"compose valu={valu} {kw}: err={err:.3e}")
    assert err < TOL[cfg.dtype]


def test_forward_is_deterministic():
    cfg = cfg_of(dtype="bf16", B=2, C=20, H=16, W=24, p=4, D=256, heads=4, group_sizes=(8, 3))
    pr = make_problem(cfg)
    a = run_forward(pr)
    b = run_forward(pr)
    assert torch.equal(a, b)


@pytest.mark.parametrize("kw", [
    dict(dtype="f32", B=2, C=7, H=8, W=12, p=2, D=32, heads=4, group_sizes=(3, 2, 2)),      # generic projection
    dict(dtype="bf16", B=2, C=20, H=16, W=24, p=4, D=256, heads=4, group_sizes=(8, 3)),     # 128 x 128 MFMA tiles
    dict(dtype="bf16", B=1, C=6, H=8, W=8, p=2, D=64, heads=2, group_sizes=(2, 2, 2)),      # generic bf16 path
    dict(dtype="bf16", B=3, C=4, H=160, W=192, p=8, D=256, heads=4, group_sizes=(4,)),      # N = 480: 256 x 256 tiles, ragged
])
def test_forward_with_positional_embedding_matches_oracle(kw):
    cfg = cfg_of(**kw)
    say(f"forward + positional embedding {kw}")
    pr = make_problem(cfg)
    d = cfg.dtype
    pos = np.random.Generator(np.random.PCG64(31)).standard_normal((cfg.N, cfg.D)).astype(np.float32)
    if d == "bf16":
        from workloads import round_to_bf16
        pos = round_to_bf16(pos)
    out = dchag.dchag_forward_pos(dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d),
                                  [dev_level(lv, d) for lv in pr.levels], cfg.p, cfg.heads, dev(pos, d))
    torch.cuda.synchronize()
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, pos=pos).reshape(cfg.B, cfg.N, cfg.D)
    err = rel_err(host(out), want)
    say(f"  err={err:.3e}")
    assert err < TOL[d]


def test_forward_with_positional_embedding_full_size():
    cfg = get_config("hyperspectral")
    pr = make_problem(cfg)
    from workloads import round_to_bf16
    pos = round_to_bf16(np.random.Generator(np.random.PCG64(32)).standard_normal((cfg.N, cfg.D)).astype(np.float32))
    d = "bf16"
    out = dchag.dchag_forward_pos(dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d),
                                  [dev_level(lv, d) for lv in pr.levels], cfg.p, cfg.heads, dev(pos, d))
    torch.cuda.synchronize()
    bs, ns = sample_patches(cfg.B, cfg.N, 4, seed=18)
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, sample=(bs, ns), pos=pos)
    got = host(out[torch.from_numpy(bs).long().cuda(), torch.from_numpy(ns).long().cuda()])
    err = rel_err(got, want)
    say(f"full-size positional: err={err:.3e}")
    assert err < TOL["bf16"]


def test_forward_can_be_captured_in_a_graph_and_replayed():
    """dchag_forward allocates nothing and synchronises nothing, so a caller may capture it in a HIP graph.
    Every replay, with eager work and synchronisations in between, must reproduce the eager result bit for bit."""
    cfg = cfg_of(dtype="bf16", B=2, C=20, H=32, W=48, p=4, D=256, heads=4, group_sizes=(8, 3))
    pr = make_problem(cfg)
    d = "bf16"
    x, We, be, ce = dev(pr.x, d), dev(pr.We, d), dev(pr.be, d), dev(pr.ce, d)
    levels = [dev_level(lv, d) for lv in pr.levels]
    wsb = dchag.dchag_workspace_bytes(dchag.DCHAG_BF16, cfg.B, cfg.C, cfg.H, cfg.W, cfg.p, cfg.D, cfg.heads,
                                      list(cfg.group_sizes), 1)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    out = torch.empty((cfg.B, cfg.N, cfg.D), dtype=torch.bfloat16, device="cuda")

    def step():
        dchag.dchag_forward(x, We, be, ce, levels, cfg.p, cfg.heads, out=out, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                            # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager = out.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, capture_error_mode="relaxed"):
        step()
    for rep in range(3):
        out.zero_()
        ws.random_(0, 255)                                # the workspace holds nothing a replay depends on
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager result"
        step()                                            # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(out, eager)


FLAT1024 = ShapeCfg("flat1024", "bf16", 4, 1024, 128, 128, 8, 1024, 16, (1024,), "ar1", 2)


@pytest.mark.parametrize("name,per_batch", [("weather", 22), ("hyperspectral", 14), ("wide", 40), ("deep", 22),
                                            ("deep1000", 22), ("hyperspectral_linear", 14),
                                            ("hyperspectral_flat", 14), ("flat1024", 6)])
def test_forward_full_size_on_sampled_patches(name, per_batch):
    """Every configuration of the benchmark at full size (and the flat layer at the sweep's largest channel count,
    whose value GEMM is dealt to eight items per group).  The sample holds, per batch item, the first and last patch
    and the seams of the 32- and 128-patch tiles, and over the batch every position inside a 32-patch tile and every
    tile of the patch axis (where B * per_batch allows), so the ends of every XCD's item range are in it."""
    cfg = FLAT1024 if name == "flat1024" else get_config(name)
    _forward_on_sampled_patches(cfg, name, per_batch, covering=True)


@pytest.mark.parametrize("name", ["hyperspectral", "deep1000"])
def test_forward_full_size_fast_and_generic_routes_agree_everywhere(monkeypatch, name):
    """The whole output, every (b, n), of the MFMA path against the shape-generic level kernels (another tiling, the
    projected values materialised and rounded once more): two independent GPU routes, compared at full size within the
    bf16 tolerance.  The oracle samples patches; this covers every tile and item boundary."""
    cfg = get_config(name)
    say(f"full-size {name}: generating inputs")
    pr = make_problem(cfg)
    fast = run_forward(pr).float()
    monkeypatch.setenv("DCHAG_GENERIC_LEVEL", "1")
    say(f"full-size {name}: generic route")
    slow = run_forward(pr).float()
    scale = float(slow.abs().max())
    worst = float((fast - slow).abs().amax(dim=-1).max()) / scale
    per_row = (fast - slow).abs().amax(dim=-1) / scale                      # [B, N]
    say(f"full-size {name}: fast vs generic, max|d|/max|ref| over all {per_row.numel()} patches = {worst:.3e}")
    assert torch.isfinite(fast).all() and worst < TOL["bf16"]


@pytest.mark.parametrize("narrow", [False, True])
def test_forward_linear_first_level_patch_tiles(monkeypatch, narrow):
    """The fused tokenizer + linear first level with 128 patches per workgroup (taken when that leaves a workgroup per
    compute unit) and with 64: N = 500 patches (ragged last tile either way), 16 pixels per patch, groups 4 + 4 + ... + 1."""
    if narrow:
        monkeypatch.setenv("DCHAG_MIX_NARROW", "1")
    cfg = cfg_of(dtype="bf16", B=4, C=33, H=80, W=100, p=4, D=512, heads=8, group_sizes=(4, 9),
                 level_kinds=("linear", "attention"))
    _forward_on_sampled_patches(cfg, f"linear first level, narrow={narrow}", 10)


@pytest.mark.parametrize("route", ["ring", "ring_shape_1", "registers", "registers_narrow"])
def test_forward_linear_first_level_of_8x8_patches(monkeypatch, route):
    """The fused tokenizer + linear first level on 8 x 8 patches: the kernel that streams a member's patches and weights
    through an LDS ring (workgroups of 128 patches x 256 columns with three stages, one per compute unit, or 128 x 128 with
    two stages, two per compute unit), and the two
    that pass them through registers; N = 204 patches (two tiles of 128 or four of 64,
    the last ragged), two 256-column slices, groups 4 + 4 + 4 + 1."""
    if route.startswith("ring_shape_"):
        monkeypatch.setenv("DCHAG_RING_SHAPE", route[-1])
    elif route != "ring":
        monkeypatch.setenv("DCHAG_FIRST_LEVEL_REGS", "1")
    if route == "registers_narrow":
        monkeypatch.setenv("DCHAG_MIX_NARROW", "1")
    cfg = cfg_of(dtype="bf16", B=2, C=13, H=96, W=136, p=8, D=512, heads=8, group_sizes=(4, 4),
                 level_kinds=("linear", "attention"))
    _forward_on_sampled_patches(cfg, f"linear first level of 8 x 8 patches, {route}", 30)


def _forward_on_sampled_patches(cfg, name, per_batch, covering=False):
    """The configurations of the benchmark at full size, in the launch configuration the benchmark
    times; the oracle computes a seeded sample of patches (every weight takes part in every patch)."""
    say(f"full-size {name}: generating inputs")
    pr = make_problem(cfg)
    say(f"full-size {name}: running the GPU path")
    out = run_forward(pr)
    sampler = sample_patches_covering if covering else sample_patches
    bs, ns = sampler(cfg.B, cfg.N, per_batch, seed=17)
    say(f"full-size {name}: oracle on {bs.size} patches")
    want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, sample=(bs, ns))
    got = host(out[torch.from_numpy(bs).long().cuda(), torch.from_numpy(ns).long().cuda()])
    err = rel_err(got, want)
    mx, el, rms = err_figures(got, want)
    say(f"full-size {name}: max|d|/max|ref| = {mx:.3e} (gated), element-wise |d|/max(|ref|, rms ref) = {el:.3e}, "
        f"rms(d)/rms(ref) = {rms:.3e}")
    assert err < TOL[cfg.dtype]
    # property that holds at any size: every output row is finite and no row was left untouched
    assert torch.isfinite(out.float()).all()
    assert (out.float().abs().amax(dim=-1) > 0).all()
