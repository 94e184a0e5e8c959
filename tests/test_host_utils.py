"""Host-side helpers that the GPU tests and the benchmark lean on (no GPU needed): the seeded generators' block-keyed
streams, the bf16 rounding, the covering patch sampler, the benchmark's error figures and its reader of the committed
HBM-traffic profile, and the build options of the timing-probe libraries."""
import importlib.util
import os

import numpy as np
import pytest
import torch

import workloads
from workloads import get_config, make_problem, round_to_bf16, sample_patches_covering

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_round_to_bf16_is_round_to_nearest_even():
    rng = np.random.Generator(np.random.PCG64(5))
    a = (rng.standard_normal(1 << 16) * 3).astype(np.float32)
    a[:6] = [0.0, -0.0, 1.0, 1.00390625, 1.0078125, 3.0e38]        # ties in both directions, a value near the top
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = round_to_bf16(a)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.array_equal(round_to_bf16(got), got)                 # idempotent


def test_large_tensors_do_not_depend_on_the_number_of_threads(monkeypatch):
    cfg = workloads.ShapeCfg("t", "bf16", 1, 40, 64, 64, 8, 512, 8, (8, 5), "ar1", 11)   # Wv of level 1: 5 * 2^18 * ... > one block
    monkeypatch.setattr(workloads, "_BLOCK", 1 << 12)              # many blocks per tensor at this size
    monkeypatch.setattr(workloads, "_THREADS", 1)
    a = make_problem(cfg)
    monkeypatch.setattr(workloads, "_THREADS", 7)
    b = make_problem(cfg)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.We, b.We)
    for la, lb in zip(a.levels, b.levels):
        assert np.array_equal(la.Wv, lb.Wv) and np.array_equal(la.Wk, lb.Wk) and np.array_equal(la.query, lb.query)
    # the values are N(0, 1/D) as the recipe says, and blocks are not copies of one another
    w = a.levels[0].Wv.reshape(-1)
    assert abs(float(w.std()) * np.sqrt(cfg.D) - 1.0) < 0.02 and abs(float(w.mean())) < 1e-3
    assert not np.array_equal(w[: 1 << 12], w[1 << 12: 1 << 13])


def test_tiny_configuration_is_still_the_single_stream_draw():
    """Small tensors come straight from the one seeded stream (the frozen oracle output of the tiny case depends on it)."""
    cfg = get_config("tiny")
    pr = make_problem(cfg)
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    mu = rng.uniform(-1.0, 1.0, size=cfg.C).astype(np.float32)
    sg = rng.uniform(0.5, 2.0, size=cfg.C).astype(np.float32)
    x = rng.standard_normal((cfg.B, cfg.C, cfg.H, cfg.W), dtype=np.float32) * sg[None, :, None, None] + mu[None, :, None, None]
    assert np.array_equal(pr.x, x.astype(np.float32))


@pytest.mark.parametrize("B,N,per_batch", [(2, 256, 22), (1, 2048, 40), (4, 256, 14), (1, 5, 16), (2, 128, 8), (3, 33, 4)])
def test_sample_patches_covering(B, N, per_batch):
    bs, ns = sample_patches_covering(B, N, per_batch, seed=17)
    want = min(per_batch, N)
    assert bs.dtype == np.int32 and ns.dtype == np.int32 and bs.size == B * want
    assert ns.min() >= 0 and ns.max() < N
    for b in range(B):
        mine = ns[bs == b]
        assert mine.size == want and np.unique(mine).size == want and np.all(np.diff(mine) > 0)
        forced = [n for n in (0, N - 1, 31, 32, 127, 128) if 0 <= n < N][:want]
        assert set(forced) <= set(int(n) for n in mine)
    if B * want >= 32 + 6 * B and N >= 64:
        assert len(set(int(n) % 32 for n in ns)) == 32             # every position inside a 32-patch tile
    assert np.array_equal(sample_patches_covering(B, N, per_batch, seed=17)[1], ns)      # seeded


def test_error_report_figures():
    bench = load_bench()
    want = np.array([[4.0, 0.0, -2.0, 0.001]])
    got = want + np.array([[0.04, 0.02, 0.0, 0.001]])
    rep = bench.error_report(got, want)
    rms = float(np.sqrt(np.mean(want ** 2)))
    assert rep["max_norm"] == pytest.approx(0.04 / 4.0)
    assert rep["elementwise"] == pytest.approx(max(0.04 / 4.0, 0.02 / rms, 0.001 / rms))
    assert rep["rms"] == pytest.approx(float(np.sqrt(np.mean(np.array([0.04, 0.02, 0.0, 0.001]) ** 2))) / rms)


def test_measured_traffic_comes_from_the_committed_profile():
    bench = load_bench()
    v = bench.measured_traffic("hyperspectral", "fused_vagg", 1)
    text = open(os.path.join(ROOT, "profiles", "hbm_traffic_hyperspectral.txt")).read()
    line = next(ln for ln in text.splitlines() if ln.startswith("k_vagg_mfma (1/2)"))
    assert v == pytest.approx(float(line.split()[-2]) * 1e6) and 1.0e9 < v < 3.0e9
    assert bench.measured_traffic("hyperspectral", "fused_vagg", 2) < v
    assert bench.measured_traffic("wide", "fused_vagg", 1) is None           # no such profile committed
    assert bench.measured_traffic("hyperspectral", "no_such_stage", 1) is None


def test_stage_model_counts_what_is_executed():
    bench = load_bench()
    cfg = get_config("hyperspectral")
    lv_in = workloads.level_inputs(cfg.C, cfg.group_sizes)
    bound, flops = bench.stage_model(cfg, lv_in, "fused_vagg", 1)
    assert bound == "mfma" and flops == 2.0 * cfg.tokens * cfg.D * cfg.D               # 1.0995e12: the value GEMM alone
    bound, by = bench.stage_model(cfg, lv_in, "key_prep", 0)
    assert bound == "hbm" and by == 2 * (16 + 1) * cfg.D * cfg.D * 2                 # Wq and Wk of 16 + 1 groups, bf16
    assert bench.stage_model(cfg, lv_in, "key_prep", 2)[1] == 2 * cfg.D * cfg.D * 2


def test_probe_builds_need_their_own_output_file():
    from paper_2506_21411_amd.build import LIB, build
    with pytest.raises(ValueError):
        build(verbose=False, out=LIB, defines=["DCHAG_GEMM_PROBE=8"])
