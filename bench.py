#!/usr/bin/env python3
"""Benchmark of the D-CHAG hot path on one MI355X.

One "step" is one dchag_forward call (tokenize + every aggregation level) over one batch of
seeded synthetic input that is already resident in HBM.  The metric is aggregated
channel-patch tokens per second, B*C*N / time.  Prints ONE JSON line.  --mode folded / backward
times dchag_forward_folded / dchag_backward the same way (the default run reports them as side lines).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload hyperspectral|weather|...]
                    [--mode forward|folded|backward] [--peaks] [--flat-sweep]

Before the W warm-up steps the device is kept busy with the same step for --spin-ms milliseconds: after an idle
phase (here: the host-side generation of the inputs) the first tens of launches of a heavy kernel run up to 35 %
slower while the power state settles, which has nothing to do with the kernels.  The K timed steps follow the
W warm-up steps directly.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"mfma_bf16_tflops": 2500.0, "hbm_gbs": 8000.0, "fp32_tflops": 157.3}

# Stage names of the library's timing records -> kernel name prefixes in the rocprofv3 summaries under profiles/.
STAGE_KERNEL = {"fused_vagg": "k_vagg_mfma", "tokenize": "k_tokenize_ws", "tokenize_mix": "k_tokenize_reduce_ring",
                "tokenize_attend": "k_tokenize_reduce_ring", "oproj": "k_linear_dl"}


def measured_traffic(workload, stage, level):
    """HBM-side bytes per launch of a kernel, read from profiles/hbm_traffic_<workload>.txt (two rocprofv3 --pmc runs,
    FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a plain 1 GiB copy; the file states the
    scales).  None where no such profile has been committed for the workload and kernel."""
    kern = STAGE_KERNEL.get(stage)
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if kern is None or not os.path.exists(path):
        return None
    rows = [ln.split() for ln in open(path) if ln.startswith(kern)]
    rows = [r for r in rows if len(r) >= 2 and r[-1] == "MB"]
    if not rows:
        return None
    # several launches of one kernel per step are listed as (i/m), level 1 first
    pick = rows[min(level, len(rows)) - 1] if level >= 1 else rows[0]
    try:
        return float(pick[-2]) * 1e6
    except ValueError:
        return None


def error_report(got, want):
    """The three error figures reported beside every oracle comparison (y = GPU, r = oracle, d = y - r):
    max_norm = max|d| / max|r| (the gated one), elementwise = max_i |d_i| / max(|r_i|, rms r), rms = rms d / rms r."""
    import numpy as np
    d = np.abs(np.asarray(got, dtype=np.float64) - want)
    rms_r = float(np.sqrt(np.mean(np.square(want))))
    return {"max_norm": float(d.max() / np.abs(want).max()),
            "elementwise": float((d / np.maximum(np.abs(want), rms_r)).max()),
            "rms": float(np.sqrt(np.mean(np.square(d))) / rms_r),
            "definition": "max_norm = max|y-r|/max|r| (gate: 2e-2 bf16, 1e-4 fp32); elementwise = max_i |y_i-r_i| / "
                          "max(|r_i|, rms r); rms = rms(y-r)/rms(r)"}


def stage_model(cfg, levels_in, stage, level, fused_tokens=False):
    """Algorithmic work of one launch of a stage: (bound, amount, unit) with amount in flops or bytes.
    fused_tokens: the level's reverse step at the tokens ran as one kernel (no separate softmax stage)."""
    es = 4 if cfg.dtype == "f32" else 2
    B, N, D, h = cfg.B, cfg.N, cfg.D, cfg.heads
    if stage == "tokenize":
        by = B * cfg.C * cfg.H * cfg.W * es + cfg.C * D * cfg.p * cfg.p * es + B * cfg.C * N * D * es
        return "hbm", by
    if stage == "bwd_tokenize":
        # token gradients read for dWe and again for dx; pixels in, pixel gradients out, weights in and out
        return "hbm", (2 * B * cfg.C * N * D + 2 * B * cfg.C * cfg.H * cfg.W + 2 * cfg.C * D * cfg.p * cfg.p) * es
    if stage == "key_prep":
        # Wq and Wk of every group read once: of one level, or (level 0) of all attention levels of the call
        kinds = list(cfg.level_kinds or ["attention"] * len(cfg.group_sizes))
        lvls = range(len(levels_in)) if level == 0 else [level - 1]
        return "hbm", sum(2 * ((levels_in[i] + cfg.group_sizes[i] - 1) // cfg.group_sizes[i]) * D * D * es
                          for i in lvls if kinds[i] == "attention")
    cin = levels_in[level - 1]
    g = cfg.group_sizes[level - 1]
    G = (cin + g - 1) // g
    tok = B * cin * N
    if stage == "tokenize_mix":
        # tokenizer fused with a linear first level: pixels, tokenizer and mixing weights in, group tokens out
        return "hbm", (B * cfg.C * cfg.H * cfg.W + cfg.C * D * cfg.p * cfg.p + G * g * D + B * G * N * D) * es
    if stage == "fold_value":
        # weight-only: Wf[c] = Wv[k(c)] We[c] (and the two folded bias vectors)
        return "mfma", 2.0 * cfg.C * D * D * (cfg.p * cfg.p + 2)
    if stage == "tokenize_attend":
        # tokenizer fused with an attention first level (value projection folded into the tokenizer weights):
        # pixels, folded weights and softmax weights in, pre-projection outputs out
        return "hbm", (B * cfg.C * cfg.H * cfg.W + cfg.C * D * cfg.p * cfg.p + B * G * N * D) * es + tok * h * 4
    if stage == "channel_mix":
        return "hbm", (tok * D + G * g * D + B * G * N * D) * es
    if stage == "vproj":
        return "mfma", 2.0 * tok * D * D
    if stage == "oproj":
        return "mfma", 2.0 * B * G * N * D * D
    if stage == "fused_vagg":
        # the value projection itself; the weighted sum in its epilogue runs on the vector ALUs and is not counted
        # (SQ_INSTS_VALU_MFMA_MOPS_BF16 x 512 of the kernel gives exactly this number)
        return "mfma", 2.0 * tok * D * D
    if stage == "scores":
        if level == 1 and cfg.dtype == "bf16":
            # first level of a forward call: scores come from the pixels through composed weights
            return "hbm", B * cfg.C * cfg.H * cfg.W * es + cfg.C * D * cfg.p * cfg.p * es + 2 * tok * h * 4
        return "hbm", tok * D * es + tok * h * 4
    if stage == "softmax_agg":
        return "hbm", tok * D * es + tok * h * 4 + B * G * N * D * es
    if stage in ("query", "fold"):
        return "hbm", G * D * D * es
    # weight-folded forward and backward: u / w are the per-head tensors [B,G,N,h,D]
    uw = B * G * N * h * D * es
    if stage == "head_sums":
        return "hbm", tok * D * es + tok * h * 4 + uw
    if stage == "head_vproj":
        # every u row (D values) yields only D/heads outputs: 2*D/heads flops per byte of u, far below the ridge
        return "hbm", uw + B * G * N * D * es + G * D * D * es
    if stage == "bwd_oproj":
        return "mfma", 4.0 * B * G * N * D * D
    if stage == "bwd_value":
        # dWv reads u and d_o, w = Wv_a^T d_o_a is written once: bound by the two per-head tensors
        return "hbm", 2 * uw + 2 * B * G * N * D * es + 2 * G * D * D * es
    if stage == "bwd_softmax":
        return "hbm", tok * D * es + uw + 3 * tok * h * 4
    if stage == "bwd_tokens":
        if fused_tokens:
            # one kernel: tokens and w in once, token gradients out, softmax weights in, partial key-path sums out
            return "hbm", uw + 2 * tok * D * es + tok * h * 4
        return "hbm", uw + tok * D * es + 2 * tok * h * 4
    if stage == "bwd_key_query":
        return "hbm", tok * D * es + tok * h * 4 + 3 * G * D * D * es
    if stage == "bwd_channel_mix":
        return "hbm", (2 * tok * D + 2 * B * G * N * D + 2 * G * g * D) * es
    return "hbm", 0.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="hyperspectral")
    ap.add_argument("--mode", default="forward", choices=["forward", "folded", "backward"],
                    help="what one step is: dchag_forward (the headline), dchag_forward_folded, or dchag_backward")
    ap.add_argument("--cpu-patches", type=int, default=384, help="patches the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--spin-ms", type=float, default=300.0,
                    help="milliseconds of untimed steps before the warm-up steps (settles the power state)")
    ap.add_argument("--no-other", action="store_true",
                    help="only the timed call: no staged calls, no yardsticks, no other calls or workloads")
    ap.add_argument("--peaks", action="store_true",
                    help="only measure the achievable rates (MFMA-only loop, stream copy) and print them")
    ap.add_argument("--library", default=None,
                    help="another build of libdchag.so (a timing-probe build of paper_2506_21411_amd.build --define ...)")
    ap.add_argument("--flat-sweep", action="store_true",
                    help="also time the hyperspectral shape at C = 128 .. 1024 channels as one flat layer and as the "
                         "two-level hierarchy (groups of 32), forward")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy kernel (reads 1 GiB, writes 1 GiB): the yardstick "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the hierarchy is run locally; no collectives). "
              "Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2506_21411_amd as dchag
    from workloads import get_config, level_inputs, make_problem, sample_patches, sample_patches_covering

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.library:
        dchag.use_library(args.library)
    dchag.load_library()

    def events():
        return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def measure_peaks():
        """Achievable rates on this device: a loop of nothing but bf16 MFMAs, and a 1 GiB stream copy."""
        sink = torch.empty(1024 * 512, dtype=torch.float32, device="cuda")
        best = 0.0
        for _ in range(3):
            dchag.dchag_yardstick_mfma(2000, sink)
        for _ in range(5):
            e0, e1 = events()
            e0.record()
            flops = dchag.dchag_yardstick_mfma(20000, sink)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        copy = 0.0
        for _ in range(3):
            dchag.dchag_yardstick_copy(dst, src)
        for _ in range(5):
            e0, e1 = events()
            e0.record()
            nbytes = dchag.dchag_yardstick_copy(dst, src)
            e1.record()
            torch.cuda.synchronize()
            copy = max(copy, 2.0 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        read = 0.0
        for _ in range(3):
            dchag.dchag_yardstick_read(src, sink)
        for _ in range(5):
            e0, e1 = events()
            e0.record()
            nbytes = dchag.dchag_yardstick_read(src, sink)
            e1.record()
            torch.cuda.synchronize()
            read = max(read, nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        del src, dst, sink
        torch.cuda.empty_cache()
        return {"mfma_bf16_tflops": round(best, 1), "copy_gbs": round(copy, 1), "read_gbs": round(read, 1),
                "how": "dchag_yardstick_mfma (16 wavefronts per compute unit, 8 independent 32x32x16 bf16 MFMAs per "
                       "round, registers only), dchag_yardstick_copy (1 GiB read + 1 GiB written; bytes moved = 2 GiB) "
                       "and dchag_yardstick_read (1 GiB read), best of 5 each"}

    if args.peaks:
        print(json.dumps({"achievable": measure_peaks(), "nominal": PEAK}))
        return 0

    def prepare(cfg):
        tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        pr = make_problem(cfg)

        def dev(a):
            return None if a is None else torch.from_numpy(a).to("cuda").to(tdt).contiguous()

        levels = [dchag.LevelWeights(lv.group_size, dev(lv.query), dev(lv.Wq), dev(lv.Wk), dev(lv.Wv), dev(lv.Wo),
                                     dev(lv.bq), dev(lv.bk), dev(lv.bv), dev(lv.bo),
                                     kind=1 if lv.kind == "linear" else 0) for lv in pr.levels]
        dt = dchag.DCHAG_F32 if cfg.dtype == "f32" else dchag.DCHAG_BF16
        wsb = max(dchag.dchag_workspace_bytes(dt, cfg.B, cfg.C, cfg.H, cfg.W, cfg.p, cfg.D, cfg.heads,
                                              list(cfg.group_sizes), which) for which in (1, 2))
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        out = torch.empty((cfg.B, cfg.N, cfg.D), dtype=tdt, device="cuda")
        t = (dev(pr.x), dev(pr.We), dev(pr.be), dev(pr.ce), levels, ws, out)
        return pr, t

    def prepare_backward(cfg, t):
        """Gradient buffers, a seeded upstream gradient and the workspace of dchag_backward."""
        x, We, be, ce, levels, _, out = t
        grads = []
        for lv in levels:
            if lv.kind == 1:
                grads.append(dchag.LevelGrads(dWv=torch.empty_like(lv.Wv), dbv=torch.empty_like(lv.bv)))
            else:
                grads.append(dchag.LevelGrads(**{"d" + n: torch.empty_like(getattr(lv, n)) for n in
                                                 ("query", "Wq", "Wk", "Wv", "Wo", "bq", "bk", "bv", "bo")}))
        g = torch.Generator(device="cuda")
        g.manual_seed(7)
        dout = torch.randn(out.shape, generator=g, device="cuda", dtype=torch.float32).to(out.dtype)
        dt = dchag.DCHAG_F32 if cfg.dtype == "f32" else dchag.DCHAG_BF16
        wsb = dchag.dchag_workspace_bytes(dt, cfg.B, cfg.C, cfg.H, cfg.W, cfg.p, cfg.D, cfg.heads,
                                          list(cfg.group_sizes), 3)
        return {"grads": grads, "dout": dout, "dx": torch.empty_like(x), "dWe": torch.empty_like(We),
                "dtb": torch.empty_like(ce), "ws": torch.empty(wsb, dtype=torch.uint8, device="cuda")}

    def make_step(cfg, t, call, bw=None, folded=None):
        x, We, be, ce, levels, ws, out = t
        if call == "dchag_forward":
            return lambda: dchag.dchag_forward(x, We, be, ce, levels, cfg.p, cfg.heads, out=out, workspace=ws)
        if call == "dchag_forward_folded":
            return lambda: dchag.dchag_forward_folded(x, We, be, ce, levels, cfg.p, cfg.heads, out=out, workspace=ws)
        if call == "dchag_forward_prefolded":
            return lambda: dchag.dchag_forward_prefolded(x, We, be, ce, levels, cfg.p, cfg.heads, folded, out=out,
                                                         workspace=ws)
        if call == "dchag_backward":
            return lambda: dchag.dchag_backward(x, We, be, ce, levels, cfg.p, cfg.heads, bw["dout"], bw["grads"],
                                                dx=bw["dx"], dWe=bw["dWe"], dtok_bias=bw["dtb"], workspace=bw["ws"])
        raise ValueError(call)

    def spin_up(step, ms):
        if ms <= 0:
            return
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < ms:
            for _ in range(10):
                step()
            torch.cuda.synchronize()

    def timed(step, warmup, steps, profile=False):
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        e0, e1 = events()
        if profile:
            dchag.dchag_profile_begin()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        recs = dchag.dchag_profile_end() if profile else []
        return max(e0.elapsed_time(e1), 0.0) / steps, wall_ms / steps, recs

    def stage_table(cfg, recs, steps):
        """Per-stage averages over a profiled region, each against the roofline that bounds it."""
        lv_in = level_inputs(cfg.C, cfg.group_sizes)
        agg = {}
        for name, level, dur in recs:
            a = agg.setdefault((name, level), [0.0, 0])
            a[0] += dur
            a[1] += 1
        stages = []
        for (name, level), (tot, cnt) in agg.items():
            fused = name == "bwd_tokens" and ("bwd_softmax", level) not in agg
            bound, amount = stage_model(cfg, lv_in, name, level, fused)
            avg = tot / steps                            # per step: a stage may take several launches
            if bound == "mfma":
                ach, peak, unit = amount / (avg * 1e-3) / 1e12, PEAK["mfma_bf16_tflops"] if cfg.dtype == "bf16" else PEAK["fp32_tflops"], "TFLOP/s"
            else:
                ach, peak, unit = amount / (avg * 1e-3) / 1e9, PEAK["hbm_gbs"], "GB/s"
            stages.append({"stage": name, "level": level, "avg_ms": round(avg, 5), "launches": cnt // steps, "bound": bound,
                           "achieved": round(ach, 2), "peak": peak, "unit": unit, "frac": round(ach / peak, 4)})
        stages.sort(key=lambda s: -s["avg_ms"])
        return stages

    def dominant(stages):
        d = stages[0]
        return {"kernel": f"{d['stage']}@level{d['level']}", "bound": d["bound"], "achieved": d["achieved"], "peak": d["peak"],
                "unit": d["unit"], "frac": d["frac"], "avg_ms": d["avg_ms"]}

    def oracle_check(cfg, pr, out, bs, ns):
        """The CPU oracle on the sampled patches against the GPU's output there; returns (seconds, error report)."""
        import oracle
        t0 = time.perf_counter()
        want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, sample=(bs, ns))
        dt_cpu = time.perf_counter() - t0
        got = out[torch.from_numpy(bs).long().cuda(), torch.from_numpy(ns).long().cuda()].to(torch.float64).cpu().numpy()
        return dt_cpu, error_report(got, want)

    cfg = get_config(args.workload)
    pr, t = prepare(cfg)
    call = {"forward": "dchag_forward", "folded": "dchag_forward_folded", "backward": "dchag_backward"}[args.mode]
    bwd = prepare_backward(cfg, t) if args.mode == "backward" else None
    step = make_step(cfg, t, call, bw=bwd)
    spin_up(step, args.spin_ms)
    # the timed pass (value), then the same steps again with per-launch events (roofline)
    ms, wall_plain, _ = timed(step, args.warmup, args.steps)
    ms_prof, _, recs = timed(step, 1, args.steps, profile=True)
    tokens = cfg.tokens
    value = tokens / (ms * 1e-3)
    stages = stage_table(cfg, recs, args.steps)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)          # elementwise kernel: 2^30 bytes in, 2^30 bytes out
        torch.cuda.synchronize()
        del src, dst

    # --no-other leaves only the timed call in the process (what the rocprofv3 runs under profiles/ want)
    achievable = None if args.no_other else measure_peaks()
    roofline = None
    if stages:
        roofline = dominant(stages)
        d0 = stages[0]
        roofline["traffic"] = measured_traffic(cfg.name, d0["stage"], d0["level"])
        if achievable:
            ach_peak = achievable["mfma_bf16_tflops"] if roofline["bound"] == "mfma" else achievable["read_gbs"]
            roofline["achievable_peak"] = ach_peak
            roofline["frac_of_achievable"] = round(roofline["achieved"] / ach_peak, 4)

    # the staged entry points on the same workload: dchag_tokenize, then dchag_aggregate_level on level 1 with its
    # tokens coming from HBM (its score kernel is the HBM-bound aggregation stage the target names)
    staged = None
    if pr.levels[0].kind == "attention" and args.mode == "forward" and cfg.dtype == "bf16" and not args.no_other:
        x, We, be, ce, levels, ws, out = t
        tok = dchag.dchag_tokenize(x, We, be, ce, cfg.p)
        lvl_out = dchag.dchag_aggregate_level(tok, levels[0], cfg.heads)
        agg_step = lambda: dchag.dchag_aggregate_level(tok, levels[0], cfg.heads, out=lvl_out)
        spin_up(agg_step, args.spin_ms / 3)
        _, _, srecs = timed(agg_step, 5, 20, profile=True)
        acc = {}
        for name, level, dur in srecs:
            acc.setdefault(name, []).append(dur)
        es = 4 if cfg.dtype == "f32" else 2
        sc_ms = sum(acc["scores"]) / len(acc["scores"])
        # algorithmic bytes: every token read once, one fp32 softmax weight per (token, head) written once
        sc_bytes = cfg.tokens * cfg.D * es + cfg.tokens * cfg.heads * 4
        sc_gbs = sc_bytes / (sc_ms * 1e-3) / 1e9
        staged = {"call": "dchag_aggregate_level(level 1), tokens read from HBM; 20 calls after 5 warm-up calls",
                  "stage_ms": {k: round(sum(v) / len(v), 5) for k, v in acc.items()},
                  "scores_stage": {"bound": "hbm", "achieved": round(sc_gbs, 1), "peak": PEAK["hbm_gbs"], "unit": "GB/s",
                                   "frac": round(sc_gbs / PEAK["hbm_gbs"], 4),
                                   "frac_of_achievable": round(sc_gbs / achievable["read_gbs"], 4),
                                   "note": "scores + softmax over the group: every token read once (2*D bytes), "
                                           "softmax weights written once (4*heads bytes per token)"}}
        del tok, lvl_out

    # the two stages the target names, side by side: the value-projection GEMM (MFMA) and the aggregation stage (HBM)
    targets = None
    if args.mode == "forward" and cfg.dtype == "bf16":
        gemm = next((s_ for s_ in stages if s_["stage"] == "fused_vagg" and s_["level"] == 1), None)
        targets = {"gemm_stage": None if gemm is None else
                   {"kernel": "k_vagg_mfma (level-1 value projection, inside dchag_forward)", "bound": "mfma",
                    "achieved": gemm["achieved"], "peak": gemm["peak"], "unit": gemm["unit"], "frac": gemm["frac"],
                    "frac_of_achievable": round(gemm["achieved"] / achievable["mfma_bf16_tflops"], 4) if achievable else None,
                    "goal": 0.5},
                   "aggregation_stage": None if staged is None else
                   dict(staged["scores_stage"], kernel="k_scores_softmax (dchag_aggregate_level, tokens from HBM)", goal=0.6)}

    # the second named stage also sits inside the roofline block, next to the dominant kernel (the first)
    if roofline and targets and targets.get("aggregation_stage"):
        a = targets["aggregation_stage"]
        roofline["aggregation_stage"] = {k_: a[k_] for k_ in ("kernel", "bound", "achieved", "peak", "unit", "frac")}

    # the CPU oracle on a bounded sample of the same workload (reported baseline, not a target)
    cpu = None
    if args.cpu_patches > 0 and args.mode != "backward":
        import oracle
        per_b = max(1, args.cpu_patches // cfg.B)
        bs, ns = sample_patches(cfg.B, cfg.N, per_b, seed=23)
        dt_cpu, err = oracle_check(cfg, pr, t[6], bs, ns)
        cpu = {"value": bs.size * cfg.C / dt_cpu, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"{bs.size} of {cfg.B * cfg.N} patches ({bs.size * cfg.C} channel-patch tokens), fp64, "
                         f"{dt_cpu:.1f} s; GPU-vs-oracle max|err|/max|ref| on them = {err['max_norm']:.2e}",
               "error": err}

    def side(cfg2, t2, call2, warm=5, steps=10, bw=None, folded=None, label=None):
        """One side line: time of a call on a workload, and its dominant stage against that stage's roofline."""
        st2 = make_step(cfg2, t2, call2, bw=bw, folded=folded)
        spin_up(st2, 60.0)
        ms2, _, _ = timed(st2, warm, steps)
        _, _, r2 = timed(st2, 1, steps, profile=True)
        row = {"workload": cfg2.name, "call": label or call2, "tokens": cfg2.tokens, "ms_per_step": round(ms2, 4),
               "value": cfg2.tokens / (ms2 * 1e-3), "unit": "tokens/s"}
        tab = stage_table(cfg2, r2, steps)
        if tab:
            row["dominant"] = dominant(tab)
        return row

    other = []
    if not args.no_other and args.workload == "hyperspectral" and args.mode == "forward":
        # the same workload through the other calls (their own stage tables come with --mode)
        other.append(side(cfg, t, "dchag_forward_folded"))
        xf, Wef, bef, cef, lvf, wsf, outf = t
        folded = dchag.dchag_fold_value(Wef, bef, cef, lvf, cfg.p, cfg.heads)
        if folded is not None:
            other.append(side(cfg, t, "dchag_forward_prefolded", folded=folded,
                              label="dchag_forward_prefolded (weights folded once, outside)"))
        del folded
        bw = prepare_backward(cfg, t)
        other.append(side(cfg, t, "dchag_backward", warm=2, steps=5, bw=bw, label="dchag_backward (recomputes the forward)"))
        # a training step that keeps its activations: dchag_forward_keep + dchag_backward_kept on one workspace

        def train_step():
            dchag.dchag_forward_keep(xf, Wef, bef, cef, lvf, cfg.p, cfg.heads, bw["ws"], out=outf)
            dchag.dchag_backward(xf, Wef, bef, cef, lvf, cfg.p, cfg.heads, bw["dout"], bw["grads"], dx=bw["dx"],
                                 dWe=bw["dWe"], dtok_bias=bw["dtb"], workspace=bw["ws"], kept=True)
        mst, _, _ = timed(train_step, 2, 5)
        other.append({"workload": "hyperspectral", "call": "dchag_forward_keep + dchag_backward_kept (one training step)",
                      "tokens": cfg.tokens, "ms_per_step": round(mst, 4), "value": cfg.tokens / (mst * 1e-3),
                      "unit": "tokens/s"})
        del bw
        # the forward with the positional embedding added in the last projection's epilogue
        pos = torch.randn((cfg.N, cfg.D), device="cuda", dtype=torch.float32).to(outf.dtype)
        msp, _, _ = timed(lambda: dchag.dchag_forward_pos(xf, Wef, bef, cef, lvf, cfg.p, cfg.heads, pos, out=outf,
                                                          workspace=wsf), 3, 10)
        other.append({"workload": "hyperspectral", "call": "dchag_forward_pos", "tokens": cfg.tokens,
                      "ms_per_step": round(msp, 4), "value": cfg.tokens / (msp * 1e-3), "unit": "tokens/s"})
        del xf, Wef, bef, cef, lvf, wsf, outf, pos
        del t, step
        torch.cuda.empty_cache()
        # the other configurations (forward, with the oracle's error on a sample spread over the kernels' tiles), the
        # D-CHAG-L variant of the headline shape and the flat single-layer baseline
        for wl in ("weather", "tiny", "wide", "deep", "deep1000", "hyperspectral_linear", "hyperspectral_flat"):
            c2 = get_config(wl)
            p2, t2 = prepare(c2)
            row = side(c2, t2, "dchag_forward")
            if wl in ("weather", "tiny", "wide", "deep", "deep1000"):
                bs2, ns2 = sample_patches_covering(c2.B, c2.N, max(1, 16 // c2.B), seed=29)
                dt2, err2 = oracle_check(c2, p2, t2[6], bs2, ns2)
                row["oracle"] = {"patches": int(bs2.size), "seconds": round(dt2, 1), "error": err2}
            other.append(row)
            if wl in ("weather", "hyperspectral_linear"):
                other.append(side(c2, t2, "dchag_forward_folded"))
            if wl == "hyperspectral_linear":        # and its backward (forward recomputation included)
                other.append(side(c2, t2, "dchag_backward", warm=2, steps=5, bw=prepare_backward(c2, t2),
                                  label="dchag_backward (recomputes the forward)"))
            del p2, t2
            torch.cuda.empty_cache()

    # hierarchy against the flat single layer over the channel count (forward, hyperspectral shape otherwise)
    sweep = []
    if args.flat_sweep:
        from workloads import ShapeCfg
        base = get_config("hyperspectral")
        torch.cuda.empty_cache()
        for C in (128, 256, 512, 1024):
            row = {"C": C}
            for kind, gsz in (("flat", (C,)), ("hier_g32", (32, C // 32))):
                c4 = ShapeCfg(f"sweep_{kind}_{C}", "bf16", base.B, C, base.H, base.W, base.p, base.D, base.heads, gsz,
                              "ar1", 2)
                _, t4 = prepare(c4)
                ms4, _, _ = timed(make_step(c4, t4, "dchag_forward"), 3, 10)
                row[kind + "_ms"] = round(ms4, 4)
                row[kind + "_tokens_per_s"] = c4.tokens / (ms4 * 1e-3)
                del t4
                torch.cuda.empty_cache()
            sweep.append(row)

    line = {
        "metric": "aggregated channel-patch tokens/sec (B*C*N) through tokenize + hierarchical aggregation, "
                  + {"forward": "forward", "folded": "forward (value projection behind the weighted sum)",
                     "backward": "backward (with forward recomputation)"}[args.mode],
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "call": call, "B": cfg.B, "C": cfg.C, "H": cfg.H, "W": cfg.W, "patch": cfg.p,
                   "N": cfg.N, "D": cfg.D, "heads": cfg.heads, "group_sizes": list(cfg.group_sizes),
                   "level_kinds": list(cfg.level_kinds or ["attention"] * len(cfg.group_sizes)),
                   "tokens_per_step": tokens, "spin_up_ms_before_warmup": args.spin_ms},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "targets": targets,
        "achievable_peaks": achievable,
        "stages": stages,
        "ms_per_step_with_stage_events": ms_prof,
        "wall_ms_per_step": wall_plain,
        "staged_entry_points": staged,
        "other_workloads": other,
    }
    if sweep:
        line["flat_sweep"] = sweep
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
