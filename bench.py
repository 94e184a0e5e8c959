#!/usr/bin/env python3
"""Benchmark of the D-CHAG hot path on one MI355X.

One "step" is one dchag_forward call (tokenize + every aggregation level) over one batch of
seeded synthetic input that is already resident in HBM.  The metric is aggregated
channel-patch tokens per second, B*C*N / time.  Prints ONE JSON line.  --mode folded / backward
times dchag_forward_folded / dchag_backward the same way (the default run reports them as side lines).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload hyperspectral|weather|...]
                    [--mode forward|folded|backward]
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

# HBM-side bytes per launch of the dominant kernel, from the two rocprofv3 --pmc runs summarised in
# profiles/hbm_traffic_hyperspectral.txt (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, the scales a plain
# 1 GiB copy kernel gives for the same counters).  Valid for that workload and kernel only.
MEASURED_TRAFFIC = {("hyperspectral", "fused_vagg", 1): 1678.0e6}


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
    ap.add_argument("--no-other", action="store_true", help="skip the short weather-like side measurement")
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
    from workloads import get_config, level_inputs, make_problem, sample_patches

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dchag.load_library()

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

    mode = {"name": args.mode, "bwd": None}

    def step(cfg, t):
        x, We, be, ce, levels, ws, out = t
        if mode["name"] == "forward":
            dchag.dchag_forward(x, We, be, ce, levels, cfg.p, cfg.heads, out=out, workspace=ws)
        elif mode["name"] == "folded":
            dchag.dchag_forward_folded(x, We, be, ce, levels, cfg.p, cfg.heads, out=out, workspace=ws)
        else:
            bw = mode["bwd"]
            dchag.dchag_backward(x, We, be, ce, levels, cfg.p, cfg.heads, bw["dout"], bw["grads"], dx=bw["dx"],
                                 dWe=bw["dWe"], dtok_bias=bw["dtb"], workspace=bw["ws"])

    def timed(cfg, t, warmup, steps, profile):
        for _ in range(warmup):
            step(cfg, t)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if profile:
            dchag.dchag_profile_begin()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            step(cfg, t)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        recs = dchag.dchag_profile_end() if profile else []
        return max(e0.elapsed_time(e1), 0.0) / steps, wall_ms / steps, recs

    cfg = get_config(args.workload)
    pr, t = prepare(cfg)
    if args.mode == "backward":
        mode["bwd"] = prepare_backward(cfg, t)
    # untimed-stage pass first (value), then the same steps again with per-launch events (roofline)
    ms_plain, wall_plain, _ = timed(cfg, t, args.warmup, args.steps, profile=False)
    ms_prof, _, recs = timed(cfg, t, 1, args.steps, profile=True)
    ms = ms_plain
    tokens = cfg.tokens
    value = tokens / (ms * 1e-3)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)          # elementwise kernel: 2^30 bytes in, 2^30 bytes out
        torch.cuda.synchronize()
        del src, dst

    # per-stage averages over the profiled region
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
        avg = tot / args.steps                       # per step: a stage may take several launches
        if bound == "mfma":
            ach, peak, unit = amount / (avg * 1e-3) / 1e12, PEAK["mfma_bf16_tflops"] if cfg.dtype == "bf16" else PEAK["fp32_tflops"], "TFLOP/s"
        else:
            ach, peak, unit = amount / (avg * 1e-3) / 1e9, PEAK["hbm_gbs"], "GB/s"
        stages.append({"stage": name, "level": level, "avg_ms": round(avg, 5), "launches": cnt // args.steps, "bound": bound,
                       "achieved": round(ach, 2), "peak": peak, "unit": unit, "frac": round(ach / peak, 4)})
    stages.sort(key=lambda s: -s["avg_ms"])
    dom = stages[0] if stages else None
    roofline = None
    if dom:
        roofline = {"kernel": f"{dom['stage']}@level{dom['level']}", "bound": dom["bound"], "achieved": dom["achieved"],
                    "peak": dom["peak"], "unit": dom["unit"], "frac": dom["frac"],
                    "traffic": MEASURED_TRAFFIC.get((cfg.name, dom["stage"], dom["level"])),
                    "avg_ms": dom["avg_ms"]}

    # the CPU oracle on a bounded sample of the same workload (reported baseline, not a target)
    cpu = None
    if args.cpu_patches > 0 and args.mode != "backward":
        import oracle
        per_b = max(1, args.cpu_patches // cfg.B)
        bs, ns = sample_patches(cfg.B, cfg.N, per_b, seed=23)
        t0 = time.perf_counter()
        want = oracle.forward(pr.x, pr.We, pr.be, pr.ce, pr.levels, cfg.p, cfg.heads, sample=(bs, ns))
        dt_cpu = time.perf_counter() - t0
        got = t[6][torch.from_numpy(bs).long().cuda(), torch.from_numpy(ns).long().cuda()].to(torch.float64).cpu().numpy()
        err = float(np.abs(got - want).max() / np.abs(want).max())
        cpu = {"value": bs.size * cfg.C / dt_cpu, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"{bs.size} of {cfg.B * cfg.N} patches ({bs.size * cfg.C} channel-patch tokens), fp64, "
                         f"{dt_cpu:.1f} s; GPU-vs-oracle max|err|/max|ref| on them = {err:.2e}"}

    # the staged entry points on the same workload: dchag_tokenize, then dchag_aggregate_level on level 1
    # with its tokens coming from HBM (its score kernel is the HBM-bound aggregation stage)
    staged = None
    if not args.no_other and pr.levels[0].kind == "attention" and args.mode == "forward":
        x, We, be, ce, levels, ws, out = t
        tok = dchag.dchag_tokenize(x, We, be, ce, cfg.p)
        lvl_out = dchag.dchag_aggregate_level(tok, levels[0], cfg.heads)
        torch.cuda.synchronize()
        dchag.dchag_profile_begin()
        for _ in range(5):
            dchag.dchag_aggregate_level(tok, levels[0], cfg.heads, out=lvl_out)
        torch.cuda.synchronize()
        acc = {}
        for name, level, dur in dchag.dchag_profile_end():
            acc.setdefault(name, []).append(dur)
        es = 4 if cfg.dtype == "f32" else 2
        sc_ms = sum(acc["scores"]) / len(acc["scores"])
        # algorithmic bytes: every token read once, one fp32 softmax weight per (token, head) written once
        sc_bytes = cfg.tokens * cfg.D * es + cfg.tokens * cfg.heads * 4
        staged = {"call": "dchag_aggregate_level(level 1), tokens read from HBM",
                  "stage_ms": {k: round(sum(v) / len(v), 5) for k, v in acc.items()},
                  "scores_stage": {"bound": "hbm", "achieved": round(sc_bytes / (sc_ms * 1e-3) / 1e9, 1),
                                   "peak": PEAK["hbm_gbs"], "unit": "GB/s",
                                   "frac": round(sc_bytes / (sc_ms * 1e-3) / 1e9 / PEAK["hbm_gbs"], 4),
                                   "note": "scores + softmax over the group: every token read once (2*D bytes), "
                                           "softmax weights written once (4*heads bytes per token)"}}
        del tok, lvl_out

    other = []
    if not args.no_other and args.workload == "hyperspectral" and args.mode == "forward":
        # the same workload through the other two calls (their own stage tables come with --mode)
        mode["name"] = "folded"
        msf, _, _ = timed(cfg, t, 3, 10, profile=False)
        other.append({"workload": "hyperspectral", "call": "dchag_forward_folded", "tokens": cfg.tokens,
                      "ms_per_step": round(msf, 4), "value": cfg.tokens / (msf * 1e-3), "unit": "tokens/s"})
        # the same with everything that depends on the weights alone prepared once, outside the timed calls
        xf, Wef, bef, cef, lvf, wsf, outf = t
        folded = dchag.dchag_fold_value(Wef, bef, cef, lvf, cfg.p, cfg.heads)
        if folded is not None:
            for _ in range(3):
                dchag.dchag_forward_prefolded(xf, Wef, bef, cef, lvf, cfg.p, cfg.heads, folded, out=outf, workspace=wsf)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                dchag.dchag_forward_prefolded(xf, Wef, bef, cef, lvf, cfg.p, cfg.heads, folded, out=outf, workspace=wsf)
            e1.record()
            torch.cuda.synchronize()
            mspf = e0.elapsed_time(e1) / 10
            other.append({"workload": "hyperspectral", "call": "dchag_forward_prefolded (weights folded once, outside)",
                          "tokens": cfg.tokens, "ms_per_step": round(mspf, 4), "value": cfg.tokens / (mspf * 1e-3),
                          "unit": "tokens/s"})
        del xf, Wef, bef, cef, lvf, wsf, outf, folded
        mode["name"], mode["bwd"] = "backward", prepare_backward(cfg, t)
        msb, _, _ = timed(cfg, t, 2, 5, profile=False)
        other.append({"workload": "hyperspectral", "call": "dchag_backward (recomputes the forward)",
                      "tokens": cfg.tokens, "ms_per_step": round(msb, 4), "value": cfg.tokens / (msb * 1e-3),
                      "unit": "tokens/s"})
        # a training step that keeps its activations: dchag_forward_keep + dchag_backward_kept on one workspace
        bw = mode["bwd"]
        xk, Wk_, bk_, ck_, lvk, _, outk = t

        def train_step():
            dchag.dchag_forward_keep(xk, Wk_, bk_, ck_, lvk, cfg.p, cfg.heads, bw["ws"], out=outk)
            dchag.dchag_backward(xk, Wk_, bk_, ck_, lvk, cfg.p, cfg.heads, bw["dout"], bw["grads"], dx=bw["dx"],
                                 dWe=bw["dWe"], dtok_bias=bw["dtb"], workspace=bw["ws"], kept=True)
        for _ in range(2):
            train_step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            train_step()
        e1.record()
        torch.cuda.synchronize()
        mst = e0.elapsed_time(e1) / 5
        other.append({"workload": "hyperspectral", "call": "dchag_forward_keep + dchag_backward_kept (one training step)",
                      "tokens": cfg.tokens, "ms_per_step": round(mst, 4), "value": cfg.tokens / (mst * 1e-3),
                      "unit": "tokens/s"})
        del xk, Wk_, bk_, ck_, lvk, outk, bw
        mode["name"], mode["bwd"] = "forward", None
        # the forward with the positional embedding added in the last projection's epilogue
        xx, Wee, bee, cee, lvls, wss, outt = t
        pos = torch.randn((cfg.N, cfg.D), device="cuda", dtype=torch.float32).to(outt.dtype)
        for _ in range(3):
            dchag.dchag_forward_pos(xx, Wee, bee, cee, lvls, cfg.p, cfg.heads, pos, out=outt, workspace=wss)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            dchag.dchag_forward_pos(xx, Wee, bee, cee, lvls, cfg.p, cfg.heads, pos, out=outt, workspace=wss)
        e1.record()
        torch.cuda.synchronize()
        msp = e0.elapsed_time(e1) / 10
        other.append({"workload": "hyperspectral", "call": "dchag_forward_pos", "tokens": cfg.tokens,
                      "ms_per_step": round(msp, 4), "value": cfg.tokens / (msp * 1e-3), "unit": "tokens/s"})
        del xx, Wee, bee, cee, lvls, wss, outt, pos
        del t
        torch.cuda.empty_cache()
        c2 = get_config("weather")
        _, t2 = prepare(c2)
        ms2, _, _ = timed(c2, t2, 3, 10, profile=False)
        other.append({"workload": "weather", "tokens": c2.tokens, "ms_per_step": round(ms2, 4),
                      "value": c2.tokens / (ms2 * 1e-3), "unit": "tokens/s"})
        mode["name"] = "folded"
        ms2f, _, _ = timed(c2, t2, 3, 10, profile=False)
        other.append({"workload": "weather", "call": "dchag_forward_folded", "tokens": c2.tokens,
                      "ms_per_step": round(ms2f, 4), "value": c2.tokens / (ms2f * 1e-3), "unit": "tokens/s"})
        mode["name"] = "forward"
        del t2
        torch.cuda.empty_cache()
        # the same hyperspectral shape with a linear first level (D-CHAG-L), cross-attention at the top, and as
        # one flat cross-attention layer over all 512 channels (the baseline the hierarchy is compared with)
        for wl in ("hyperspectral_linear", "hyperspectral_flat"):
            c3 = get_config(wl)
            _, t3 = prepare(c3)
            ms3, _, _ = timed(c3, t3, 3, 10, profile=False)
            other.append({"workload": wl, "tokens": c3.tokens, "ms_per_step": round(ms3, 4),
                          "value": c3.tokens / (ms3 * 1e-3), "unit": "tokens/s"})
            if wl == "hyperspectral_linear":        # and its backward (forward recomputation included)
                mode["name"], mode["bwd"] = "backward", prepare_backward(c3, t3)
                ms3b, _, _ = timed(c3, t3, 2, 5, profile=False)
                other.append({"workload": wl, "call": "dchag_backward (recomputes the forward)", "tokens": c3.tokens,
                              "ms_per_step": round(ms3b, 4), "value": c3.tokens / (ms3b * 1e-3), "unit": "tokens/s"})
                mode["name"], mode["bwd"] = "forward", None
            del t3
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
                ms4, _, _ = timed(c4, t4, 3, 10, profile=False)
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
        "config": {"workload": cfg.name, "call": {"forward": "dchag_forward", "folded": "dchag_forward_folded",
                                                  "backward": "dchag_backward"}[args.mode], "B": cfg.B, "C": cfg.C, "H": cfg.H, "W": cfg.W, "patch": cfg.p, "N": cfg.N,
                   "D": cfg.D, "heads": cfg.heads, "group_sizes": list(cfg.group_sizes),
                   "level_kinds": list(cfg.level_kinds or ["attention"] * len(cfg.group_sizes)),
                   "tokens_per_step": tokens},
        "roofline": roofline,
        "cpu_baseline": cpu,
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
