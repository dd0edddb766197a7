#!/usr/bin/env python3
"""Benchmark of the vocabulary-layer hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input:
p x vp_output_fwd, vp_combine_stats, p x vp_output_bwd (all p shards of the configuration run
in sequence on the one GPU).  The headline workload is the largest configuration, cfg4
(N=4096, h=8192, V=256000, p=16, bf16, logits recomputed in the backward pass); the other
configurations are timed briefly as well and reported under "per_config", each with its own
roofline entry.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line.  value = 6*N*h*V / step time (the paper's FLOP model for the output
layer, appendix A), in TFLOP/s.  With recomputed logits the hardware executes 8*N*h*V flops per
step; that rate is reported next to it as "hardware_tflops" and is never the headline value.
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

import numpy as np  # noqa: E402

BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
# L2-miss / fabric traffic per launch of the GEMM kernels: what leaves the eight L2s towards the memory-side
# cache and HBM.  NOT measured by this run (counters cannot be read from inside the process): the figures
# are copied from the committed rocprofv3 --pmc summaries (FETCH_SIZE, WRITE_SIZE in KiB per dispatch;
# profiles/output_layer_<config>.txt, which state the command).  A plain 256 MiB copy in the same counter
# runs reads 0.5x its size on FETCH_SIZE and 1.0x on WRITE_SIZE, hence the factors.
PMC_FETCH_FACTOR, PMC_WRITE_FACTOR = 2.0, 1.0
PMC_KIB = {   # kernel -> (FETCH_SIZE, WRITE_SIZE); dH is the accumulating launch (all shards but the first)
    "cfg2_llama": {"gemm_bf16_fwd_stats": (106407.0, 46354.1), "gemm_bf16_dH": (132114.7, 80896.0),
                   "gemm_bf16_dW": (99353.0, 80384.0)},
    "cfg3_large_vocab": {"gemm_bf16_fwd_stats": (443979.2, 189183.5), "gemm_bf16_dH": (420997.1, 80896.0),
                         "gemm_bf16_dW": (404757.8, 309940.4)},
    "cfg4_very_large_vocab": {"gemm_bf16_fwd_stats": (859749.0, 51943.3), "gemm_bf16_dlogits": (856499.4, 177420.7),
                              "gemm_bf16_dH": (837983.0, 158828.7), "gemm_bf16_dW": (945260.4, 615018.7)},
}
METRIC = "vocab-layer fwd+bwd TFLOP/s and tokens/s per GPU; % of bf16 MFMA peak"


def dev(x):
    import torch
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(x).cuda()


def time_steps(step, steps, warmup):
    """Returns (wall ms per step, event ms per step) for `steps` calls after `warmup` calls."""
    import torch
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def profiled_steps(vp, step, steps):
    """Per-kernel average launch duration (ms) over `steps` more steps, from HIP events the
    library records around each of its kernel launches on the launch stream."""
    import torch
    torch.cuda.synchronize()
    vp.vp_profile_enable(True)
    try:
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        rec = vp.vp_profile_read()
    finally:
        vp.vp_profile_enable(False)
    return {k: {"ms_per_launch": ms / n, "launches_per_step": n / steps, "ms_per_step": ms / steps}
            for k, (ms, n) in rec.items()}


def make_output_plan(vp, cfg, seeded_numpy, algorithm=1, host=None):
    """Inputs of an output-layer configuration in HBM.  seeded_numpy=True uses the host
    generator shared with the oracle tests (host = (H, [W_r]) if the caller has drawn them already);
    otherwise tensors of the same distribution are drawn on the GPU (only timed, never compared)."""
    import torch
    import synth_inputs as si
    labels = si.make_labels(cfg)
    if seeded_numpy:
        if host is None:
            host = (si.make_H(cfg), [si.make_W_shard(cfg, r) for r in range(cfg.p)])
        H = dev(host[0])
        Ws = [dev(w) for w in host[1]]
    else:
        g = torch.Generator(device="cuda")
        g.manual_seed(si.BASE_SEED)
        tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        H = (torch.randn((cfg.N, cfg.h), generator=g, device="cuda") * cfg.h_std).to(tdt)
        Ws = [(torch.randn((cfg.Vs, cfg.h), generator=g, device="cuda") * cfg.w_std).to(tdt) for _ in range(cfg.p)]
    return vp.OutputLayerPlan(H, Ws, dev(labels), cfg.save_logits, algorithm=algorithm)


def output_numbers(cfg, ms):
    tflops = cfg.model_flops / (ms * 1e-3) / 1e12
    hw_flops = cfg.model_flops * (1.0 if cfg.save_logits else 8.0 / 6.0)
    return {
        "ms_per_step": ms,
        "model_tflops": tflops,
        "hardware_tflops": hw_flops / (ms * 1e-3) / 1e12,
        "pct_bf16_mfma_peak": 100.0 * tflops / BF16_MFMA_PEAK_TFLOPS if cfg.dtype == "bf16" else None,
        "tokens_per_s": cfg.N / (ms * 1e-3),
        "tokens_per_s_per_shard_device": cfg.N * cfg.p / (ms * 1e-3),
    }


def gemm_roofline(cfg, kernels):
    """Roofline entry for the slowest of the bf16 MFMA GEMM kernels."""
    names = [k for k in kernels if k.startswith("gemm_bf16")]
    if not names:
        return None
    dom = max(names, key=lambda k: kernels[k]["ms_per_step"])
    flops_per_launch = 2.0 * cfg.N * cfg.h * cfg.Vs
    ach = flops_per_launch / (kernels[dom]["ms_per_launch"] * 1e-3) / 1e12
    pmc = PMC_KIB.get(cfg.name, {}).get(dom)
    traffic = None if pmc is None else (PMC_FETCH_FACTOR * pmc[0] + PMC_WRITE_FACTOR * pmc[1]) * 1024.0
    # algorithmic bytes of one launch: both operands read once, the output written once (dH += also reads it)
    ab = {"gemm_bf16_fwd_stats": 2.0 * (cfg.N * cfg.h + cfg.Vs * cfg.h) + (2.0 * cfg.N * cfg.Vs if cfg.save_logits else 0.0),
          "gemm_bf16_dlogits": 2.0 * (cfg.N * cfg.h + cfg.Vs * cfg.h) + 2.0 * cfg.N * cfg.Vs,
          "gemm_bf16_dH": 2.0 * (cfg.N * cfg.Vs + cfg.Vs * cfg.h) + 8.0 * cfg.N * cfg.h,
          "gemm_bf16_dW": 2.0 * (cfg.N * cfg.Vs + cfg.N * cfg.h) + 4.0 * cfg.Vs * cfg.h}.get(dom)
    return {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": ach / BF16_MFMA_PEAK_TFLOPS, "flops_per_launch": flops_per_launch,
            "avg_launch_ms": kernels[dom]["ms_per_launch"], "traffic": traffic, "traffic_unit": "bytes per launch",
            "traffic_kind": "L2-miss / fabric bytes (2.0 x FETCH_SIZE + WRITE_SIZE)",
            "traffic_source": None if pmc is None else
            "not measured by this run: copied from the committed counter summary profiles/output_layer_%s.txt" % cfg.name,
            "algorithmic_bytes_per_launch": ab}


def cpu_sample_rows(cfg, requested):
    """Token rows of the CPU leg: all of them when the oracle's step is below about 10 TFLOP of fp64 work
    (some 10-30 s on the host of a GPU machine), else the largest multiple of 256 rows that is."""
    if requested > 0:
        return min(requested, cfg.N)
    rows = int(10e12 / (6.0 * cfg.h * cfg.V)) // 256 * 256
    return min(cfg.N, max(256, rows))


def cpu_baseline(cfg, sample_rows, host):
    """The oracle (Algorithm 1 on the CPU, fp64) on the first `sample_rows` token rows of the
    same inputs, all p shards, forward and backward.  The rate does not depend on the number of rows
    (every row costs 6 h V flops), so a sample gives the full workload's rate without extrapolation."""
    import synth_inputs as si
    from oracle import vp_oracle as oc
    try:
        from threadpoolctl import threadpool_info
        cores = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    sample_rows = cpu_sample_rows(cfg, sample_rows)
    H = si.as_f64(host[0][:sample_rows])
    labels = si.make_labels(cfg)[:sample_rows]
    Ws = [si.as_f64(w) for w in host[1]]
    t0 = time.perf_counter()
    out = oc.output_layer_alg1(H, Ws, labels)
    dt = time.perf_counter() - t0
    flops = 6.0 * sample_rows * cfg.h * cfg.V
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "seconds": dt, "loss_on_sample": float(out["loss"]),
            "sample": "oracle.output_layer_alg1 (NumPy fp64) on the first %d of %d token rows of %s, all %d shards, "
                      "forward + backward (%.1f TFLOP of the step's %.1f)" % (
                          sample_rows, cfg.N, cfg.name, cfg.p, flops / 1e12, cfg.model_flops / 1e12)}


def bench_embedding(vp, cfg, steps, warmup):
    import torch
    import synth_inputs as si
    ids = si.make_labels(cfg)
    g = torch.Generator(device="cuda")
    g.manual_seed(si.BASE_SEED + 5)
    tables = [(torch.randn((cfg.Vs, cfg.h), generator=g, device="cuda") * cfg.table_std).to(torch.bfloat16)
              for _ in range(cfg.p)]
    gout = (torch.randn((cfg.N, cfg.h), generator=g, device="cuda") * cfg.grad_std).to(torch.bfloat16)
    plan = vp.EmbeddingPlan(tables, dev(ids), gout)
    _, fwd_ms = time_steps(plan.forward, steps, warmup)
    _, bwd_ms = time_steps(plan.backward, steps, warmup)
    kern = profiled_steps(vp, lambda: (plan.forward(), plan.backward()), steps)
    uniq = len(np.unique(ids))
    fwd_bytes = cfg.p * cfg.N * cfg.h * 2 + cfg.N * cfg.h * 2 + cfg.p * cfg.N * 8
    bwd_bytes = cfg.N * cfg.h * 2 + 2 * uniq * cfg.h * 4 + cfg.p * cfg.N * 8
    return {
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "fwd_algorithmic_bytes": fwd_bytes, "bwd_algorithmic_bytes": bwd_bytes,
        "fwd_GBs": fwd_bytes / (fwd_ms * 1e-3) / 1e9, "bwd_GBs": bwd_bytes / (bwd_ms * 1e-3) / 1e9,
        "fwd_frac_hbm_peak": fwd_bytes / (fwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "bwd_frac_hbm_peak": bwd_bytes / (bwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "tokens_per_s_fwd_bwd": cfg.N / ((fwd_ms + bwd_ms) * 1e-3),
        "unique_ids": uniq, "kernels": kern,
        # dominant kernel of the input layer: the gather (algorithmic bytes of one shard over its launch time)
        "roofline": {"bound": "hbm", "kernel": "embed_fwd",
                     "achieved": fwd_bytes / cfg.p / (kern["embed_fwd"]["ms_per_launch"] * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": fwd_bytes / cfg.p / (kern["embed_fwd"]["ms_per_launch"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "bytes_per_launch": fwd_bytes / cfg.p, "avg_launch_ms": kern["embed_fwd"]["ms_per_launch"],
                     # FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 per launch (profiles/input_layer_cfg5_embedding.txt)
                     "traffic": (2.0 * 2524.4 + 65564.3) * 1024.0, "traffic_unit": "bytes per launch",
                     "traffic_kind": "L2-miss / fabric bytes (2.0 x FETCH_SIZE + WRITE_SIZE)",
                     "traffic_source": "not measured by this run: copied from the committed counter summary "
                                       "profiles/input_layer_cfg5_embedding.txt"},
    }


def mfma_sustained(vp, cfg):
    """What the matrix cores sustain with no memory traffic at all, for operands distributed like this
    configuration's H and W (and, for contrast, for zeros), over the instruction shapes and issue orders of
    vp_profile_mfma_variant: the power-limited envelope of any bf16 GEMM on these values.  TFLOP/s."""
    import torch
    blocks = 256
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    frags = 32
    x = torch.randn(frags, 256 * 8, generator=g, device="cuda")
    # fragments 0-3 of every group of 8 feed one operand (values like H), 4-7 the other (values like W)
    std = torch.tensor([cfg.h_std if (f % 8) < 4 else cfg.w_std for f in range(frags)], device="cuda")[:, None]
    hw = (x * std).to(torch.bfloat16).contiguous().view(-1)
    zeros = torch.zeros_like(hw)
    names = ["32x32x16 by columns", "32x32x16 snake", "32x32x16 k-chain of 2", "32x32x16 k-chain of 4",
             "16x16x32 by columns", "16x16x32 snake"]
    res = {}
    for label, src in (("operands_like_H_and_W", hw), ("zero_operands", zeros)):
        per = {}
        for v in range(vp.vp_profile_mfma_variant_count()):
            iters = 4096 // (1 if v < 2 else (2 if v == 2 else 4))
            for _ in range(3):
                vp.vp_profile_mfma_variant(src, out, iters, blocks, v)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flops = 0.0
            for _ in range(10):
                flops += vp.vp_profile_mfma_variant(src, out, iters, blocks, v)
            e1.record()
            torch.cuda.synchronize()
            per[names[v]] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
        res[label] = per
    res["envelope_like_H_and_W"] = max(res["operands_like_H_and_W"].values())
    return res


def gemm_timeline(vp, cfg, reps=3):
    """Itemised time budget of the fast GEMM launches of the last shard's passes S and T, from the phase stamps the
    kernel writes when its timeline is switched on (vp_profile_gemm_trace): per workgroup and output tile, the
    100 MHz counter and the shader clock at tile start, first operands landed, main loop done, epilogue done.
    All figures in microseconds per launch, averaged over workgroups (and over `reps` launches)."""
    import torch
    pl = make_output_plan(vp, cfg, seeded_numpy=False)
    for _ in range(2):
        pl.step()
    torch.cuda.synchronize()
    buf = torch.zeros(8 + 256 * 64 * 8, dtype=torch.int64, device="cuda")
    runs = ["gemm_bf16_fwd_stats", "gemm_bf16_dH", "gemm_bf16_dW"]
    if not cfg.save_logits:
        runs.insert(1, "gemm_bf16_dlogits")
    out = {}
    for name in runs:
        acc = []
        for _ in range(reps):
            # whole steps back to back, so that the traced launch (the last one of this kernel: every launch
            # overwrites the records) runs in the clock and cache state of the timed benchmark
            buf.zero_()
            vp.vp_profile_gemm_trace(buf, name)
            pl.step()
            pl.step()
            torch.cuda.synchronize()
            vp.vp_profile_gemm_trace(None)
            w = buf.cpu().numpy()
            grid, tiles, cap = int(w[0]), int(w[1]), int(w[2])
            rec = w[8:8 + grid * cap * 8].reshape(grid, cap, 4, 2).astype(np.float64)
            valid = rec[:, :, 3, 0] > 0                      # tiles this workgroup really had
            t = rec[:, :, :, 0] * 0.01                        # 100 MHz counter -> microseconds
            clk = rec[:, :, :, 1]
            t0 = t[:, 0, 0].min()
            end = np.where(valid, t[:, :, 3], 0).max(axis=1)  # last stamp of every workgroup
            span = end.max() - t0
            pro = np.where(valid, t[:, :, 1] - t[:, :, 0], 0).sum(axis=1)
            main = np.where(valid, t[:, :, 2] - t[:, :, 1], 0).sum(axis=1)
            epi = np.where(valid, t[:, :, 3] - t[:, :, 2], 0).sum(axis=1)
            start_skew = (t[:, 0, 0] - t0)
            main_clk = np.where(valid, clk[:, :, 2] - clk[:, :, 1], 0).sum() / max(main.sum(), 1e-9) / 1e3   # GHz
            acc.append({"span_us": span, "prologue_us": pro.mean(), "main_loop_us": main.mean(),
                        "epilogue_us": epi.mean(), "launch_skew_us": start_skew.mean(),
                        "idle_at_end_us": (end.max() - end).mean(),
                        "tiles": tiles, "workgroups": grid, "tiles_per_workgroup_max": cap,
                        "main_loop_clock_GHz": main_clk,
                        "epilogue_us_per_tile": np.where(valid, t[:, :, 3] - t[:, :, 2], 0).sum() / valid.sum(),
                        "main_loop_us_per_tile": np.where(valid, t[:, :, 2] - t[:, :, 1], 0).sum() / valid.sum()})
            # workgroups are dealt to the 8 XCDs round-robin: busy time (all phases) per XCD, and its spread
            busy = pro + main + epi
            acc[-1]["busy_us_min"] = busy.min()
            acc[-1]["busy_us_max"] = busy.max()
            for x in range(8):
                acc[-1]["busy_us_xcd%d" % x] = busy[x::8].mean()
        out[name] = {k: float(np.mean([a[k] for a in acc])) for k in acc[0]}
        flops = 2.0 * cfg.N * cfg.h * cfg.Vs
        out[name]["main_loop_tflops"] = flops / (out[name]["main_loop_us"] * 1e-6) / 1e12 * (
            out[name]["tiles"] / (out[name]["workgroups"] * out[name]["tiles_per_workgroup_max"]))
        out[name]["span_tflops"] = flops / (out[name]["span_us"] * 1e-6) / 1e12
    del pl
    torch.cuda.empty_cache()
    return out


def bench_barrier_overlap(vp, cfg, steps):
    """The barrier's on-device work (vp_combine_stats) on a side stream of default priority while the
    next pass S (a stand-in for the transformer work the paper overlaps its barriers with) runs on the
    main stream.  Reports the three wall times per iteration; hidden = both ~ compute alone."""
    import torch
    pl = make_output_plan(vp, cfg, seeded_numpy=False)
    pl.forward()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()

    def compute():
        vp.vp_output_fwd(pl.H, pl.W[0], pl.labels, 0, pl.local_max[0], pl.local_sumexp[0], pl.local_target[0],
                         pl.logits[0] if pl.logits is not None else None, pl.workspace)

    lm, ls, lt = pl.local_max.clone(), pl.local_sumexp.clone(), pl.local_target.clone()

    def barrier(stream=None):
        vp.vp_combine_stats(lm, ls, lt, pl.global_max, pl.global_sumexp, pl.loss_rows, pl.loss, stream)

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def both():
        side.wait_stream(main)
        barrier(side)
        compute()
        main.wait_stream(side)

    out = {"compute_ms": timed(compute), "barrier_ms": timed(barrier), "both_ms": timed(both)}
    out["hidden_fraction_of_barrier"] = max(0.0, min(1.0, (out["compute_ms"] + out["barrier_ms"] - out["both_ms"])
                                                   / out["barrier_ms"]))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg4_very_large_vocab", help="headline output-layer configuration")
    ap.add_argument("--only-headline", action="store_true", help="skip the per_config section")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise copy of 256 MiB (read 256 MiB, write 256 MiB) five times, so "
                         "that a counter run of this command carries a kernel of known HBM traffic")
    ap.add_argument("--cpu-sample-rows", type=int, default=0,
                    help="token rows of the CPU leg; 0 = as many as keep the oracle near 10 TFLOP of work")
    ap.add_argument("--timeline", action="store_true",
                    help="only print the itemised per-launch time budget (prologue / main loop / epilogue / idle) of "
                         "the GEMM kernels of --config, from the kernel's own phase stamps")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the p shards of a configuration run in sequence "
              "on it); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2411_05288_amd as vp
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    cfg = si.CONFIGS[args.config]
    if args.timeline:
        print(json.dumps({"timeline": gemm_timeline(vp, cfg), "config": cfg.name}))
        return
    if isinstance(cfg, si.EmbedConfig):
        # profiling aid: only the input-layer configuration, reported in GB/s of algorithmic bytes
        emb = bench_embedding(vp, cfg, args.steps, args.warmup)
        print(json.dumps({"metric": "input-layer gather + scatter-add, algorithmic HBM GB/s", "value": emb["fwd_GBs"],
                          "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "config": {"workload": "%s: V=%d p=%d Vs=%d h=%d N=%d" % (cfg.name, cfg.V, cfg.p, cfg.Vs,
                                                                                  cfg.h, cfg.N)},
                          "embedding": emb}))
        return
    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    host = (si.make_H(cfg), [si.make_W_shard(cfg, r) for r in range(cfg.p)])
    plan = make_output_plan(vp, cfg, seeded_numpy=True, host=host)
    wall_ms, ev_ms = time_steps(plan.step, args.steps, args.warmup)
    kernels = profiled_steps(vp, plan.step, args.steps)
    nums = output_numbers(cfg, wall_ms)
    loss = float(plan.loss.cpu()[0])
    del plan
    torch.cuda.empty_cache()

    per_config = {}
    if not args.only_headline:
        for name, c in si.CONFIGS.items():
            if name == args.config:
                per_config[name] = dict(nums, kernels=kernels, roofline=gemm_roofline(cfg, kernels))
                continue
            k_steps = max(3, min(args.steps, 10))
            if isinstance(c, si.EmbedConfig):
                per_config[name] = bench_embedding(vp, c, k_steps, 3)
                continue
            pl = make_output_plan(vp, c, seeded_numpy=False)
            w_ms, _ = time_steps(pl.step, k_steps, 2)
            kern = profiled_steps(vp, pl.step, k_steps)
            per_config[name] = dict(output_numbers(c, w_ms), kernels=kern, roofline=gemm_roofline(c, kern))
            del pl
            torch.cuda.empty_cache()
        # the Llama-like workload through Algorithm 2 (one barrier; same three products per shard), and the
        # barrier on a side stream next to a pass S of that workload
        c2 = si.CONFIGS["cfg2_llama"]
        pl = make_output_plan(vp, c2, seeded_numpy=False, algorithm=2)
        k_steps = max(3, min(args.steps, 10))
        w_ms, _ = time_steps(pl.step, k_steps, 2)
        kern = profiled_steps(vp, pl.step, k_steps)
        per_config[c2.name + "_algorithm2"] = dict(output_numbers(c2, w_ms), kernels=kern)
        del pl
        torch.cuda.empty_cache()
        per_config["barrier_overlap_" + c2.name] = bench_barrier_overlap(vp, c2, 50)
        torch.cuda.empty_cache()

    roof = gemm_roofline(cfg, kernels)
    if roof is not None:
        # context for frac: the MFMA-only rate this chip sustains on such operand values (power limited)
        roof["mfma_only_sustained_tflops"] = mfma_sustained(vp, cfg)
        roof["frac_of_sustained_envelope"] = roof["achieved"] / roof["mfma_only_sustained_tflops"]["envelope_like_H_and_W"]
    out = {
        "metric": METRIC,
        "value": nums["model_tflops"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "event_ms_per_step": ev_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "tokens_per_s": nums["tokens_per_s"],
        "tokens_per_s_per_shard_device": nums["tokens_per_s_per_shard_device"],
        "pct_bf16_mfma_peak": nums["pct_bf16_mfma_peak"],
        "hardware_tflops": nums["hardware_tflops"],
        "pct_bf16_mfma_peak_hardware_flops": 100.0 * nums["hardware_tflops"] / BF16_MFMA_PEAK_TFLOPS,
        "loss": loss,
        "config": {"workload": "%s: N=%d h=%d V=%d p=%d Vs=%d %s, logits %s; fwd + combine + bwd of all p shards "
                               "in sequence on one GPU" % (cfg.name, cfg.N, cfg.h, cfg.V, cfg.p, cfg.Vs, cfg.dtype,
                                                           "stored" if cfg.save_logits else "recomputed"),
                   "N": cfg.N, "h": cfg.h, "V": cfg.V, "p": cfg.p, "Vs": cfg.Vs,
                   "model_flops_per_step": cfg.model_flops},
        "roofline": roof,
        "kernels": kernels,
        "cpu_baseline": None if args.no_cpu_baseline else cpu_baseline(cfg, args.cpu_sample_rows, host),
        "per_config": per_config,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
