#!/usr/bin/env python3
"""Benchmark of the M-AVG hot path on one MI355X.

A "step" is one meta round of Algorithm 1 on synthetic data: K local
minibatch-SGD steps on each of the P learners (kavg_local_steps) followed by
the fused meta step (kavg_meta_update).  Prints ONE JSON line:

  value       learner-samples/s = P*K*B*steps / wall time of the timed rounds
              (inputs resident in device memory before the clock starts)
  roofline    the dominant kernel class of the round, its algorithmic bytes
              per launch over its average launch duration (HIP events on the
              library's stream, recorded inside the timed region)
  cpu_baseline  the CPU oracle, as it stands, on a bounded sample of the same
              workload (reported for context, not a target)
  other_workloads  the remaining training workloads, same measurements,
              noisy_wide once more with deferred weight updates, and the
              convolutional workload (times per kernel class, flops against the MFMA peak)
  meta_update the fused meta step alone on the meta-only workload
              (P=64 replicas of an 11.2M-parameter fp32 vector), GB/s vs HBM peak
  ceilings    what this device streams (read, write, 1:1) and multiplies (bf16
              MFMA chain) with nothing else to do, from the library's probe kernels

The headline workload is `large`, the largest single-GPU configuration.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2110_00625_amd import kavg, synth                                   # noqa: E402
from paper_2110_00625_amd.configs import (WORKLOADS, CONV_WORKLOADS, META_ONLY, flops_per_learner_step,  # noqa: E402
                                          conv_flops_per_learner_step, num_params)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
FP32_PEAK_TFLOPS = 157.3


def class_model(w, learner_momentum=False):
    """Algorithmic bytes and flops of one launch-set (all layers) of each kernel
    class for ONE local step of all P learners, and of one meta pass."""
    P, B, d = w.P, w.B, w.dims
    L = len(d) - 1
    bf = w.dtype == kavg.KAVG_BF16
    e = 2 if bf else 4                      # operand element size
    vel = 8 if learner_momentum else 0      # velocity read + write per parameter
    ldz = (d[L] + 7) // 8 * 8
    head = d[L] <= 16       # few classes: the last layer's forward and data gradient run inside the loss kernel
    by = {"forward": 0, "backward": 0, "update": 0}
    fl = {"forward": 0, "backward": 0, "update": 0}
    for l in range(1, L + 1):
        wsz = d[l] * d[l - 1]
        ld_out = ldz if l == L else d[l]
        if head and l == L:     # both head kernels: A_{L-1} twice, W_L, dZ_L, dZ_{L-1}, master/shadow of W_L
            by["head"] = P * (2 * e * B * d[l - 1] + e * wsz + 3 * e * B * ld_out + e * B * d[l - 1]
                              + (8 + vel) * wsz + (8 + vel) * d[l])
            fl["head"] = P * 6 * B * wsz
            continue
        # forward: weights once, bias, input rows, output rows
        by["forward"] += P * (e * wsz + 4 * d[l] + e * B * d[l - 1] + (4 * B * ld_out if l == L else e * B * d[l]))
        fl["forward"] += P * 2 * B * wsz
        # update: master read + write (fp32, or its two 16-bit planes: 4 bytes either way), bias read +
        # write, dZ and A once
        by["update"] += P * ((8 + vel) * wsz + (8 + vel) * d[l] + e * B * (ld_out + d[l - 1]))
        fl["update"] += P * 2 * B * wsz
        if l > 1:   # data gradient: weights once, dZ_l, mask read, dZ_{l-1} written
            by["backward"] += P * (e * wsz + e * B * ld_out + 2 * e * B * d[l - 1])
            fl["backward"] += P * 2 * B * wsz
    n = num_params(d)
    by["meta"] = (2 * P + 4) * 4 * n
    fl["meta"] = (2 * P + 3) * n
    return by, fl


KERNEL_SOURCES = ("gemm_bf16.hip", "meta_update.hip", "head.hip", "sampling_loss.hip", "split.h", "kavg_internal.h")


def source_digest():
    """Digest of the files that define the kernels whose traffic is recorded under profiles/."""
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2110_00625_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def stored_traffic(workload, kernel_class):
    """HBM bytes per launch from the rocprofv3 --pmc runs recorded under profiles/,
    or None when absent or taken from other kernel sources than the current ones."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic.json.txt")
    if not os.path.exists(path):
        return None
    try:
        rec = json.load(open(path))
    except Exception:
        return None
    if rec.get("source_digest") != source_digest():
        return None
    return rec.get("traffic_bytes_per_launch", {}).get(workload, {}).get(kernel_class)


def cpu_baseline(w, data, beta=0.0, target_flops=3.0e12):
    """The oracle, as it stands, on whole meta rounds of this workload restricted to its first
    learners (learners are independent between meta steps, so the rate per learner-sample is that
    of the full workload).  The sample is sized to about target_flops of arithmetic (some tens of
    seconds on the host), never less than one learner for one round."""
    from threadpoolctl import threadpool_info
    from oracle import mavg_oracle as O
    per_learner_round = w.K * flops_per_learner_step(w.dims, w.B)
    learners = max(1, min(w.P, int(target_flops / per_learner_round)))
    rounds = max(1, min(3, int(target_flops / (learners * per_learner_round))))
    o = O.MAvgOracle(learners, w.K, w.lr, w.mu, w.dims, w.B, bf16=(w.dtype == kavg.KAVG_BF16),
                     index_seed=w.seeds["index"], learner_momentum=beta)
    o.set_data(data["X32"], data["y"])
    o.set_params(data["w0"])
    t0 = time.perf_counter()
    for _ in range(rounds):
        o.local_steps()
        o.meta_update()
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    return {"value": rounds * learners * w.K * w.B / dt, "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "threads": "BLAS threads of numpy's matmul (the rest of the oracle is single-threaded numpy)",
            "host_cores_available": len(os.sched_getaffinity(0)),
            "sample": "%d meta round(s) of %s with %d of its %d learners: %d learner-samples, %.1f s of wall time" % (
                rounds, w.name, learners, w.P, rounds * learners * w.K * w.B, dt)}


def bench_meta_only(torch, passes=200, warmup=5):
    w = META_ONLY
    n, P = w.flat_n, w.P
    stride = (n + 63) // 64 * 64
    g = torch.Generator(device="cuda").manual_seed(w.seeds["data"])
    base = torch.randn(n, device="cuda", generator=g) * 0.05
    v = torch.randn(n, device="cuda", generator=g) * 1e-3
    reps = torch.empty((P, stride), device="cuda")
    reps[:, :n] = base + torch.randn((P, n), device="cuda", generator=g) * 1e-3
    wt = base.clone()
    for _ in range(warmup):
        kavg.kavg_meta_update_flat(wt, v, reps, w.mu)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(passes):
        kavg.kavg_meta_update_flat(wt, v, reps, w.mu)
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / passes
    bytes_pass = (2 * P + 4) * 4 * n
    gbs = bytes_pass / (ms * 1e-3) / 1e9
    # context: what a plain device copy of the same replica block reaches on this machine (same 1:1
    # read/write mix as the meta step)
    dst = torch.empty_like(reps)
    for _ in range(3):
        dst.copy_(reps)
    ev0.record()
    for _ in range(20):
        dst.copy_(reps)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * reps.numel() * 4 / (ev0.elapsed_time(ev1) / 20 * 1e-3) / 1e9
    return {"plain_copy_GBps": copy_gbs, "workload": "meta_only: P=%d replicas of n=%d fp32, mu=%.2f, %d passes" % (P, n, w.mu, passes),
            "ms_per_pass": ms, "bytes_per_pass": bytes_pass, "GBps": gbs, "peak_GBps": HBM_PEAK_GBS,
            "frac": gbs / HBM_PEAK_GBS}


def bench_ceilings(torch, nbytes=1 << 31, reps=10):
    """What this device reaches with the meta step's access pattern and nothing else to do
    (kavg_probe): read-only, write-only and 1:1 read/write streams over `nbytes`, and a chain of
    bf16 matrix-core instructions without memory traffic."""
    a = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
    b = torch.empty_like(a)
    sink = torch.zeros(1, device="cuda")
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    out = {"bytes": nbytes, "pattern": "16-byte non-temporal accesses, 16 interleaved rows per lane"}
    for name, kind in (("read_GBps", kavg.PROBE_READ), ("write_GBps", kavg.PROBE_WRITE), ("copy_GBps", kavg.PROBE_COPY)):
        for _ in range(2):
            kavg.kavg_probe(kind, a, b, sink=sink)
        ev0.record()
        work = 0.0
        for _ in range(reps):
            work += kavg.kavg_probe(kind, a, b, sink=sink)
        ev1.record()
        torch.cuda.synchronize()
        out[name] = work / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    kavg.kavg_probe(kavg.PROBE_MFMA, iters=2000, sink=sink)
    ev0.record()
    work = kavg.kavg_probe(kavg.PROBE_MFMA, iters=20000, sink=sink)
    ev1.record()
    torch.cuda.synchronize()
    out["mfma_bf16_TFLOPs"] = work / (ev0.elapsed_time(ev1) * 1e-3) / 1e12
    return out


def run_workload(torch, w, steps, warmup, learner_momentum=0.0, copy_calibration=False, refresh=1):
    """`warmup` untimed meta rounds (every kernel class bracketed by HIP events: the per-class
    breakdown), then `steps` timed ones with inputs resident in device memory.  Returns the
    measurements and the host-side inputs (for the CPU baseline)."""
    data = synth.make_workload_inputs(w)
    bf = w.dtype == kavg.KAVG_BF16
    g = kavg.MAvg(w.P, w.K, w.lr, w.mu, w.dims, w.B, w.dtype, index_seed=w.seeds["index"])
    X = torch.from_numpy(data["Xbits"].view(np.int16) if bf else data["X32"]).cuda()
    y = torch.from_numpy(data["y"]).cuda()
    g.set_data(X, y)
    if learner_momentum > 0:
        g.set_learner_momentum(learner_momentum)
    g.set_params(data["w0"])
    if refresh > 1:
        g.set_refresh(min(refresh, w.K))

    if copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                                  # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst

    fused = g.fused        # small fp32 model: indices, K steps and losses are ONE launch, bracketed as "forward"
    classes = ["index", "forward", "loss", "backward", "update", "meta", "head", "correction"]
    bracketed = max(warmup, 1)
    if warmup >= 2:                      # the first round pays one-off costs (code upload, cold caches): untimed, unbracketed
        g.local_steps()
        g.meta_update()
        bracketed = warmup - 1
    g.profile(classes)
    for _ in range(bracketed):
        g.local_steps()
        g.meta_update()
    breakdown = g.profile_read()
    heavy = max(("forward", "backward", "update", "meta"), key=lambda c: breakdown[c][0])
    if fused:
        heavy = "forward"

    # timed region: only the dominant class carries events, and only one launch in EVERY of it
    # (an event pair costs ~10 us of stream time; 17 is coprime with the launches per round, so
    # the sample walks evenly over the layers)
    EVERY = 17
    g.profile([heavy], every=EVERY)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        g.local_steps()
        g.meta_update()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = g.profile_read()
    g.profile([])
    loss_last = float(g.losses()[-1].mean())
    g.close()
    del X, y
    torch.cuda.empty_cache()

    samples = w.P * w.K * w.B * steps
    by, fl = class_model(w, learner_momentum > 0)
    ms_sampled, sampled = prof[heavy]
    per_round = w.K if heavy != "meta" else 1
    n_layers = len(w.dims) - 1
    head = w.dims[-1] <= 16
    per_step = {"meta": 1, "update": n_layers - (1 if head else 0), "forward": n_layers - (1 if head else 0),
                "backward": n_layers - 1 - (1 if head else 0)}[heavy]
    launches = per_step * per_round * steps
    if fused:                                                  # the one launch does the work of every class of the K steps
        launches = steps
        by = dict(by, forward=sum(by[c] for c in ("forward", "backward", "update")) * w.K)
        fl = dict(fl, forward=sum(fl[c] for c in ("forward", "backward", "update")) * w.K)
        per_round = 1
    ms_heavy = ms_sampled / max(sampled, 1) * launches         # sampled mean launch time x all launches of the class
    bytes_heavy = by[heavy] * per_round * steps                # all launches of the class in the timed region
    flops_heavy = fl[heavy] * per_round * steps
    t_hbm = bytes_heavy / (HBM_PEAK_GBS * 1e9)
    peak_flops = (MFMA_BF16_PEAK_TFLOPS if bf else FP32_PEAK_TFLOPS) * 1e12
    t_mfma = flops_heavy / peak_flops
    if t_hbm >= t_mfma or heavy == "meta":
        achieved = bytes_heavy / (ms_heavy * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS}
    else:
        achieved = flops_heavy / (ms_heavy * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": peak_flops / 1e12, "unit": "TFLOP/s",
                "frac": achieved / (peak_flops / 1e12)}
    roof.update({"traffic": stored_traffic(w.name, heavy) if refresh == 1 else None, "kernel_class": heavy, "launches": launches,
                 "launches_timed": sampled, "avg_launch_us": 1e3 * ms_heavy / max(launches, 1),
                 "algorithmic_bytes_per_launch": bytes_heavy / max(launches, 1),
                 "flops_per_launch": flops_heavy / max(launches, 1)})

    # all dense products of the local steps against the matrix-core peak (context for the roofline)
    gemm_ms = sum(breakdown[c][0] for c in ("forward", "backward", "update"))
    gemm_flops = (fl["forward"] if fused else sum(fl[c] for c in ("forward", "backward", "update")) * w.K) * bracketed
    local_mfma = {"achieved_TFLOPs": gemm_flops / (gemm_ms * 1e-3) / 1e12, "peak_TFLOPs": peak_flops / 1e12,
                  "frac": gemm_flops / (gemm_ms * 1e-3) / peak_flops,
                  "note": "forward+backward+update launches of the profiled warm-up rounds"}
    # every class against the HBM roofline, from the bracketed warm-up rounds
    per_class = {}
    for c in classes:
        ms_c = breakdown[c][0] / bracketed
        if c in by and ms_c > 0 and (refresh == 1 or c == "meta") and not (fused and c != "meta"):
            rounds_bytes = by[c] * (1 if c == "meta" else w.K)
            per_class[c] = {"ms_per_round": ms_c, "hbm_frac": rounds_bytes / (ms_c * 1e-3) / 1e9 / HBM_PEAK_GBS}
        else:
            per_class[c] = {"ms_per_round": ms_c}
    res = {
        "value": samples / dt, "ms_per_step": 1e3 * dt / steps, "steps": steps, "warmup": warmup,
        "dtype": "bf16" if bf else "f32",
        "config": {"workload": "%s: P=%d K=%d B=%d mu=%g lr=%g MLP %s, N=%d%s%s" % (
            w.name, w.P, w.K, w.B, w.mu, w.lr, "-".join(map(str, w.dims)), w.N,
            ", learner momentum %g" % learner_momentum if learner_momentum > 0 else "",
            ", replicas refreshed every %d local steps (deferred updates)" % min(refresh, w.K) if refresh > 1 else ""),
            "step": "one meta round = K local steps on P learners + fused meta step" + (
                "; the K local steps run as ONE launch (model on chip)" if fused else ""),
            "samples_per_step": w.P * w.K * w.B, "flops_per_step": flops_per_learner_step(w.dims, w.B) * w.P * w.K},
        "roofline": roof, "local_steps_mfma": local_mfma, "kernel_classes": per_class, "final_mean_loss": loss_last,
    }
    return res, data


def run_conv_workload(torch, w, steps, warmup):
    """The convolutional workload: `warmup` rounds with every kernel class bracketed, then `steps`
    timed rounds without events."""
    data = synth.make_conv_workload_inputs(w)
    g = kavg.MAvg(w.P, w.K, w.lr, w.mu, w.dims, w.B, kavg.KAVG_BF16, index_seed=w.seeds["index"],
                  conv=(w.H, w.W, w.channels))
    X = torch.from_numpy(data["Xbits"].view(np.int16).reshape(w.N, w.H, w.W, w.channels[0])).cuda()
    g.set_data(X, torch.from_numpy(data["y"]).cuda())
    g.set_params(data["w0"])
    classes = ["index", "forward", "loss", "backward", "update", "meta", "head"]
    bracketed = max(warmup, 1)
    if warmup >= 2:                      # the first round pays one-off costs: untimed, unbracketed
        g.local_steps()
        g.meta_update()
        bracketed = warmup - 1
    g.profile(classes)
    for _ in range(bracketed):
        g.local_steps()
        g.meta_update()
    breakdown = g.profile_read()
    g.profile([])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        g.local_steps()
        g.meta_update()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    loss_first, loss_last = float(g.losses()[0].mean()), float(g.losses()[-1].mean())
    g.close()
    del X
    torch.cuda.empty_cache()
    flops = conv_flops_per_learner_step(w.H, w.W, w.channels, w.dims, w.B) * w.P * w.K
    return {
        "value": w.P * w.K * w.B * steps / dt, "ms_per_step": 1e3 * dt / steps, "steps": steps, "dtype": "bf16",
        "config": {"workload": "%s: P=%d K=%d B=%d mu=%g lr=%g, %dx%d images, 3x3 convolutions %s, mean over positions, "
                               "MLP %s, N=%d" % (w.name, w.P, w.K, w.B, w.mu, w.lr, w.H, w.W, "-".join(map(str, w.channels)),
                                                 "-".join(map(str, w.dims)), w.N),
                   "samples_per_step": w.P * w.K * w.B, "flops_per_step": flops},
        "flops_fraction_of_bf16_mfma_peak": flops / (dt / steps) / (MFMA_BF16_PEAK_TFLOPS * 1e12),
        "achieved_TFLOPs": flops / (dt / steps) / 1e12,
        "kernel_classes": {c: {"ms_per_round": breakdown[c][0] / bracketed} for c in classes},
        "final_mean_loss": loss_last,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large", choices=[k for k, v in WORKLOADS.items() if v.dims] + list(CONV_WORKLOADS),
                    help="the headline workload (default: the largest single-GPU configuration)")
    ap.add_argument("--also", default="noisy_wide,cifar_mlp,tiny",
                    help="comma-separated further workloads reported under other_workloads ('' = none)")
    ap.add_argument("--refresh", type=int, default=1,
                    help="headline workload: bring the stored replicas up to date every m local steps (deferred "
                         "updates; 1 = every step, the default)")
    ap.add_argument("--also-deferred", default="noisy_wide:16",
                    help="workload:m pairs also run with deferred updates and reported under other_workloads ('' = none)")
    ap.add_argument("--also-conv", default="cifar_conv",
                    help="convolutional workloads reported under other_workloads ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-meta-only", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true")
    ap.add_argument("--learner-momentum", type=float, default=0.0,
                    help="heavy-ball momentum inside every learner (variant of Section 2; default off = Algorithm 1)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy (reference dispatch for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all P learners on one MI355X); --gpus %d is not "
              "supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    kavg.load_library()
    if args.workload in CONV_WORKLOADS:
        # the convolutional workload as the line's subject: its dense products are bound by the matrix cores
        r = run_conv_workload(torch, CONV_WORKLOADS[args.workload], args.steps, args.warmup)
        dense_ms = sum(r["kernel_classes"][c]["ms_per_round"] for c in ("forward", "backward", "update"))
        ach = r["config"]["flops_per_step"] / (dense_ms * 1e-3) / 1e12
        out = {"metric": "learner-samples/sec (all P on 1 GPU); meta-update GB/s vs HBM peak",
               "value": r["value"], "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
               "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
               "dtype": "bf16", "data": "synthetic", "config": r["config"],
               "roofline": {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                            "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                            "kernel_class": "forward+backward+update of the bracketed warm-up rounds"},
               "kernel_classes": r["kernel_classes"], "final_mean_loss": r["final_mean_loss"]}
        print(json.dumps(out))
        return
    w = WORKLOADS[args.workload]
    res, data = run_workload(torch, w, args.steps, args.warmup, args.learner_momentum, args.copy_calibration,
                             refresh=args.refresh)
    out = {
        "metric": "learner-samples/sec (all P on 1 GPU); meta-update GB/s vs HBM peak",
        "value": res["value"], "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": res["dtype"], "data": "synthetic", "config": res["config"],
        "roofline": res["roofline"], "local_steps_mfma": res["local_steps_mfma"],
        "kernel_classes": res["kernel_classes"], "final_mean_loss": res["final_mean_loss"],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, data, args.learner_momentum)
    del data
    others = {}
    for name in [x for x in args.also.split(",") if x and x != args.workload]:
        r, _ = run_workload(torch, WORKLOADS[name], min(args.steps, 20), min(args.warmup, 3))
        others[name] = {k: r[k] for k in ("value", "ms_per_step", "steps", "dtype", "config", "roofline",
                                          "local_steps_mfma", "kernel_classes")}
    for pair in [x for x in args.also_deferred.split(",") if x]:
        name, m = pair.split(":")
        r, _ = run_workload(torch, WORKLOADS[name], min(args.steps, 20), min(args.warmup, 3), refresh=int(m))
        # deferred updates change which bytes and flops a class moves; only times are reported for it
        others["%s, replicas refreshed every %s steps" % (name, m)] = {
            "value": r["value"], "ms_per_step": r["ms_per_step"], "steps": r["steps"], "dtype": r["dtype"],
            "config": r["config"],
            "flops_fraction_of_bf16_mfma_peak": r["config"]["flops_per_step"] / (r["ms_per_step"] * 1e-3) / (MFMA_BF16_PEAK_TFLOPS * 1e12),
            "kernel_classes": {k: {"ms_per_round": v["ms_per_round"]} for k, v in r["kernel_classes"].items()}}
    for name in [x for x in args.also_conv.split(",") if x]:
        others[name] = run_conv_workload(torch, CONV_WORKLOADS[name], min(args.steps, 10), min(args.warmup, 2))
    if others:
        out["other_workloads"] = others
    if not args.no_meta_only:
        out["meta_update"] = bench_meta_only(torch)
    if not args.no_ceilings:
        out["ceilings"] = bench_ceilings(torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
