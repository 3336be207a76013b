#!/usr/bin/env python3
"""Benchmark of the IST hot path on one MI355X.

A "step" is one IST round over one set of synthetic mini-batches:
    ist_partition -> ist_subnet_steps (k local SGD steps on all S subnets) -> ist_merge
(Section 2.1 of the paper).  Inputs are resident in HBM before the timed region.
Prints ONE JSON line for the headline workload (default: the wide stress network, the
largest benchmark configuration a single GPU trains in bf16): subnet-SGD samples/s over
whole rounds, the roofline of the dominant kernel (timed with HIP events inside the
library, in a second pass over the same rounds), the CPU oracle timed on the host cores,
a timed 1 GiB device copy, and (key "other_workloads") the same throughput and phase
figures for the remaining benchmark configurations.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np
import torch

import ist_inputs as gen

PEAK = {"hbm_GBs": 8000.0, "bf16_TFLOPs": 2500.0, "f32_TFLOPs": 157.3}

# What a HIP-event bracket around one launch reads beyond the kernel's own duration (dispatch and
# marker latency), in microseconds: bracket average minus rocprofv3's kernel-trace average of the same
# kernels in the same run (2.3 .. 2.7 us for every kernel checked, see profiles/).
EVENT_OVERHEAD_US = 2.4

# HBM bytes per launch of the kernels that can dominate a workload, from two rocprofv3 --pmc runs of
# this script (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter reads for the 1 GiB
# device copies this script starts with; the runs and the scale factors are in profiles/.
# {workload: {kernel label: bytes}}.  A dominant kernel without an entry is an error: re-measure.
MEASURED_TRAFFIC = {
    # the tiny network: every kernel takes about 5 us and any of them can come out on top
    "cfg1": {
        "gemm_bwd_data_f32_64x64_t256": 0.113e6,                       # read 0.097 MB (47.4 KiB x 2.000) + written 0.016 MB
        "gemm_fwd_relu_f32_64x64_t256": 0.111e6,                       # read 0.095 MB + written 0.016 MB
        "gemm_fwd_logits_f32_64x64_t256": 0.069e6,                     # read 0.065 MB + written 0.004 MB
        "gemm_update_f32_64x64_t256_persistent_x3_bias": 0.411e6,      # read 0.339 MB + written 0.072 MB
        "softmax_xent": 0.084e6,                                       # read 0.079 MB + written 0.005 MB
    },
    # the three update products of a step and their bias updates in one launch:
    # read 77.05 MB (FETCH_SIZE 37623.1 KiB x 2.000) + written 34.16 MB (WRITE_SIZE 33360.7 KiB x 1.000)
    "cfg2": {"gemm_update_f32_64x64_t256_persistent_x3_bias": 111.21e6},
    # the two 128 x 128 update products of a step (first and second layer, averaged): read 54.76 MB (26738.7 KiB x 2.000)
    # + written 33.55 MB
    "cfg3": {"gemm_update_bf16_128x128_t256_persistent": 88.31e6},
    "cfg4": {
        # read 1797.7 MB (877819.1 KiB x 2.000) + written 894.8 MB (873813.3 KiB x 1.000), average of the three layers
        "gemm_update_bf16_256x256_t512_persistent": 2692.5e6,
        # read 1007.8 MB + written 67.1 MB (every operand byte fetched once: tiles are ordered by XCD)
        "gemm_fwd_relu_bf16_256x256_t512": 1074.9e6,
        # read 1275.4 MB + written 67.1 MB
        "gemm_bwd_data_bf16_256x256_t512": 1342.5e6,
    },
    "speech8192": {
        "gemm_fwd_relu_f32_64x64_t1024": 79.81e6,                      # read 75.62 MB + written 4.19 MB
        "gemm_update_f32_128x128_t256_persistent": 319.34e6,           # read 185.10 MB + written 134.24 MB
        "gemm_update_f32_64x64_t256_persistent_x3_bias": 229.90e6,     # read 161.54 MB + written 68.36 MB
    },
    "cfg5": {
        # backward launch of the wide output layer: read 1407.7 MB (687385.7 KiB x 2.000) + written 1421.3 MB
        # (1388001.0 KiB x 1.000): W_t read once and written once
        "k_wide_out_backward_bf16_c128": 2829.0e6,
        # statistics launch: read 1396.8 MB, written 0.6 MB
        "k_wide_out_stats_bf16_c128": 1397.4e6,
    },
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20, help="timed IST rounds")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg4", choices=sorted(gen.CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the short runs of the other benchmark configurations (key other_workloads)")
    ap.add_argument("--allow-unmeasured-traffic", action="store_true",
                    help="report roofline.traffic = null instead of failing when the dominant kernel has no "
                         "counter measurement on file (for runs that make that measurement)")
    ap.add_argument("--resample", action="store_true",
                    help="steady-state rounds: k local steps, then ist_resample (merge + partition by the next "
                         "permutation in one pass) instead of separate merge and partition calls")
    ap.add_argument("--normalize", action="store_true",
                    help="standardise hidden-neuron inputs over the mini-batch (Section 2.2 of the paper); "
                         "off for the headline metric")
    return ap.parse_args()


# ---------------------------------------------------------------- inputs on device
def device_problem(cfg: gen.ISTConfig, rounds_of_data: int, dev):
    """Weights, permutations and batches resident on the device.  Small workloads
    come from the NumPy generators (same arrays the parity tests use); the large
    ones are drawn with torch's device generator in the same distributions."""
    td = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    g = torch.Generator(device=dev)
    g.manual_seed(gen.SEED_BASE + 100 * cfg.idx)
    small = sum(cfg.dims[i] * cfg.dims[i + 1] for i in range(cfg.t)) <= 3e7
    if small:
        Ws, bs = gen.make_weights(cfg)
        dW = [torch.from_numpy(w).to(dev).to(td) for w in Ws]
        db = [torch.from_numpy(b).to(dev).to(td) for b in bs]
    else:
        dW, db = [], []
        for l in range(1, cfg.t + 1):
            a = float(np.sqrt(6.0 / (cfg.dims[l] + cfg.dims[l - 1])))
            W = torch.empty((cfg.dims[l], cfg.dims[l - 1]), dtype=td, device=dev)
            rows = max(1, (1 << 26) // cfg.dims[l - 1])
            for r0 in range(0, cfg.dims[l], rows):          # chunked: no fp32 copy of 8 GB layers
                r1 = min(cfg.dims[l], r0 + rows)
                W[r0:r1] = ((torch.rand((r1 - r0, cfg.dims[l - 1]), generator=g, device=dev) * 2 - 1) * a).to(td)
            dW.append(W)
            db.append(torch.zeros(cfg.dims[l], dtype=td, device=dev))
    perms = [[torch.randperm(cfg.dims[l], generator=g, device=dev).to(torch.int32)
              for l in range(1, cfg.t)] for _ in range(rounds_of_data)]
    rows = cfg.S * cfg.k * cfg.B
    data = []
    for r in range(rounds_of_data):
        if cfg.input == "csr":
            if r == 0:
                rp, ci, va, y = gen.make_csr_batches(cfg, r)
                data.append(dict(csr=(torch.from_numpy(rp).to(dev), torch.from_numpy(ci).to(dev),
                                      torch.from_numpy(va).to(dev).to(td)),
                                 y=torch.from_numpy(y.reshape(-1)).to(dev), X=None))
            else:
                data.append(data[0])
            continue
        if cfg.x_dist == "uniform":
            X = torch.rand((rows, cfg.dims[0]), generator=g, device=dev).to(td)
        else:
            X = torch.randn((rows, cfg.dims[0]), generator=g, device=dev).to(td)
        y = torch.randint(0, cfg.dims[-1], (rows,), generator=g, device=dev, dtype=torch.int32)
        data.append(dict(X=X, y=y, csr=None))
    return dW, db, perms, data


# ---------------------------------------------------------------- algorithmic work
def work_model(cfg: gen.ISTConfig):
    """Algorithmic FLOPs / bytes per kernel class for ONE round (all S subnets)."""
    S, B, k, t = cfg.S, cfg.B, cfg.k, cfg.t
    e = 4 if cfg.dtype == "f32" else 2
    R = [cfg.width(l) for l in range(1, t + 1)]
    Cc = [cfg.width(l - 1) for l in range(1, t + 1)]
    dense = [not (l == 1 and cfg.input == "csr") for l in range(1, t + 1)]
    p = [R[i] * Cc[i] for i in range(t)]
    fwd = sum(2 * B * p[i] * S for i in range(t) if dense[i]) * k
    bwd = sum(2 * B * p[i] * S for i in range(1, t)) * k
    upd = sum(2 * B * p[i] * S for i in range(t) if dense[i]) * k
    full = [cfg.dims[l] * cfg.dims[l - 1] for l in range(1, t + 1)]
    subs = [S * p[i] for i in range(t)]
    # line-granular minimum: partition reads every matrix once and writes the subnets;
    # merge reads the subnets and writes their lines, and for middle layers (both
    # endpoints hidden) has to read and rewrite every row to keep the unowned entries.
    part_bytes = sum(full[i] + subs[i] for i in range(t)) * e
    merge_bytes = sum((2 * full[i] + subs[i]) if 0 < i < t - 1 else (full[i] + subs[i])
                      for i in range(t)) * e
    useful = 2 * sum(subs) * e
    # weight bytes the k steps move when every product reads its operands once: forward read,
    # backward-data read (not layer 1), update read + write
    step_weight_bytes = sum((4 if i > 0 else 3) * subs[i] for i in range(t)) * e * k
    return dict(partition_bytes=part_bytes, merge_bytes=merge_bytes, useful_copy_bytes=useful,
                flops_round=fwd + bwd + upd, step_weight_bytes=step_weight_bytes)


def run_round(ctx, cfg, dW, db, perms, d, loss=None, resample=False):
    if resample:   # the subnets of this round were made by the previous round's re-sampling
        ctx.subnet_steps(d["y"], cfg.lr, cfg.k, cfg.B, X=d["X"], csr=d["csr"], loss_out=loss)
        ctx.resample(dW, db, perms)
        return
    ctx.partition(dW, db, perms)
    ctx.subnet_steps(d["y"], cfg.lr, cfg.k, cfg.B, X=d["X"], csr=d["csr"], loss_out=loss)
    ctx.merge(dW, db)


def cpu_baseline(cfg: gen.ISTConfig, budget_s: float):
    """The oracle, as it stands, timed on the host cores on a bounded sample."""
    from oracle import ist_oracle as orc
    threads = orc.omp_threads()
    if cfg.idx <= 2:
        Ws, bs = gen.make_weights(cfg)
        X, y = gen.make_dense_batches(cfg)
        n, t_tot = 0, 0.0
        while t_tot < budget_s and n < 50:
            perms = gen.make_perms(cfg, n)
            t0 = time.perf_counter()
            orc.ist_round(Ws, bs, perms, cfg.S, cfg.lr, cfg.k, cfg.dtype, y, X=X)
            t_tot += time.perf_counter() - t0
            n += 1
        return dict(value=n * cfg.S * cfg.k * cfg.B / t_tot, unit="samples/s", cores=threads,
                    kind="oracle", sample=f"{n} full rounds of {cfg.name} (partition + S*k local steps + merge)")
    # large workloads: one local step of one subnet at full subnet width.  A round is S*k such steps
    # plus partition and merge, so B / (time of that step) is the samples/s the oracle would sustain
    # over the S*k steps of a round.
    rng = np.random.default_rng(0)
    widths = [cfg.width(l) for l in range(cfg.t + 1)]
    Wl = [rng.uniform(-0.01, 0.01, (widths[l], widths[l - 1])) for l in range(1, cfg.t + 1)]
    bl = [np.zeros(widths[l]) for l in range(1, cfg.t + 1)]
    y = rng.integers(0, widths[-1], (1, cfg.B)).astype(np.int32)
    if cfg.input == "csr":
        c1 = gen.scaled(cfg, S=1, k=1)
        rp, ci, va, _ = gen.make_csr_batches(c1)
        kw = dict(csr=(rp, ci, va.astype(np.float64)))
    else:
        kw = dict(X=rng.standard_normal((1, cfg.B, widths[0])))
    # the same mini-batch again and again until the budget is used (at least 2 steps, at most 8)
    n, t_tot = 0, 0.0
    while n < 2 or (t_tot < budget_s and n < 8):
        t0 = time.perf_counter()
        orc.subnet_sgd(Wl, bl, y, cfg.lr, 1, cfg.dtype, **kw)
        t_tot += time.perf_counter() - t0
        n += 1
    dt = t_tot / n
    return dict(value=cfg.B / dt, unit="samples/s", cores=threads, kind="oracle",
                sample=f"{n} local steps of 1 subnet of {cfg.name} at full subnet width (B={cfg.B}), {dt:.2f} s each; "
                       f"a round is S*k = {cfg.S * cfg.k} such steps ({cfg.S * cfg.k * dt:.0f} s) plus partition and merge")


def timed_copy(dev, reps=5):
    """A plain 1 GiB device-to-device copy: reference dispatch for the rocprofv3 byte counters, and
    the copy rate this GPU reaches (bytes read + written per second)."""
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)       # 1 GiB
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(reps):
        dst.copy_(src)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / reps
    del src, dst
    return 2.0 * (1 << 30) / (ms * 1e-3) / 1e9


def roofline_of(cfg, kernels, workload_key, allow_unmeasured):
    """Roofline entry of the kernel label with the largest total time.  Which roof binds follows
    from the launch's arithmetic intensity (algorithmic flops / algorithmic bytes, both reported by
    the library per launch) against the ridge of the two peaks."""
    dom = kernels[0]
    sec = dom["avg_launch_us"] * 1e-6
    peak_t = PEAK["f32_TFLOPs"] if cfg.dtype == "f32" else PEAK["bf16_TFLOPs"]
    ridge = peak_t * 1e12 / (PEAK["hbm_GBs"] * 1e9)
    fl, by = dom["flops_per_launch"], dom["bytes_per_launch"]
    traffic = MEASURED_TRAFFIC.get(workload_key, {}).get(dom["label"])
    if traffic is None and not allow_unmeasured:
        raise SystemExit(f"bench.py: no measured HBM traffic on file for the dominant kernel '{dom['label']}' of "
                         f"{workload_key}: run the two rocprofv3 --pmc passes (FETCH_SIZE, WRITE_SIZE) and add the "
                         "entry to MEASURED_TRAFFIC, or pass --allow-unmeasured-traffic")
    common = dict(kernel=dom["label"], traffic=traffic, avg_launch_us=dom["avg_launch_us"],
                  flops_per_launch=fl, bytes_per_launch=by,
                  arithmetic_intensity=(fl / by if by > 0 else None), ridge_flop_per_byte=ridge)
    mfma = fl / sec / 1e12 if fl > 0 else None
    hbm = by / sec / 1e9 if by > 0 else None
    if fl > 0 and (by <= 0 or fl / by >= ridge):
        return dict(bound="mfma", achieved=mfma, peak=peak_t, unit="TFLOP/s", frac=mfma / peak_t,
                    hbm_GBs=hbm, **common)
    if by > 0:
        return dict(bound="hbm", achieved=hbm, peak=PEAK["hbm_GBs"], unit="GB/s", frac=hbm / PEAK["hbm_GBs"],
                    mfma_TFLOPs=mfma, mfma_frac=(mfma / peak_t if mfma else None), **common)
    return dict(bound="hbm", achieved=None, peak=PEAK["hbm_GBs"], unit="GB/s", frac=None, **common)


def run_workload(key, args, dev, steps, warmup, profile_pass, want_roofline):
    """Timed rounds, phase times and (optionally) the per-kernel pass of one workload."""
    from paper_1910_02120_amd import ISTContext
    cfg = gen.CONFIGS[key]
    nd = min(cfg.rounds, 4) if cfg.idx <= 3 else 1
    dW, db, perms, data = device_problem(cfg, nd, dev)
    ctx = ISTContext(cfg.dims, cfg.S, cfg.dtype, cfg.input, True, max_B=cfg.B, device="cuda:0",
                     normalize=args.normalize)
    loss = torch.zeros(cfg.S * cfg.k, dtype=torch.float32, device=dev)
    rs = args.resample
    if rs:
        ctx.partition(dW, db, perms[0])

    for i in range(warmup):
        run_round(ctx, cfg, dW, db, perms[i % nd], data[i % nd], loss, rs)
    torch.cuda.synchronize()
    first_loss = loss.cpu().numpy().reshape(cfg.S, cfg.k).copy()

    # ---------------- timed region: whole rounds ----------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        run_round(ctx, cfg, dW, db, perms[i % nd], data[i % nd], loss, rs)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_round = elapsed / steps * 1e3
    samples_round = cfg.S * cfg.k * cfg.B
    value = samples_round * steps / elapsed
    assert np.isfinite(loss.cpu().numpy()).all(), "non-finite loss"

    # ---------------- phase times (events on the stream the library launches on) ----------------
    st = torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    phase = np.zeros(3)
    reps = max(3, min(steps, 10))
    for i in range(reps):
        d = data[i % nd]
        if rs:   # phases: (nothing), steps, re-sampling
            ev[0].record(st)
            ev[1].record(st); ctx.subnet_steps(d["y"], cfg.lr, cfg.k, cfg.B, X=d["X"], csr=d["csr"])
            ev[2].record(st); ctx.resample(dW, db, perms[i % nd])
        else:
            ev[0].record(st); ctx.partition(dW, db, perms[i % nd])
            ev[1].record(st); ctx.subnet_steps(d["y"], cfg.lr, cfg.k, cfg.B, X=d["X"], csr=d["csr"])
            ev[2].record(st); ctx.merge(dW, db)
        ev[3].record(st); torch.cuda.synchronize()
        phase += [ev[j].elapsed_time(ev[j + 1]) for j in range(3)]
    phase /= reps
    wm = work_model(cfg)
    peak_t = PEAK["f32_TFLOPs"] if cfg.dtype == "f32" else PEAK["bf16_TFLOPs"]
    steps_s = phase[1] * 1e-3
    phases = {
        "partition_ms": phase[0], "steps_ms": phase[1], "merge_ms": phase[2],
        "steps_samples_per_s": samples_round / steps_s,
        "steps_TFLOPs": wm["flops_round"] / steps_s / 1e12,
        "steps_frac_of_mfma_peak": wm["flops_round"] / steps_s / 1e12 / peak_t,
        "steps_weight_GBs": wm["step_weight_bytes"] / steps_s / 1e9,
        "steps_frac_of_hbm_peak_weights_only": wm["step_weight_bytes"] / steps_s / 1e9 / PEAK["hbm_GBs"],
    }
    if not rs:
        phases.update({
            "partition_GBs_line_granular": wm["partition_bytes"] / (phase[0] * 1e-3) / 1e9,
            "merge_GBs_line_granular": wm["merge_bytes"] / (phase[2] * 1e-3) / 1e9,
            "partition_frac_of_hbm_peak": wm["partition_bytes"] / (phase[0] * 1e-3) / 1e9 / PEAK["hbm_GBs"],
            "merge_frac_of_hbm_peak": wm["merge_bytes"] / (phase[2] * 1e-3) / 1e9 / PEAK["hbm_GBs"],
            "partition_GBs_useful": wm["useful_copy_bytes"] / (phase[0] * 1e-3) / 1e9,
            "merge_GBs_useful": wm["useful_copy_bytes"] / (phase[2] * 1e-3) / 1e9,
        })

    # ---------------- per-kernel pass: the same rounds again, HIP events around every launch ----------------
    # (events are recorded by the library on the stream it launches on; bracketing every launch
    # widens the gaps between kernels, so this pass is kept apart from the throughput timing above)
    roof, classes, kernels = None, {}, []
    if profile_pass:
        ctx.profile_enable(True)
        ctx.profile_reset()
        pr = max(2, min(steps, 5))
        for i in range(pr):
            run_round(ctx, cfg, dW, db, perms[i % nd], data[i % nd], None, rs)
        prof = ctx.profile_read()
        kernels = ctx.profile_kernels()
        ctx.profile_enable(False)
        classes = {kname: dict(ms_per_round=ms / pr, launches_per_round=n / pr) for kname, (ms, n) in prof.items()}
        for kr in kernels:
            kr["ms_per_round"] = kr.pop("ms") / pr
            kr["avg_bracket_us"] = kr["ms_per_round"] * pr * 1e3 / kr["launches"]
            kr["avg_launch_us"] = max(kr["avg_bracket_us"] - EVENT_OVERHEAD_US, 0.1)
            kr["flops_per_launch"] = kr.pop("flops") / kr["launches"]
            kr["bytes_per_launch"] = kr.pop("bytes") / kr["launches"]
            kr["launches_per_round"] = kr.pop("launches") / pr
        kernels.sort(key=lambda kr: -kr["ms_per_round"])
        if want_roofline:
            roof = roofline_of(cfg, kernels, key, args.allow_unmeasured_traffic)
    ctx.close()
    del ctx, dW, db, perms, data, loss
    gc.collect()
    torch.cuda.empty_cache()
    return dict(cfg=cfg, value=value, ms_round=ms_round, phases=phases, classes=classes, kernels=kernels,
                roofline=roof, first_loss=first_loss, resample_ms=(phase[2] if rs else None))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: all S subnets are resident on a single MI355X and there is "
              "no multi-GPU path in this build; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = torch.device("cuda:0")
    copy_GBs = timed_copy(dev)

    r = run_workload(args.workload, args, dev, args.steps, args.warmup, not args.no_profile_pass, True)
    cfg = r["cfg"]

    others = {}
    if not args.no_others:
        for key in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
            if key == args.workload:
                continue
            n = 20 if key in ("cfg1", "cfg2", "cfg3") else 5
            o = run_workload(key, args, dev, n, 2, False, False)
            ph = o["phases"]
            tot = ph["partition_ms"] + ph["steps_ms"] + ph["merge_ms"]
            others[o["cfg"].name] = {
                "samples_per_s": o["value"], "ms_per_round": o["ms_round"], "rounds_timed": n, "dtype": o["cfg"].dtype,
                "phase_fraction": {"partition": ph["partition_ms"] / tot, "steps": ph["steps_ms"] / tot,
                                   "merge": ph["merge_ms"] / tot},
                "phases": ph,
            }

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, args.cpu_seconds)

    first_loss = r["first_loss"]
    out = {
        "metric": "subnet-SGD samples/sec (all S subnets, 1 GPU) + partition/merge GB/s",
        "value": r["value"], "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_round"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "dims": list(cfg.dims), "S": cfg.S, "B": cfg.B, "k": cfg.k,
                   "lr": cfg.lr, "input": cfg.input, "normalize": bool(args.normalize), "resample": bool(args.resample),
                   "step": "one IST round: partition + k local SGD steps on S subnets + merge"},
        "phases": r["phases"],
        "resample_ms": r["resample_ms"],
        "kernel_classes": r["classes"],
        "kernels": r["kernels"][:8],
        "event_overhead_us": EVENT_OVERHEAD_US,
        "measured_copy_GBs": copy_GBs,
        "measured_copy_frac_of_hbm_peak": copy_GBs / PEAK["hbm_GBs"],
        "roofline": r["roofline"],
        "cpu_baseline": cpu,
        "other_workloads": others,
        "loss_first_round": [float(first_loss[:, 0].mean()), float(first_loss[:, -1].mean())],
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
