#!/usr/bin/env python3
"""Benchmark of the IST hot path on one MI355X.

A "step" is one IST round over one set of synthetic mini-batches:
    ist_partition -> ist_subnet_steps (k local SGD steps on all S subnets) -> ist_merge
(Section 2.1 of the paper).  Inputs are resident in HBM before the timed region.
Prints ONE JSON line: subnet-SGD samples/s over whole rounds, plus the roofline
of the dominant kernel class (timed with HIP events inside the library, in a
second pass of the same region) and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
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
# kernels in the same run (2.3 .. 2.7 us for every kernel of the default workload, see profiles/).
EVENT_OVERHEAD_US = 2.4

# HBM bytes per launch of the dominant kernel, from two rocprofv3 --pmc runs of this script
# (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter reads for the 1 GiB copy of
# --calibrate-copy; the runs and the scale factors are in profiles/.  {workload: {kernel label: bytes}}
MEASURED_TRAFFIC = {
    # the three update products of a step and their bias updates in one launch:
    # read 77.05 MB (FETCH_SIZE 37621.5 KiB x 2.000) + written 34.16 MB (WRITE_SIZE 33360.7 KiB x 1.000)
    "cfg2": {"gemm_update_f32_64x64_t256_persistent_x3_bias": 111.21e6},
    # read 1684.4 MB (822492.4 KiB x 2.000) + written 894.8 MB (873813.3 KiB x 1.000)
    "cfg4": {"gemm_update_bf16_256x256_t512_persistent": 2579.2e6},
    # second cross-entropy pass (dz^T): read 2840.2 MB (1386890.0 KiB x 2.000) + written 2839.0 MB (2772420.1 KiB x 1.000)
    "cfg5": {"gemm_fwd_dzt_bf16_128x128_t256_persistent": 5679.2e6},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20, help="timed IST rounds")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg2", choices=sorted(gen.CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--resample", action="store_true",
                    help="steady-state rounds: k local steps, then ist_resample (merge + partition by the next "
                         "permutation in one pass) instead of separate merge and partition calls")
    ap.add_argument("--normalize", action="store_true",
                    help="standardise hidden-neuron inputs over the mini-batch (Section 2.2 of the paper); "
                         "off for the headline metric")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run a plain device copy of 1 GiB three times (reference dispatch for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
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
    return dict(gemm_forward=("mfma", fwd), gemm_backward_data=("mfma", bwd), gemm_update=("mfma", upd),
                partition_copy=("hbm", part_bytes), merge_copy=("hbm", merge_bytes),
                useful_copy_bytes=useful, flops_round=fwd + bwd + upd)


RESAMPLE = False


def run_round(ctx, cfg, dW, db, perms, d, loss=None):
    if RESAMPLE:   # the subnets of this round were made by the previous round's re-sampling
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
    # large workloads: one local step of one subnet at full width, scaled by nothing:
    # samples/s of that step is what S*k such steps would sustain
    rng = np.random.default_rng(0)
    widths = [cfg.width(l) for l in range(cfg.t + 1)]
    Wl = [rng.uniform(-0.01, 0.01, (widths[l], widths[l - 1])) for l in range(1, cfg.t + 1)]
    bl = [np.zeros(widths[l]) for l in range(1, cfg.t + 1)]
    y = rng.integers(0, widths[-1], (1, cfg.B)).astype(np.int32)
    if cfg.input == "csr":
        c1 = gen.scaled(cfg, S=1, k=1)
        rp, ci, va, _ = gen.make_csr_batches(c1)
        t0 = time.perf_counter()
        orc.subnet_sgd(Wl, bl, y, cfg.lr, 1, cfg.dtype, csr=(rp, ci, va.astype(np.float64)))
    else:
        X = rng.standard_normal((1, cfg.B, widths[0]))
        t0 = time.perf_counter()
        orc.subnet_sgd(Wl, bl, y, cfg.lr, 1, cfg.dtype, X=X)
    dt = time.perf_counter() - t0
    return dict(value=cfg.B / dt, unit="samples/s", cores=threads, kind="oracle",
                sample=f"1 local step of 1 subnet of {cfg.name} at full subnet width (B={cfg.B})")


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: all S subnets are resident on a single MI355X and there is "
              "no multi-GPU path in this build; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    from paper_1910_02120_amd import ISTContext
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = torch.device("cuda:0")
    cfg = gen.CONFIGS[args.workload]
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)       # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    nd = min(cfg.rounds, 4) if cfg.idx <= 3 else 1
    dW, db, perms, data = device_problem(cfg, nd, dev)
    ctx = ISTContext(cfg.dims, cfg.S, cfg.dtype, cfg.input, True, max_B=cfg.B, device="cuda:0",
                     normalize=args.normalize)
    loss = torch.zeros(cfg.S * cfg.k, dtype=torch.float32, device=dev)
    global RESAMPLE
    RESAMPLE = args.resample
    if RESAMPLE:
        ctx.partition(dW, db, perms[0])

    for i in range(args.warmup):
        run_round(ctx, cfg, dW, db, perms[i % nd], data[i % nd], loss)
    torch.cuda.synchronize()
    first_loss = loss.cpu().numpy().reshape(cfg.S, cfg.k).copy()

    # ---------------- timed region: K whole rounds ----------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run_round(ctx, cfg, dW, db, perms[i % nd], data[i % nd], loss)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_round = elapsed / args.steps * 1e3
    samples_round = cfg.S * cfg.k * cfg.B
    value = samples_round * args.steps / elapsed
    assert np.isfinite(loss.cpu().numpy()).all(), "non-finite loss"

    # ---------------- phase times (events on the stream the library launches on) ----------------
    st = torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    phase = np.zeros(3)
    reps = max(3, min(args.steps, 10))
    for i in range(reps):
        d = data[i % nd]
        if RESAMPLE:   # phases: (nothing), steps, re-sampling
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

    # ---------------- per-kernel pass: the same rounds again, HIP events around every launch ----------------
    # (events are recorded by the library on the stream it launches on; bracketing every launch
    # widens the gaps between kernels, so this pass is kept apart from the throughput timing above)
    roof, classes, kernels = None, {}, []
    if not args.no_profile_pass:
        ctx.profile_enable(True)
        ctx.profile_reset()
        pr = max(2, min(args.steps, 5))
        for i in range(pr):
            run_round(ctx, cfg, dW, db, perms[i % nd], data[i % nd], None)
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
        dom = kernels[0]
        sec = dom["avg_launch_us"] * 1e-6
        traffic = MEASURED_TRAFFIC.get(args.workload, {}).get(dom["label"])
        if dom["flops_per_launch"] > 0:
            peak = PEAK["f32_TFLOPs"] if cfg.dtype == "f32" else PEAK["bf16_TFLOPs"]
            ach = dom["flops_per_launch"] / sec / 1e12
            roof = dict(kernel=dom["label"], bound="mfma", achieved=ach, peak=peak, unit="TFLOP/s", frac=ach / peak,
                        traffic=traffic, avg_launch_us=dom["avg_launch_us"], flops_per_launch=dom["flops_per_launch"])
        elif dom["bytes_per_launch"] > 0:
            ach = dom["bytes_per_launch"] / sec / 1e9
            roof = dict(kernel=dom["label"], bound="hbm", achieved=ach, peak=PEAK["hbm_GBs"], unit="GB/s",
                        frac=ach / PEAK["hbm_GBs"], traffic=traffic, avg_launch_us=dom["avg_launch_us"],
                        bytes_per_launch=dom["bytes_per_launch"])
        else:
            roof = dict(kernel=dom["label"], bound="hbm", achieved=None, peak=PEAK["hbm_GBs"], unit="GB/s",
                        frac=None, traffic=traffic, avg_launch_us=dom["avg_launch_us"])

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, args.cpu_seconds)

    peak_t = PEAK["f32_TFLOPs"] if cfg.dtype == "f32" else PEAK["bf16_TFLOPs"]
    out = {
        "metric": "subnet-SGD samples/sec (all S subnets, 1 GPU) + partition/merge GB/s",
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_round, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "dims": list(cfg.dims), "S": cfg.S, "B": cfg.B, "k": cfg.k,
                   "lr": cfg.lr, "input": cfg.input, "normalize": bool(args.normalize), "resample": bool(args.resample), "step": "one IST round: partition + k local SGD steps on S subnets + merge"},
        "phases": {
            "partition_ms": phase[0], "steps_ms": phase[1], "merge_ms": phase[2],
            "steps_samples_per_s": samples_round / (phase[1] * 1e-3),
            "steps_TFLOPs": wm["flops_round"] / (phase[1] * 1e-3) / 1e12,
            "steps_frac_of_mfma_peak": wm["flops_round"] / (phase[1] * 1e-3) / 1e12 / peak_t,
            "partition_GBs_line_granular": wm["partition_copy"][1] / (phase[0] * 1e-3) / 1e9,
            "merge_GBs_line_granular": wm["merge_copy"][1] / (phase[2] * 1e-3) / 1e9,
            "partition_GBs_useful": wm["useful_copy_bytes"] / (phase[0] * 1e-3) / 1e9,
            "merge_GBs_useful": wm["useful_copy_bytes"] / (phase[2] * 1e-3) / 1e9,
        },
        "resample_ms": (phase[2] if RESAMPLE else None),
        "kernel_classes": classes,
        "kernels": kernels[:8],
        "event_overhead_us": EVENT_OVERHEAD_US,
        "roofline": roof,
        "cpu_baseline": cpu,
        "loss_first_round": [float(first_loss[:, 0].mean()), float(first_loss[:, -1].mean())],
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
