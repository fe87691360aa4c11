#!/usr/bin/env python3
"""Benchmark of the decoupled data-parallel training step on one MI355X.

A step is one dds_step: every module's forward, backward, replica-mean SGD update and
weight snapshot for one batch of W*B synthetic CIFAR-shaped samples, inputs already in
HBM. Prints ONE JSON line: samples/s plus the roofline record of the dominant kernel
class and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"bf16": 2500.0, "f32": 157.3}  # dense MFMA TFLOP/s of MI355X


def hip_event_timer():
    """HIP events through libamdhip64 (works on any stream, unlike torch.cuda.Event)."""
    import torch
    bundled = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    hip = ctypes.CDLL(bundled if os.path.exists(bundled) else "libamdhip64.so")  # the runtime torch and libdds use
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    return hip


def read_traffic(workload_name, key):
    """HBM bytes per launch (of the dominant kernel, or of all GEMM kernels) from the rocprofv3
    FETCH_SIZE / WRITE_SIZE runs, if the summary for this workload has been recorded under
    profiles/ (else None)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 3 and f[0] == workload_name and f[1] == key:
            return float(f[2])
    return None


def algorithmic_bytes_per_step(wl, residual_passes=True):
    """HBM bytes one step has to move if every tensor crossed HBM exactly once per pass: for each
    convolution / linear layer 3 x (input + output) activations (forward, dgrad, wgrad) in the compute
    precision, plus the fp32 master weights read and written by the update and the compute-precision
    copy read by the three passes; a residual block adds its projection (a convolution) or two more passes
    over the block's tensor. Pools, rings and sign planes are left out: a lower bound."""
    es = 2 if wl.precision == "bf16" else 4
    n = wl.W * wl.B
    c, h, w = wl.in_shape
    blk = (c, h, w)
    total = 0
    for op in wl.ops:
        k = op["op"]
        if k == "conv":
            ho = (h + 2 * op["pad"] - op["k"]) // op["stride"] + 1
            wo = (w + 2 * op["pad"] - op["k"]) // op["stride"] + 1
            nw = op["cout"] * op["cin"] * op["k"] * op["k"]
            total += 3 * n * (op["cin"] * h * w + op["cout"] * ho * wo) * es + nw * (8 + 3 * es)
            c, h, w = op["cout"], ho, wo
        elif k == "linear":
            total += 3 * n * (op["cin"] + op["cout"]) * es + op["cin"] * op["cout"] * (8 + 3 * es)
            c, h, w = op["cout"], 1, 1
        elif k == "res_begin":
            blk = (c, h, w)
        elif k == "res_add":
            sc = op.get("shortcut")
            if sc:  # projection: a convolution from the block input to the block output
                nw = sc["cout"] * sc["cin"] * sc["k"] * sc["k"]
                total += 3 * n * (sc["cin"] * blk[1] * blk[2] + c * h * w) * es + nw * (8 + 3 * es)
            elif residual_passes:  # identity: the block input is read once more going forward, its gradient once going back
                total += 2 * n * c * h * w * es
        elif k == "maxpool2":
            h, w = h // 2, w // 2
        elif k == "gap":
            h, w = 1, 1
    return total


def cpu_baseline(wl, seconds_budget=20.0):
    """The oracle as it stands on a bounded sample: same K / W / delays / layers with a
    reduced per-replica batch, timed over steady-state iterations."""
    import torch
    from dds_inputs import make_batch, make_params, workload
    from oracle import fdg
    # per-group batch of the sample: large enough that per-sample cost is close to the full shape's (measured on
    # the ResNet-18 configuration: 17.7 samples/s at batch 2, ~20 at batch 16), small enough for ~20-30 s in all
    small_b = {"cfg0_mlp": wl.B, "cfg1_cnn": 32, "cfg2_resnet18": 16, "cfg3_resnet56": 4, "cfg4_resnet34w": 1}.get(wl.name, 2)
    small = workload(wl.name, B=small_b)
    pipe = fdg.Pipeline(small.ops, small.bounds, small.W, make_params(small, 0), small.lr, small.momentum)
    pipe.keep_history = False
    warm = 2 * (small.K - 1)
    t_used, n = 0.0, 0
    t = 0
    while True:
        batches = [make_batch(small, 0, t, s) for s in range(small.W)]
        t0 = time.perf_counter()
        pipe.step(batches)
        dt = time.perf_counter() - t0
        if t >= warm:
            t_used += dt
            n += 1
            if t_used > seconds_budget or n >= 50:
                break
        t += 1
    sps = n * small.W * small.B / t_used
    return {"value": sps, "unit": "samples/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"{n} steady-state steps of {small.name} with per-replica batch {small.B} "
                      f"(full K={small.K}, W={small.W}); fp64"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg2_resnet18")
    ap.add_argument("--batch", type=int, default=None, help="override per-replica batch (debug only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a 1 GiB device-to-device tensor copy, five times (the kernel of known size that the "
                         "FETCH_SIZE / WRITE_SIZE counters of the rocprofv3 summaries under profiles/ are scaled by)")
    ap.add_argument("--activations", default="store", choices=["store", "recompute"],
                    help="what delayed modules keep between forward and backward: every saved tensor (default) or "
                         "input, output and a parameter snapshot, with a second forward pass before the backward")
    ap.add_argument("--mixing", default="mean",
                    help="'mean' (the headline path: exact averaging, one weight copy) or 'ring:ALPHA' "
                         "(ring communication graph, every data-group keeps its own weights)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (all K x W module-replica pairs live on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(1)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": "5 copies of 1 GiB (elementwise copy kernel: 1 GiB read + 1 GiB written each)"}))
        return
    import paper_2509_05679_amd as P
    from dds_inputs import make_batch, make_params, workload

    wl = workload(args.workload, B=args.batch)
    warmup = args.warmup if args.warmup is not None else 2 * (wl.K - 1) + 5
    warmup = max(warmup, 2 * (wl.K - 1))  # timed steps are steady state: every module forwards, backwards, updates
    mixing = None
    if args.mixing != "mean":
        from dds_inputs.configs import ring_mixing
        kind, _, alpha = args.mixing.partition(":")
        if kind != "ring" or not alpha:
            sys.exit("bench.py: --mixing takes 'mean' or 'ring:ALPHA'")
        mixing = ring_mixing(wl.W, float(alpha))
    spec = P.Spec.from_workload(wl, mixing, args.activations)
    tr = P.Trainer(spec, wl.W)
    init = make_params(wl, 0)
    for k0 in range(wl.K):
        tr.dds_set_params(k0, init[k0])
    # a small pool of resident synthetic batches, cycled
    pool = 4
    xs = [[torch.from_numpy(make_batch(wl, 0, t, s)[0]).cuda() for s in range(wl.W)] for t in range(pool)]
    ys = [[torch.from_numpy(make_batch(wl, 0, t, s)[1]).cuda() for s in range(wl.W)] for t in range(pool)]
    stream = torch.cuda.current_stream()
    for t in range(warmup):
        tr.dds_step(xs[t % pool], ys[t % pool])
    torch.cuda.synchronize()

    hip = hip_event_timer()
    e0, e1 = ctypes.c_void_p(), ctypes.c_void_p()
    hip.hipEventCreate(ctypes.byref(e0))
    hip.hipEventCreate(ctypes.byref(e1))
    sp = ctypes.c_void_p(stream.cuda_stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    hip.hipEventRecord(e0, sp)
    for t in range(args.steps):
        tr.dds_step(xs[(warmup + t) % pool], ys[(warmup + t) % pool])
    hip.hipEventRecord(e1, sp)
    hip.hipEventSynchronize(e1)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = ctypes.c_float()
    hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1)
    ms_per_step = ms.value / args.steps
    loss = tr.dds_get_loss()
    # four more regions of the same length: `value` is the median region of the five
    first_region = ms_per_step
    runs = [ms_per_step]
    for r in range(4):
        hip.hipEventRecord(e0, sp)
        for t in range(args.steps):
            tr.dds_step(xs[(warmup + t) % pool], ys[(warmup + t) % pool])
        hip.hipEventRecord(e1, sp)
        hip.hipEventSynchronize(e1)
        hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1)
        runs.append(ms.value / args.steps)
    ms_per_step = sorted(runs)[2]
    samples = wl.W * wl.B
    flops = tr.dds_gemm_flops_per_step()
    launches = tr.dds_launches_last_step()

    # Roofline of the dominant kernel class: the MFMA implicit-GEMM kernels (forward, dgrad
    # and wgrad of every conv / linear layer). Two further, untimed passes bracket each of
    # those launches with HIP events on the stream it is launched on (dds_profile):
    # achieved = algorithmic FLOPs (2*M*N*K per launch) / summed launch durations.
    #  - serial pass (mode 2): modules run one after another, every launch has the chip to
    #    itself: this is the per-kernel figure reported as `achieved`;
    #  - concurrent pass (mode 1): the K modules share the chip as in the timed region, so
    #    durations overlap (reported per class as avg_us_concurrent).
    nprof = max(4, min(args.steps, 10))

    def profile_pass(mode):
        tr.dds_profile(mode)
        for t in range(nprof):
            tr.dds_step(xs[t % pool], ys[t % pool])
        prof = tr.dds_profile_read()
        tr.dds_profile(0)
        return prof

    prof = profile_pass(2)
    prof_conc = profile_pass(1)
    def agg(pr, keys):
        ms = sum(pr[k][0] for k in keys)
        n = sum(pr[k][1] for k in keys)
        fl = sum(pr[k][2] for k in keys)
        return ms, n, fl

    # dominant kernel: the asynchronous 3x3 conv kernel (forward + dgrad launches); it falls back
    # to all GEMM launches for workloads that never reach it (MLP, tiny channels)
    dom_keys = ("forward_dma", "dgrad_dma")
    dom_name = "conv3x3_dma_kernel (3x3 stride-1 forward + dgrad launches), each launch timed alone"
    if agg(prof, dom_keys)[1] == 0:
        dom_keys = tuple(prof)
        dom_name = "conv/linear implicit-GEMM (all forward + dgrad + wgrad launches), each launch timed alone"
    gemm_ms, gemm_launches, gemm_flops = agg(prof, dom_keys)
    all_ms, all_n, all_fl = agg(prof, tuple(prof))
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    peak = PEAK[wl.precision]
    per_class = {k: {"avg_us": 1e3 * v[0] / max(v[1], 1), "TFLOP/s": v[2] / max(v[0], 1e-9) / 1e9,
                     "launches_per_step": v[1] / nprof,
                     "avg_us_concurrent": 1e3 * prof_conc[k][0] / max(prof_conc[k][1], 1)}
                 for k, v in prof.items() if v[1] > 0}
    traffic = read_traffic(wl.name, "conv3x3_dma_bytes_per_launch" if dom_keys == ("forward_dma", "dgrad_dma") else "gemm_bytes_per_launch")
    out = {
        "metric": "training samples/sec on 1 MI355X per decoupled step",
        "value": samples / (ms_per_step * 1e-3),
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if wl.precision == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: K={wl.K} modules, W={wl.W} replicas x batch {wl.B}, {wl.precision}",
                   "launches_per_step": launches, "wall_ms_per_step": wall * 1e3 / args.steps,
                   "ms_per_step_of_5_regions": [round(v, 4) for v in runs], "first_region_ms_per_step": first_region,
                   "value_is": "median of five timed regions of `steps` consecutive steady-state steps each",
                   "loss_after": loss, "arena_GiB": tr.arena_bytes / 2 ** 30, "mixing": args.mixing, "activations": args.activations,
                   "consensus_error": tr.dds_consensus_error() if mixing is not None else 0.0},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": traffic,
                     "conv_mfma_util_pct_of_peak": 100.0 * achieved / peak,
                     "kernel": dom_name,
                     "avg_launch_us": 1e3 * gemm_ms / max(gemm_launches, 1), "per_class": per_class,
                     "all_gemm_launches": {"TFLOP/s": all_fl / max(all_ms, 1e-9) / 1e9, "avg_us": 1e3 * all_ms / max(all_n, 1),
                                           "launches_per_step": all_n / nprof},
                     "whole_step_TFLOP/s": flops / (ms_per_step * 1e-3) / 1e12,
                     "whole_step_frac": flops / (ms_per_step * 1e-3) / 1e12 / peak,
                     "whole_step_hbm": {"note": "lower bound on HBM bytes per step (see algorithmic_bytes_per_step) over the measured step time",
                                        "algorithmic_GiB_per_step": algorithmic_bytes_per_step(wl) / 2 ** 30,
                                        "conv_and_linear_passes_only_GiB": algorithmic_bytes_per_step(wl, False) / 2 ** 30,
                                        "TB/s": algorithmic_bytes_per_step(wl) / (ms_per_step * 1e-3) / 1e12,
                                        "frac_of_8_TB/s": algorithmic_bytes_per_step(wl) / (ms_per_step * 1e-3) / 8e12}},
    }
    tr.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
