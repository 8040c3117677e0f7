#!/usr/bin/env python3
"""Benchmark of the AWP/ADT hot path on one MI355X.

One step = one pass of the whole path over a synthetic CNN-shaped weight set
that is already resident in HBM:
    awp_layer_stats -> copy of L x 3 doubles to the host -> awp_update (host,
    scalar) -> adt_pack -> adt_unpack (into a separate FP32 buffer).
Prints ONE JSON line.  `value` is FP32 weight bytes through the whole pass per
second (4 N / step time).  Per-kernel durations are the dispatches' own begin /
end timestamps (HIP events bound to each launch on its stream, read through
the library's launch-timing calls) over the timed region; the roofline entry prices the
slower of the two ADT kernels against the 8 TB/s HBM peak with algorithmic
bytes (4 + r per weight).  The CPU oracle is timed beside it on a bounded
number of passes over the same weight set.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

WORKLOADS = {
    # name: (weight set, byte-count variant, start bits for the AWP state)
    "vgg16_all2": ("vgg16", "all2"),
    "vgg16_all3": ("vgg16", "all3"),
    "vgg16_all1": ("vgg16", "all1"),
    "vgg16_all4": ("vgg16", "all4"),
    "vgg16_mixed": ("vgg16", "mixed"),
    "alexnet": ("alexnet", "default"),
    "resnet50": ("resnet50", "default"),
    "tiny": ("tiny", "default"),
}


def kernel_source_digest() -> str:
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2004_02297_amd", "csrc")
    for f in sorted(os.listdir(d)):
        h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(kernel: str, workload: str):
    """HBM bytes per launch from committed rocprofv3 counter runs, if they were
    taken on the current kernel sources; otherwise None."""
    p = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(p):
        return None
    rec = json.load(open(p))
    if rec.get("kernel_source_digest") != kernel_source_digest():
        return None
    return rec.get("traffic_bytes", {}).get(workload, {}).get(kernel)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="vgg16_all2", choices=sorted(WORKLOADS))
    ap.add_argument("--cpu-seconds", type=float, default=10.0,
                    help="lower bound on the CPU-oracle timing loop (0 = skip)")
    ap.add_argument("--prime", type=int, default=150,
                    help="untimed passes before the warm-up (see PRIME_STEPS below)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region, run one plain device copy of the weight "
                         "buffer (4N bytes read, 4N written): the known-size kernel that "
                         "rocprofv3 counter runs are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no multi-GPU "
              "path); run with --gpus 1", file=sys.stderr)
        return 2

    import torch

    import paper_2004_02297_amd as adt
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    adt.load_library()
    torch.cuda.set_device(0)

    set_name, variant = WORKLOADS[args.workload]
    ws = workloads.make_weight_set(set_name)
    off = ws.layer_offsets
    L, N = ws.n_layers, ws.n_weights
    target_bytes = workloads.config_bytes(set_name, variant)

    # AWP state: the paper's VGG threshold and interval (Section V-A).  The
    # weight set does not change between steps, so delta = 0 >= T on every step
    # and each layer stays at its starting precision: the byte counts the
    # workload names are exactly what the rule hands to pack/unpack.
    T, INTERVAL, N_BITS = -2e-3, 4000, 8
    state = adt.AwpState(L)
    state.bits[:] = target_bytes.astype(np.int32) * 8

    w = torch.from_numpy(ws.weights).cuda()
    packed = torch.empty(adt.adt_packed_size(off, target_bytes), dtype=torch.uint8, device="cuda")
    w_out = torch.empty_like(w)
    stats_dev = torch.empty((L, adt.AWP_NSTATS), dtype=torch.float64, device="cuda")
    stats_host = torch.empty((L, adt.AWP_NSTATS), dtype=torch.float64, pin_memory=True)
    stream = torch.cuda.current_stream()

    def step():
        adt.awp_layer_stats(w, off, out=stats_dev)
        stats_host.copy_(stats_dev, non_blocking=True)
        stream.synchronize()
        rb = adt.awp_update(state, stats_host[:, 1].numpy(), T, INTERVAL, N_BITS)
        adt.adt_pack(w, off, rb, out=packed)
        adt.adt_unpack(packed, off, rb, out=w_out)
        return rb

    # The HIP runtime stalls once for tens of milliseconds somewhere in the first
    # few hundred launches of a process (seen at launch ~250, never again in 3000
    # steps).  PRIME_STEPS untimed passes before the warm-up keep that one-time
    # event out of the timed region whatever --warmup is.
    PRIME_STEPS = max(args.prime, 0)
    rb = target_bytes
    for _ in range(PRIME_STEPS + args.warmup):
        rb = step()
    torch.cuda.synchronize()
    assert np.array_equal(rb, target_bytes), "AWP state drifted from the workload's byte counts"

    # Exact kernel durations inside the timed region: on every TIMED_EVERY-th
    # step each launch carries its dispatch's begin / end timestamps (HIP events
    # bound to the launch, on the launch stream).  Sampling keeps the host cost
    # of such launches (about 10 us each) out of most steps.
    TIMED_EVERY = 4
    n_sampled = (args.steps + TIMED_EVERY - 1) // TIMED_EVERY
    adt.adt_timing_enable(True, 4 * n_sampled)
    adt.adt_timing_enable(False)
    adt.adt_timing_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        sampled = k % TIMED_EVERY == 0
        if sampled:
            adt.adt_timing_enable(True)
        rb = step()
        if sampled:
            adt.adt_timing_enable(False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    timing = adt.adt_timing_read()
    assert np.array_equal(rb, target_bytes)
    assert all(timing[k]["launches"] == n_sampled for k in timing), timing

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    if args.calibrate_copy:
        w_out.copy_(w)
        torch.cuda.synchronize()

    sizes = np.diff(off)
    bytes_adt = float(np.sum(sizes * (4 + target_bytes.astype(np.int64))))   # per ADT launch
    bytes_stats = 4.0 * N

    def kern(names, nbytes):
        avg = sum(timing[n]["total_ms"] for n in names) / n_sampled
        return {"avg_ms": round(avg, 5),
                "min_ms": round(sum(timing[n]["min_ms"] for n in names), 5),
                "max_ms": round(sum(timing[n]["max_ms"] for n in names), 5),
                "gbps": round(nbytes / avg / 1e6, 1),
                "hbm_frac": round(nbytes / avg / 1e6 / HBM_PEAK_GBPS, 4)}

    kernels = {"adt_pack": kern(["pack_kernel"], bytes_adt),
               "adt_unpack": kern(["unpack_kernel"], bytes_adt),
               "awp_layer_stats": kern(["stats_partial_kernel", "stats_final_kernel"], bytes_stats)}
    dom = "adt_pack" if kernels["adt_pack"]["avg_ms"] >= kernels["adt_unpack"]["avg_ms"] \
        else "adt_unpack"
    achieved = kernels[dom]["gbps"]
    t_pu = kernels["adt_pack"]["avg_ms"] + kernels["adt_unpack"]["avg_ms"]
    t_kernels = t_pu + kernels["awp_layer_stats"]["avg_ms"]

    result = {
        "metric": "ADT pack+unpack GB/s of FP32 weights (and % of HBM peak); AWP stats GB/s",
        "value": round(4.0 * N / ms_per_step / 1e6, 2),
        "unit": "GB/s of FP32 weights through one full pass (stats + AWP rule + pack + unpack)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32 bit fields (pack/unpack), f64 accumulate (stats)",
        "data": "synthetic He-normal CNN-shaped FP32 weights, resident in HBM",
        "config": {"workload": args.workload, "n_weights": N, "n_layers": L,
                   "bytes_per_layer": target_bytes.tolist(),
                   "packed_bytes": int(packed.numel())},
        "pack_unpack_fp32_gbps": round(4.0 * N / t_pu / 1e6, 1),
        "pack_unpack_moved_gbps": round(2 * bytes_adt / t_pu / 1e6, 1),
        "pack_unpack_hbm_frac": round(2 * bytes_adt / t_pu / 1e6 / HBM_PEAK_GBPS, 4),
        "stats_fp32_gbps": kernels["awp_layer_stats"]["gbps"],
        "kernels": kernels,
        "priming_steps": PRIME_STEPS,
        "kernel_timing": "dispatch begin/end timestamps on %d of the %d timed steps" % (
            n_sampled, args.steps),
        "kernel_ms_per_step": round(t_kernels, 5),
        "host_and_sync_ms_per_step": round(ms_per_step - t_kernels, 5),
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "algorithmic_bytes_per_launch": bytes_adt,
                     "traffic": recorded_traffic(dom, args.workload)},
    }

    if args.cpu_seconds > 0:
        import oracle
        ostate = oracle.AwpState(L)
        ostate.bits[:] = state.bits
        passes, c0 = 0, time.perf_counter()
        while passes < 2 or time.perf_counter() - c0 < args.cpu_seconds:
            st = oracle.stats(ws.weights, off)
            orb = oracle.awp_update(ostate, st[:, 1], T, INTERVAL, N_BITS)
            stream_bytes = oracle.pack(ws.weights, off, orb)
            oracle.unpack(stream_bytes, off, orb)
            passes += 1
        c1 = time.perf_counter()
        result["cpu_baseline"] = {
            "value": round(4.0 * N * passes / (c1 - c0) / 1e9, 3),
            "unit": result["unit"], "cores": 1, "kind": "oracle",
            "sample": "%d full passes (stats + rule + pack + unpack) of the scalar C oracle "
                      "over the same %s weight set, %.1f s" % (passes, args.workload, c1 - c0),
            "host_cpus_visible": os.cpu_count(),
        }
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
