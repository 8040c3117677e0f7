#!/usr/bin/env python3
"""Benchmark of the AWP/ADT hot path on one MI355X.

One step = one pass of the whole path (per-layer statistics -> AWP rule ->
Bitpack -> Bitunpack into a separate FP32 buffer) over a synthetic CNN-shaped
weight set that is already resident in HBM.

Every timed loop ROTATES its output buffers (packed stream and truncated
weights) over three distinct sets.  A loop that rewrites one output buffer over
and over lets the 256 MB Infinity Cache absorb part of the rewrite, which
overstates what HBM sustains; with rotation every store goes to memory that the
cache does not hold, as it does in training, where a whole forward/backward
pass runs between two passes of this path.  The in-place loop is timed too and
reported separately ("in_place_rewrite": HBM plus cache, not an HBM figure).

Implementations of the same pass, each timed over its own K steps after W
warm-up steps:

  plan path   (the headline): awp_adt_step — device-resident AWP state, one
              fused kernel that reads the weights once, no host round trip.
  plan, graph the same step captured once per buffer set into a HIP graph and
              replayed.
  three calls awp_layer_stats -> copy of L x 3 doubles to the host ->
              awp_update on the host -> adt_pack -> adt_unpack.
  plan, bf16  awp_adt_step16: truncated weights written as bfloat16 (an
              extension, not the headline).
  adt_pack_unpack: pack + unpack in one kernel, no statistics.

Prints ONE JSON line.  `value` is FP32 weight bytes through the whole pass per
second (4 N / step time) on the headline workload.  Kernel durations are the
dispatches' own begin / end timestamps (HIP events bound to each launch on its
stream, read through the library's launch-timing calls) on a sample of the
timed steps.  `roofline` prices the dominant kernel against the 8 TB/s HBM peak
with algorithmic bytes.  `configs` carries the same figures for the other
workloads, `trajectory` the 200-step AWP trajectory, `cpu_baseline` the CPU
oracle timed on full passes over the same weights.
"""
from __future__ import annotations

import argparse
import csv
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
TIMED_EVERY = 4          # launch timing is switched on for every 4th timed step
ROTATE = 3               # distinct output buffer sets a timed loop cycles through
# An idle GPU lowers its clocks and takes about 15 ms of work to raise them again
# (measured here: after 2-10 s of idleness the first 25 steps run 7-10 % slow, the
# next 40 steps 2-3 % slow, everything after that at one rate).  Every timed loop is
# therefore preceded by at least this much untimed work of the same kind, on top of
# the warm-up steps asked for; the steps it took are reported under "clock_settle".
SETTLE_SECONDS = 0.1


def settle_clocks(torch, work, seconds=SETTLE_SECONDS, first=0) -> int:
    """Run work(i), i = first, first + 1, ..., untimed until `seconds` of wall time
    have passed with the GPU busy throughout; returns the number of calls made."""
    n = 0
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(16):
            work(first + n)
            n += 1
        torch.cuda.synchronize()
    return n

WORKLOADS = {
    # name: (weight set, byte-count variant)
    "vgg16_all2": ("vgg16", "all2"),
    "vgg16_all3": ("vgg16", "all3"),
    "vgg16_all1": ("vgg16", "all1"),
    "vgg16_all4": ("vgg16", "all4"),
    "vgg16_mixed": ("vgg16", "mixed"),
    "alexnet": ("alexnet", "default"),
    "resnet50": ("resnet50", "default"),
    "tiny": ("tiny", "default"),
}
# reported under "configs" beside the headline workload (short runs)
OTHER_CONFIGS = ("vgg16_all3", "vgg16_mixed", "alexnet", "resnet50")

PAPER_CONTEXT = {
    "note": "context only, other hardware and the whole training loop: not a target for this path",
    "average_training_speedup_x86": "6.18 % (2x Xeon E5-2630 v3 + 4x Tesla GK210 over PCIe 3.0; Section V)",
    "average_training_speedup_power": "11.91 % (2x POWER9 + 4x V100 over NVLink 2.0; Section V)",
    "per_batch_kernel_times_vgg_batch64_ms": {
        "x86": {"bitpack": 19.71, "bitunpack": 4.51, "l2_norm": 3.88},
        "power9": {"bitpack": 10.51, "bitunpack": 1.11, "l2_norm": 0.93},
        "source": "Tables 2 and 3"},
}

KERNEL_SOURCES = ("adt_tables.h", "adt_tile_ops.h", "adt_launch.h", "awp_partials.h",
                  "adt_pack_unpack.hip", "awp_stats.hip", "awp_fused.hip")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")
# entry point -> substrings that select its kernels in a rocprofv3 counter CSV
TRAFFIC_KERNELS = {
    "fused_kernel": ["adt::fused_kernel<0,"],
    "adt_pack": ["adt::pack_kernel<"],
    "adt_unpack": ["adt::unpack_kernel<true, 0>", "adt::unpack_kernel<false, 0>"],
    "awp_layer_stats": ["adt::stats_partial_kernel<", "adt::stats_final_kernel<"],
    "adt_pack_unpack": ["adt::pack_unpack_kernel<"],
}


def kernel_source_digest() -> str:
    """Digest of the files that define the measured kernels and their launch shapes
    (the host-side API file and the ablation kernels are not part of it)."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2004_02297_amd", "csrc")
    for f in KERNEL_SOURCES:
        h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(kernel: str, workload: str):
    """HBM bytes per launch from committed rocprofv3 counter runs, if they were
    taken on the current kernel sources; otherwise None."""
    if not os.path.exists(TRAFFIC_FILE):
        return None
    rec = json.load(open(TRAFFIC_FILE))
    if rec.get("kernel_source_digest") != kernel_source_digest():
        return None
    return rec.get("traffic_bytes", {}).get(workload, {}).get(kernel)


def traffic_from_counters(fetch_dir: str, write_dir: str, workload: str, n_weights: int) -> int:
    """Turn two rocprofv3 --pmc runs of `bench.py --calibrate-copy` (FETCH_SIZE in one,
    WRITE_SIZE in the other; each directory holds *_counter_collection.csv) into
    profiles/traffic.json.  Each counter is scaled by what it reads for the plain
    device copy of the weight buffer (4 N bytes each way) in the same run."""
    def load(folder):
        per_kernel = {}
        for base, _, files in os.walk(folder):
            for f in files:
                if f.endswith("counter_collection.csv"):
                    for row in csv.DictReader(open(os.path.join(base, f))):
                        per_kernel.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
        if not per_kernel:
            raise SystemExit("no *_counter_collection.csv under %s" % folder)
        return per_kernel

    def mean_of(per_kernel, patterns):
        total = 0.0
        for pat in patterns:
            vals = [v for name, vs in per_kernel.items() if pat in name for v in vs]
            if vals:
                total += sum(vals) / len(vals)
        return total

    fetch, write = load(fetch_dir), load(write_dir)
    known_kib = 4.0 * n_weights / 1024
    copy_f = max(v for name, vs in fetch.items() if "copyBuffer" in name for v in vs)
    copy_w = max(v for name, vs in write.items() if "copyBuffer" in name for v in vs)
    scale_f, scale_w = known_kib / copy_f, known_kib / copy_w
    out, rows = {}, []
    for entry, patterns in TRAFFIC_KERNELS.items():
        f_kib, w_kib = mean_of(fetch, patterns), mean_of(write, patterns)
        if f_kib == 0.0 and w_kib == 0.0:
            continue
        rd, wr = f_kib * scale_f * 1024, w_kib * scale_w * 1024
        out[entry] = round(rd + wr)
        rows.append((entry, f_kib, w_kib, rd, wr))
    rec = {"kernel_source_digest": kernel_source_digest(),
           "scale": {"FETCH_SIZE": scale_f, "WRITE_SIZE": scale_w,
                     "copy_kernel_bytes_each_way": 4 * n_weights},
           "traffic_bytes": {workload: out}}
    json.dump(rec, open(TRAFFIC_FILE, "w"), indent=1)
    print("copy kernel: FETCH_SIZE %.1f KiB, WRITE_SIZE %.1f KiB for %.1f KiB each way" %
          (copy_f, copy_w, known_kib))
    print("| entry point | FETCH_SIZE KiB | WRITE_SIZE KiB | read bytes | written bytes | total |")
    for r in rows:
        print("| %s | %.1f | %.1f | %.0f | %.0f | %.0f |" % (r[0], r[1], r[2], r[3], r[4], r[3] + r[4]))
    return 0


def run_ablation(args) -> int:
    """Sustained time per call (back-to-back launches, HIP events around the
    loop on the launch stream) of production vs ablation kernels."""
    import torch

    import paper_2004_02297_amd as adt
    import workloads

    adt.load_library()
    iters = max(args.steps, 1)

    def sustained_us(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    out = {"mode": "ablation", "iters": iters, "unit": "us per call, back-to-back launches",
           "hbm_peak_gbps": HBM_PEAK_GBPS, "cases": []}
    primed = False
    for wl in ("vgg16_all2", "vgg16_all3", "resnet50"):
        set_name, variant = WORKLOADS[wl]
        ws = workloads.make_weight_set(set_name)
        off = ws.layer_offsets
        rb = workloads.config_bytes(set_name, variant)
        nbytes = float(np.sum(np.diff(off) * (4 + rb.astype(np.int64))))
        w = torch.from_numpy(ws.weights).cuda()
        p = torch.empty(adt.adt_packed_size(off, rb), dtype=torch.uint8, device="cuda")
        w2 = torch.empty_like(w)
        if not primed:          # the runtime's one-time launch stall (see PRIMING in main)
            for _ in range(max(args.prime, 0)):
                adt.adt_pack(w, off, rb, out=p)
            torch.cuda.synchronize()
            primed = True
        rows = {
            "pack: production (LDS repack, one launch)": lambda: adt.adt_pack(w, off, rb, out=p),
            "pack: 128-bit loads, direct 4r-byte stores": lambda: adt.adt_ablation(
                adt.ABLATION_VEC_DIRECT, False, w, off, rb, p),
            "pack: naive, one weight per thread": lambda: adt.adt_ablation(
                adt.ABLATION_NAIVE, False, w, off, rb, p),
            "pack: production kernel, one launch per layer": lambda: adt.adt_ablation(
                adt.ABLATION_PER_LAYER, False, w, off, rb, p),
            "unpack: production (LDS repack, one launch)": lambda: adt.adt_unpack(p, off, rb, out=w2),
            "unpack: naive, one weight per thread": lambda: adt.adt_ablation(
                adt.ABLATION_NAIVE, True, w2, off, rb, p),
            "unpack: production kernel, one launch per layer": lambda: adt.adt_ablation(
                adt.ABLATION_PER_LAYER, True, w2, off, rb, p),
        }
        case = {"workload": wl, "n_layers": int(ws.n_layers), "n_weights": int(ws.n_weights),
                "algorithmic_bytes": nbytes, "rows": {}}
        for name, fn in rows.items():
            us = sustained_us(fn)
            case["rows"][name] = {"us": round(us, 1), "gbps": round(nbytes / us / 1e3, 1),
                                  "hbm_frac": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)}
        out["cases"].append(case)
        del w, p, w2
    print(json.dumps(out))
    return 0


class Harness:
    """Timed regions over one workload.  Holds the device buffers: the weights and
    ROTATE sets of (packed stream, truncated weights)."""

    # AWP parameters: the paper's VGG threshold and interval (Section V-A).  The
    # weight set does not change between steps, so delta = 0 >= T on every step
    # and each layer stays at its starting precision: the byte counts the
    # workload names are exactly what the rule hands to pack/unpack.
    T, INTERVAL, N_BITS = -2e-3, 4000, 8

    def __init__(self, adt, torch, workloads, workload: str, steps: int, warmup: int, prime: int):
        self.adt, self.torch = adt, torch
        self.workload, self.steps, self.warmup, self.prime = workload, steps, warmup, prime
        set_name, variant = WORKLOADS[workload]
        self.ws = workloads.make_weight_set(set_name)
        self.off = self.ws.layer_offsets
        self.L, self.N = self.ws.n_layers, self.ws.n_weights
        self.rb = workloads.config_bytes(set_name, variant)
        self.start_bits = self.rb.astype(np.int32) * 8
        self.sizes = np.diff(self.off)
        r = self.rb.astype(np.int64)
        self.bytes_pack = float(np.sum(self.sizes * (4 + r)))      # per pack or unpack launch
        self.bytes_stats = 4.0 * self.N
        self.bytes_fused = float(np.sum(self.sizes * (8 + r)))     # read W, write stream + W'
        self.bytes_fused16 = float(np.sum(self.sizes * (6 + r)))   # truncated weights as 16 bit
        self.packed_bytes = int(np.sum(self.sizes * r))
        self.w = torch.from_numpy(self.ws.weights).cuda()
        self.packed = [torch.empty(4 * self.N, dtype=torch.uint8, device="cuda") for _ in range(ROTATE)]
        self.w_out = [torch.empty_like(self.w) for _ in range(ROTATE)]
        self.n_sampled = (steps + TIMED_EVERY - 1) // TIMED_EVERY

    def timed_region(self, step, prime=0, finish=None):
        """step(i) is called with the running step number; finish() (work the last
        step left to whoever needs its results first) runs inside the timed region.
        Returns (ms per step over `steps` steps, per-kernel launch timing of every
        TIMED_EVERY-th step)."""
        adt, torch = self.adt, self.torch
        for i in range(prime + self.warmup):
            step(i)
            if i % 32 == 31:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        self.settle_steps = settle_clocks(torch, step, first=prime + self.warmup)
        adt.adt_timing_enable(True, 8 * self.n_sampled)    # prepare event pairs up front
        adt.adt_timing_enable(False)
        adt.adt_timing_read()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(self.steps):
            sampled = k % TIMED_EVERY == 0
            if sampled:
                adt.adt_timing_enable(True)
            step(k)
            if sampled:
                adt.adt_timing_enable(False)
        if finish is not None:
            finish()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / self.steps, adt.adt_timing_read()

    @staticmethod
    def kern(timing, names, nbytes=None):
        if all(timing[n]["launches"] == 0 for n in names):
            return {"avg_ms": 0.0, "min_ms": 0.0, "max_ms": 0.0, "launches_timed": 0}
        avg = sum(timing[n]["total_ms"] / max(timing[n]["launches"], 1) for n in names)
        out = {"avg_ms": round(avg, 5),
               "min_ms": round(sum(timing[n]["min_ms"] for n in names), 5),
               "max_ms": round(sum(timing[n]["max_ms"] for n in names), 5),
               "launches_timed": int(timing[names[0]]["launches"])}
        if nbytes is not None and avg > 0:
            out["gbps"] = round(nbytes / avg / 1e6, 1)
            out["hbm_frac"] = round(nbytes / avg / 1e6 / HBM_PEAK_GBPS, 4)
        return out

    def roofline(self, kernel, k, nbytes, traffic_key=None):
        return {"bound": "hbm", "kernel": kernel, "achieved": k["gbps"], "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": k["hbm_frac"], "algorithmic_bytes_per_launch": nbytes,
                "traffic": recorded_traffic(traffic_key or kernel, self.workload)}

    def plan_path(self, rotate=True, out16=False, no_out=False):
        """no_out: statistics, rule and stream only (no truncated copy): the step of a
        device that only sends the stream."""
        adt, torch = self.adt, self.torch
        plan = adt.AwpPlan(self.off, self.T, self.INTERVAL, self.N_BITS, init_bits=self.start_bits)
        outs = self.w_out
        if out16:
            outs = [torch.empty(self.N, dtype=torch.bfloat16, device="cuda") for _ in range(ROTATE)]
        if no_out:
            outs = [None] * ROTATE
        m = ROTATE if rotate else 1
        # the last batch's final reduction is launched by the read: inside the timed region
        ms, timing = self.timed_region(lambda i: plan.step(self.w, self.packed[i % m], outs[i % m]),
                                       finish=plan.flush)
        got = plan.read()
        assert np.array_equal(got["bytes"], self.rb), "AWP state drifted"
        assert got["packed_size"] == self.packed_bytes
        plan.close()
        nbytes = self.bytes_pack if no_out else self.bytes_fused16 if out16 else self.bytes_fused
        kernels = {"fused_kernel": self.kern(timing, ["fused_kernel"], nbytes),
                   "final_rule_kernel": self.kern(timing, ["final_rule_kernel"]),
                   "redo_kernel": self.kern(timing, ["redo_kernel"])}
        if kernels["redo_kernel"]["launches_timed"] == 0:
            kernels["redo_kernel"]["note"] = ("not launched: the library leaves the redo pass out while "
                                              "no interval counter can reach INTERVAL")
        if kernels["final_rule_kernel"]["launches_timed"] == 0:
            kernels["final_rule_kernel"]["note"] = ("no launch of its own: while no byte count can move, a "
                                                    "batch's final reduction and rule ride at the head of "
                                                    "the next batch's fused kernel")
        t_k = sum(k["avg_ms"] for k in kernels.values())
        return {"value": round(4.0 * self.N / ms / 1e6, 2), "ms_per_step": round(ms, 5),
                "settle_steps": self.settle_steps,
                "kernels": kernels, "kernel_ms_per_step": round(t_k, 5),
                "host_and_gaps_ms_per_step": round(ms - t_k, 5),
                "moved_gbps_whole_step": round(nbytes / ms / 1e6, 1),
                "hbm_frac_whole_step": round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                "roofline": dict(self.roofline("fused_kernel", kernels["fused_kernel"], nbytes),
                                 note="the launch also carries the previous batch's final reduction and "
                                      "rule (a few dozen one-wave blocks at the head of the grid)")}

    def plan_graph_replay(self):
        """The plan's step captured once per buffer set and replayed round robin."""
        adt, torch = self.adt, self.torch
        plan = adt.AwpPlan(self.off, self.T, self.INTERVAL, self.N_BITS, init_bits=self.start_bits)
        plan.step(self.w, self.packed[0], self.w_out[0])      # the first batch only records norms
        plan.read()                   # its reduction has run: nothing is left over for the capture
        graphs = []
        side = torch.cuda.Stream()
        for j in range(ROTATE):
            g = torch.cuda.CUDAGraph()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    plan.step(self.w, self.packed[j], self.w_out[j])
            torch.cuda.current_stream().wait_stream(side)
            graphs.append(g)
        torch.cuda.synchronize()
        for i in range(self.warmup):
            graphs[i % ROTATE].replay()
        torch.cuda.synchronize()
        settle_clocks(torch, lambda i: graphs[i % ROTATE].replay())
        t0 = time.perf_counter()
        for i in range(self.steps):
            graphs[i % ROTATE].replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / self.steps
        got = plan.read()
        assert np.array_equal(got["bytes"], self.rb) and got["packed_size"] == self.packed_bytes
        plan.close()
        del graphs
        return {"value": round(4.0 * self.N / ms / 1e6, 2), "ms_per_step": round(ms, 5),
                "moved_gbps_whole_step": round(self.bytes_fused / ms / 1e6, 1),
                "hbm_frac_whole_step": round(self.bytes_fused / ms / 1e6 / HBM_PEAK_GBPS, 4),
                "note": "a captured step always holds the redo launch (the choice cannot be made per replay)"}

    def three_calls(self):
        adt, torch = self.adt, self.torch
        state = adt.AwpState(self.L)
        state.bits[:] = self.start_bits
        stats_dev = torch.empty((self.L, adt.AWP_NSTATS), dtype=torch.float64, device="cuda")
        stats_host = torch.empty((self.L, adt.AWP_NSTATS), dtype=torch.float64, pin_memory=True)
        stream = torch.cuda.current_stream()

        def step(i):
            adt.awp_layer_stats(self.w, self.off, out=stats_dev)
            stats_host.copy_(stats_dev, non_blocking=True)
            stream.synchronize()
            rb = adt.awp_update(state, stats_host[:, 1].numpy(), self.T, self.INTERVAL, self.N_BITS)
            adt.adt_pack(self.w, self.off, rb, out=self.packed[i % ROTATE])
            adt.adt_unpack(self.packed[i % ROTATE], self.off, rb, out=self.w_out[i % ROTATE])

        ms, timing = self.timed_region(step, self.prime)
        assert np.array_equal(state.bytes, self.rb), "AWP state drifted"
        kernels = {"adt_pack": self.kern(timing, ["pack_kernel"], self.bytes_pack),
                   "adt_unpack": self.kern(timing, ["unpack_kernel"], self.bytes_pack),
                   "awp_layer_stats": self.kern(timing, ["stats_partial_kernel", "stats_final_kernel"],
                                                self.bytes_stats)}
        dom = "adt_pack" if kernels["adt_pack"]["avg_ms"] >= kernels["adt_unpack"]["avg_ms"] \
            else "adt_unpack"
        t_pu = kernels["adt_pack"]["avg_ms"] + kernels["adt_unpack"]["avg_ms"]
        t_k = t_pu + kernels["awp_layer_stats"]["avg_ms"]
        return {"value": round(4.0 * self.N / ms / 1e6, 2), "ms_per_step": round(ms, 5),
                "kernels": kernels, "kernel_ms_per_step": round(t_k, 5),
                "host_and_sync_ms_per_step": round(ms - t_k, 5),
                "pack_unpack_fp32_gbps": round(4.0 * self.N / t_pu / 1e6, 1),
                "pack_unpack_moved_gbps": round(2 * self.bytes_pack / t_pu / 1e6, 1),
                "pack_unpack_hbm_frac": round(2 * self.bytes_pack / t_pu / 1e6 / HBM_PEAK_GBPS, 4),
                "stats_fp32_gbps": kernels["awp_layer_stats"]["gbps"],
                "note": "adt_unpack follows adt_pack at once and finds part of the stream in the "
                        "Infinity Cache: its figure is bytes moved per second, not HBM bytes",
                "roofline": self.roofline(dom, kernels[dom], self.bytes_pack)}

    def pack_unpack(self, launches):
        """adt_pack_unpack back to back, every launch timed."""
        adt, torch = self.adt, self.torch

        def call(i):
            adt.adt_pack_unpack(self.w, self.off, self.rb, out=self.packed[i % ROTATE],
                                weights_out=self.w_out[i % ROTATE])
        for i in range(self.prime + 5):
            call(i)
        torch.cuda.synchronize()
        settle_clocks(torch, call)
        adt.adt_timing_enable(True, launches)
        adt.adt_timing_read()
        for i in range(launches):
            call(i)
        torch.cuda.synchronize()
        t = adt.adt_timing_read()["pack_unpack_kernel"]
        adt.adt_timing_enable(False)
        avg = t["total_ms"] / max(t["launches"], 1)
        return {"entry_point": "adt_pack_unpack", "launches_timed": int(t["launches"]),
                "avg_ms": round(avg, 5), "min_ms": round(t["min_ms"], 5),
                "fp32_weights_gbps": round(4.0 * self.N / avg / 1e6, 1),
                "algorithmic_bytes_per_launch": self.bytes_fused,
                "gbps": round(self.bytes_fused / avg / 1e6, 1),
                "hbm_frac": round(self.bytes_fused / avg / 1e6 / HBM_PEAK_GBPS, 4)}

    def pack_and_unpack_apart(self, launches):
        """adt_pack and adt_unpack each in a loop of its own over the rotating buffer
        sets: the stream an unpack reads was written three launches ago and comes from
        HBM, and no unpack follows a pack.  In the three-call step the two run right
        behind each other and share the stream through the Infinity Cache."""
        adt, torch = self.adt, self.torch
        out = {}
        for name, kernel, call in (
                ("adt_pack", "pack_kernel",
                 lambda i: adt.adt_pack(self.w, self.off, self.rb, out=self.packed[i % ROTATE])),
                ("adt_unpack", "unpack_kernel",
                 lambda i: adt.adt_unpack(self.packed[i % ROTATE], self.off, self.rb,
                                          out=self.w_out[i % ROTATE]))):
            for i in range(ROTATE):             # every stream buffer holds a valid stream
                adt.adt_pack(self.w, self.off, self.rb, out=self.packed[i])
            for i in range(5):
                call(i)
            torch.cuda.synchronize()
            settle_clocks(torch, call)
            adt.adt_timing_enable(True, launches)
            adt.adt_timing_read()
            for i in range(launches):
                call(i)
            torch.cuda.synchronize()
            t = adt.adt_timing_read()[kernel]
            adt.adt_timing_enable(False)
            avg = t["total_ms"] / max(t["launches"], 1)
            out[name] = {"launches_timed": int(t["launches"]), "avg_ms": round(avg, 5),
                         "min_ms": round(t["min_ms"], 5),
                         "gbps": round(self.bytes_pack / avg / 1e6, 1),
                         "hbm_frac": round(self.bytes_pack / avg / 1e6 / HBM_PEAK_GBPS, 4)}
        out["note"] = ("each call in a loop of its own over rotating buffers (cache neutral); up to 320 MiB "
                       "adt_pack writes its stream with ordinary stores so that an unpack right behind it "
                       "finds it in the Infinity Cache, which is what the three-call step measures")
        return out

    def config_summary(self):
        """The short form reported under "configs"."""
        plan = self.plan_path()
        calls = self.three_calls()
        pu = self.pack_unpack(max(10, min(self.steps, 30)))
        k = calls["kernels"]
        return {"n_weights": self.N, "n_layers": self.L, "packed_bytes": self.packed_bytes,
                "fp32_bytes": 4 * self.N, "steps": self.steps,
                "plan_us_per_step": round(plan["ms_per_step"] * 1e3, 1),
                "plan_fp32_gbps": plan["value"],
                "fused_us": round(plan["kernels"]["fused_kernel"]["avg_ms"] * 1e3, 1),
                "fused_hbm_frac": plan["kernels"]["fused_kernel"]["hbm_frac"],
                "plan_hbm_frac_whole_step": plan["hbm_frac_whole_step"],
                "three_calls_us_per_step": round(calls["ms_per_step"] * 1e3, 1),
                "pack_us": round(k["adt_pack"]["avg_ms"] * 1e3, 1), "pack_hbm_frac": k["adt_pack"]["hbm_frac"],
                "unpack_us": round(k["adt_unpack"]["avg_ms"] * 1e3, 1),
                "unpack_moved_frac": k["adt_unpack"]["hbm_frac"],
                "stats_us": round(k["awp_layer_stats"]["avg_ms"] * 1e3, 1),
                "stats_hbm_frac": k["awp_layer_stats"]["hbm_frac"],
                "pack_unpack_us": round(pu["avg_ms"] * 1e3, 1), "pack_unpack_hbm_frac": pu["hbm_frac"],
                "fits_infinity_cache": 4 * self.N < (256 << 20)}

    def free(self):
        self.w = self.packed = self.w_out = None
        self.torch.cuda.empty_cache()


def run_trajectory(adt, torch, workloads, steps=200):
    """The AWP trajectory: VGG-16-shaped weights take `steps` steps of a multiplicative
    random walk (w += N(0, (1e-3 |w|)^2), generated on the device: input generation,
    outside the library and outside the timed events); every step runs the whole pass
    through the plan with the synthetic AWP parameters T = 0, INTERVAL = 20, N = 8
    (the paper's own thresholds cannot fire within 200 steps).  HIP events on the
    launch stream bracket each step's library work."""
    ws = workloads.make_weight_set("vgg16")
    off, N, L = ws.layer_offsets, ws.n_weights, ws.n_layers
    sizes = np.diff(off)
    w = torch.from_numpy(ws.weights).cuda()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    packed = [torch.empty(4 * N, dtype=torch.uint8, device="cuda") for _ in range(ROTATE)]
    w_out = [torch.empty_like(w) for _ in range(ROTATE)]
    plan = adt.AwpPlan(off, 0.0, 20, 8)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(steps)]
    settle_clocks(torch, lambda i: w_out[i % ROTATE].copy_(w))    # plain copies: the plan's state stays untouched
    prev, per_step = None, []
    for s in range(steps):
        if s:
            noise = torch.randn(N, generator=gen, device="cuda", dtype=torch.float32)
            w.addcmul_(noise, w.abs(), value=1e-3)
            del noise
        ev[s][0].record()
        plan.step(w, packed[s % ROTATE], w_out[s % ROTATE])
        plan.flush()                         # the step's final reduction, if it was left for later
        ev[s][1].record()
        rb = plan.read()["bytes"]            # waits; outside the step's events
        changed = prev is not None and not np.array_equal(rb, prev)
        per_step.append((ev[s][0].elapsed_time(ev[s][1]), changed,
                         float(np.sum(sizes * (8 + rb.astype(np.int64))))))
        prev = rb
    plan.close()
    ms = np.array([p[0] for p in per_step[1:]])
    ch = np.array([p[1] for p in per_step[1:]])
    out = {"steps": steps, "awp_parameters": {"T": 0.0, "interval": 20, "n_bits": 8, "start_bits": 8},
           "ms_per_step_mean": round(float(ms.mean()), 5),
           "ms_per_step_median": round(float(np.median(ms)), 5),
           "fp32_gbps_mean": round(4.0 * N / float(ms.mean()) / 1e6, 1),
           "steps_with_a_changed_byte_count": int(ch.sum()),
           "ms_per_unchanged_step": round(float(ms[~ch].mean()), 5),
           "final_bytes_per_layer": prev.tolist(),
           "final_packed_bytes": int(np.sum(sizes * prev.astype(np.int64))),
           "timing": "HIP events on the launch stream around each awp_adt_step"}
    if ch.any():
        out["ms_per_changed_step"] = round(float(ms[ch].mean()), 5)
        out["redo_cost_ms"] = round(float(ms[ch].mean() - ms[~ch].mean()), 5)
    return out


def cpu_baselines(ws, rb_start_bits, params, workload, unit, seconds):
    import oracle
    off, L, N = ws.layer_offsets, ws.n_layers, ws.n_weights
    T, INTERVAL, N_BITS = params
    ostate = oracle.AwpState(L)
    ostate.bits[:] = rb_start_bits
    passes, c0 = 0, time.perf_counter()
    while passes < 2 or time.perf_counter() - c0 < seconds:
        st = oracle.stats(ws.weights, off)
        orb = oracle.awp_update(ostate, st[:, 1], T, INTERVAL, N_BITS)
        stream_bytes = oracle.pack(ws.weights, off, orb)
        oracle.unpack(stream_bytes, off, orb)
        passes += 1
    c1 = time.perf_counter()
    single = {"value": round(4.0 * N * passes / (c1 - c0) / 1e9, 3),
              "unit": unit, "cores": 1, "kind": "oracle",
              "sample": "%d full passes (stats + rule + pack + unpack) of the scalar C oracle "
                        "over the same %s weight set, %.1f s" % (passes, workload, c1 - c0),
              "host_cpus_visible": os.cpu_count()}
    # The same oracle on all host cores: pack, unpack and the sum of squares are
    # independent per weight (Section III-A), so every layer is cut into chunks
    # that the oracle takes as layers of their own; the harness only hands the
    # chunks to threads and adds the chunks' sums of squares up per layer.
    from concurrent.futures import ThreadPoolExecutor
    n_thr = max(1, min(os.cpu_count() or 1, 16))
    chunk = 1 << 20
    pieces = [(l, a, min(a + chunk, int(off[l + 1])))
              for l in range(L) for a in range(int(off[l]), int(off[l + 1]), chunk)]

    def oracle_piece(args_):
        l, a, b = args_
        t = np.array([0, b - a], dtype=np.int64)
        rbl = orb[l:l + 1]
        sq = oracle.stats(ws.weights[a:b], t)[0, 0]
        sb = oracle.pack(ws.weights[a:b], t, rbl)
        oracle.unpack(sb, t, rbl)
        return l, sq

    with ThreadPoolExecutor(n_thr) as pool:
        passes, c0 = 0, time.perf_counter()
        while passes < 2 or time.perf_counter() - c0 < seconds:
            sumsq = np.zeros(L)
            for l, sq in pool.map(oracle_piece, pieces):
                sumsq[l] += sq
            orb = oracle.awp_update(ostate, np.sqrt(sumsq), T, INTERVAL, N_BITS)
            passes += 1
        c1 = time.perf_counter()
    multi = {"value": round(4.0 * N * passes / (c1 - c0) / 1e9, 3),
             "unit": unit, "cores": n_thr, "kind": "oracle",
             "sample": "%d full passes of the same oracle, its calls spread over %d threads in "
                       "chunks of %d weights, %.1f s" % (passes, n_thr, chunk, c1 - c0)}
    return single, multi


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="vgg16_all2", choices=sorted(WORKLOADS))
    ap.add_argument("--cpu-seconds", type=float, default=10.0,
                    help="lower bound on each CPU-oracle timing loop (0 = skip)")
    ap.add_argument("--prime", type=int, default=450,
                    help="untimed passes before the warm-up of the paths whose launches carry "
                         "large kernel-argument tables (see PRIMING below)")
    ap.add_argument("--config-steps", type=int, default=40,
                    help="timed steps per path for each workload under \"configs\" (0 = skip)")
    ap.add_argument("--trajectory-steps", type=int, default=200,
                    help="steps of the AWP trajectory (0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed regions, run one plain device copy of the weight "
                         "buffer (4N bytes read, 4N written): the known-size kernel that "
                         "rocprofv3 counter runs are scaled by")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no GPU work: turn the output folders of two rocprofv3 --pmc runs of "
                         "`bench.py --calibrate-copy` (FETCH_SIZE, WRITE_SIZE) into profiles/traffic.json")
    ap.add_argument("--ablation", action="store_true",
                    help="instead of the benchmark line, time the ablation variants (naive "
                         "per-weight kernels, direct narrow stores, one launch per layer) "
                         "against the production kernels and print one JSON line")
    args = ap.parse_args()
    if args.traffic_from:
        import workloads
        n = int(workloads.layer_sizes(workloads.SHAPES[WORKLOADS[args.workload][0]]()).sum())
        return traffic_from_counters(args.traffic_from[0], args.traffic_from[1], args.workload, n)
    if args.ablation:
        return run_ablation(args)
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (no collectives, no multi-GPU "
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

    # PRIMING.  Once per process, one HIP kernel launch blocks the host for 30-40 ms.
    # Where it happens depends on the kernel-argument bytes the process has pushed:
    # around the 360th-410th launch of adt_pack_unpack (2.8 KB of arguments: the
    # per-layer table rides in them), around the 1600th call of awp_layer_stats
    # (2.2 KB per call), never within 9000 launches of the plan path (0.3 KB per
    # step) or of a plain torch copy.  The library allocates nothing in those calls;
    # the time is spent inside the runtime's launch call.  The plan path (the
    # headline) therefore needs no priming; the paths with large arguments run
    # `--prime` untimed passes first, which keeps that one-time event of the
    # runtime out of their timed regions whatever --warmup is.
    h = Harness(adt, torch, workloads, args.workload, args.steps, args.warmup, max(args.prime, 0))
    unit = "GB/s of FP32 weights through one full pass (stats + AWP rule + pack + unpack)"

    plan = h.plan_path()
    in_place = h.plan_path(rotate=False)
    graph = h.plan_graph_replay()
    calls = h.three_calls()
    plan16 = h.plan_path(out16=True)
    plan_send = h.plan_path(no_out=True)
    fused_pack_unpack = h.pack_unpack(max(10, min(args.steps, 50)))
    apart = h.pack_and_unpack_apart(max(10, min(args.steps, 50)))
    if args.calibrate_copy:
        h.w_out[0].copy_(h.w)
        torch.cuda.synchronize()

    result = {
        "metric": "ADT pack+unpack GB/s of FP32 weights (and % of HBM peak); AWP stats GB/s",
        "value": plan["value"],
        "unit": unit,
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": plan["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32 bit fields (pack/unpack), f64 accumulate (stats)",
        "data": "synthetic He-normal CNN-shaped FP32 weights, resident in HBM",
        "config": {"workload": args.workload, "n_weights": h.N, "n_layers": h.L,
                   "bytes_per_layer": h.rb.tolist(), "packed_bytes": h.packed_bytes,
                   "path": "awp_adt_step (plan)",
                   "output_buffers": "rotating over %d sets (cache neutral)" % ROTATE},
        "kernel_timing": "dispatch begin/end timestamps on %d of the %d timed steps" % (
            h.n_sampled, args.steps),
        "roofline": plan["roofline"],
        "roofline_cache_neutral": {
            "frac": plan["roofline"]["frac"], "achieved": plan["roofline"]["achieved"],
            "note": "the same figure as `roofline`: every timed loop rotates its output buffers, "
                    "so the Infinity Cache cannot absorb rewrites; this is the HBM figure"},
        "in_place_rewrite": {
            "note": "one output buffer set rewritten every step: HBM plus Infinity Cache, "
                    "not an HBM figure",
            "value": in_place["value"], "ms_per_step": in_place["ms_per_step"],
            "fused_kernel": in_place["kernels"]["fused_kernel"],
            "hbm_frac_whole_step": in_place["hbm_frac_whole_step"]},
        "plan_graph_replay": graph,
        "fused_pack_unpack": fused_pack_unpack,
    }
    for k, v in plan.items():
        if k not in ("value", "ms_per_step", "roofline", "settle_steps"):
            result[k] = v
    result["three_call_path"] = calls
    result["pack_and_unpack_apart"] = apart
    result["plan_bf16_out"] = {"value": plan16["value"], "ms_per_step": plan16["ms_per_step"],
                               "fused_kernel": plan16["kernels"]["fused_kernel"],
                               "algorithmic_bytes_per_launch": h.bytes_fused16}
    result["plan_stream_only"] = {"value": plan_send["value"], "ms_per_step": plan_send["ms_per_step"],
                                  "fused_kernel": plan_send["kernels"]["fused_kernel"],
                                  "algorithmic_bytes_per_launch": h.bytes_pack,
                                  "note": "awp_adt_step without the truncated copy: statistics, rule and "
                                          "stream in one launch, 4 + r bytes per weight"}
    result["priming_steps"] = {"plan": 0, "three_call_path": h.prime, "fused_pack_unpack": h.prime}
    result["clock_settle"] = {
        "seconds": SETTLE_SECONDS, "untimed_plan_steps_before_the_headline_loop": plan["settle_steps"],
        "note": "an idle GPU takes about 15 ms of work to raise its clocks again (first 25 steps "
                "after idleness 7-10 % slow, the next 40 steps 2-3 % slow); every timed loop follows "
                "--warmup steps plus this much untimed work of the same kind, so the figures are "
                "those of a loop that keeps running"}

    head_ws, head_bits = h.ws, h.start_bits
    h.free()
    if args.config_steps > 0:
        configs = {}
        for name in OTHER_CONFIGS:
            if name == args.workload:
                continue
            c = Harness(adt, torch, workloads, name, args.config_steps, 5, 20)
            configs[name] = c.config_summary()
            c.free()
        result["configs"] = configs
    if args.trajectory_steps > 0:
        result["trajectory"] = run_trajectory(adt, torch, workloads, args.trajectory_steps)
    result["paper_context"] = PAPER_CONTEXT

    if args.cpu_seconds > 0:
        single, multi = cpu_baselines(head_ws, head_bits, (Harness.T, Harness.INTERVAL, Harness.N_BITS),
                                      args.workload, unit, args.cpu_seconds)
        result["cpu_baseline"] = single
        result["cpu_baseline_all_cores"] = multi
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
