#!/usr/bin/env python3
"""Benchmark of the LCD table-lookup linear layer on one MI355X.

Workload (N=1): the LLaMA-7B-shaped decoder linear set at M=1 with 3-bit indices
(q/k/v/o 4096x4096, gate/up 11008x4096, down 4096x11008), synthetic seeded inputs.  A step is
one pass of the decode hot path over the whole set: activation smoothing, table lookup +
accumulation and the row reduction for all seven matrices (index packing and table build are
offline, once per layer, and happen before the timed region).  The metric is effective GB/s on
the packed-index bytes (N*K*bits/8 summed over the set) with inputs resident in HBM.

Every timed step streams a different replica of the packed matrices (>= 600 MB in rotation), so
the 256 MB last-level cache cannot serve them; steps are replayed from a HIP graph so that the
host's launch cost is not what is measured.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=1, help="benchmark config index (1 = the metric's workload)")
    ap.add_argument("--m", type=int, default=None, help="token count (default: the config's first M)")
    ap.add_argument("--replicas", type=int, default=0, help="packed-matrix replicas in rotation (0 = enough for 600 MB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the secondary measurements (other configs)")
    ap.add_argument("--per-layer", action="store_true", help="one lcd_lut_gemv call per matrix instead of one grouped call per step")
    ap.add_argument("--bits", type=int, default=None, choices=[2, 3, 4], help="override the config's index width (4: the 16-centroid container)")
    ap.add_argument("--act-int8", action="store_true", help="INT8 activation codes (input transformation of Sec. 4.1) instead of fp16 x/s")
    ap.add_argument("--offline", action="store_true", help="time the offline kernels (assign, counts, merge, pack, table build) on the config's largest matrix instead of the hot path")
    ap.add_argument("--eager", action="store_true", help="launch every step from Python instead of replaying a HIP graph")
    ap.add_argument("--library-gemm", action="store_true", help="prefill configs: also time the vendor library's dense fp16 GEMM (torch.matmul) on the same shapes, as context for the roofline fraction")
    return ap.parse_args()


def resolve_config(index, bits=None):
    """A config of synth.configs, optionally with another index width on the same shapes."""
    import dataclasses
    import synth
    cfg = synth.get_config(index)
    if bits is not None and bits != cfg.bits:
        cfg = dataclasses.replace(cfg, bits=bits, label=f"{cfg.label} [shapes only: index width set to {bits} bits]")
    return cfg


def dependency_stages(cfg):
    """Indices of the config's matrices grouped into the launches of a decoder block: layers that read the
    same input share a launch (q, k, v | o | gate, up | down); a single matrix is a stage of its own."""
    stages, i = [], 0
    for spec in cfg.layers:
        if spec.name == "qkvo":
            stages += [[i, i + 1, i + 2], [i + 3]]
        elif spec.name == "gate_up":
            stages.append([i, i + 1])
        else:
            stages += [[i + j] for j in range(spec.count)]
        i += spec.count
    return stages


class LayerSet:
    """Device-resident inputs of one config: per matrix R replicas of (packed, lut), x, s, y, workspace."""

    def __init__(self, cfg_index, M, replicas, keep_host=False, per_layer=False, act_int8=False, bits=None):
        import numpy as np
        import torch
        import synth
        import paper_2506_12038_amd as lcd

        self.cfg = resolve_config(cfg_index, bits)
        self.per_layer = per_layer
        self.act_int8 = act_int8
        self.bits = self.cfg.bits
        self.M = M
        self.entry = lcd.lcd_lut_gemv if M <= 16 else lcd.lcd_lut_gemm
        self.mats = []
        self.host = []
        cache = {}
        for mid, spec in self.cfg.matrices():
            layer = synth.make_layer(cfg_index, mid, spec.N, spec.K, self.bits, M)
            dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
            packed0 = lcd.lcd_pack_indices(dev(layer["idx"]), self.bits)
            lut0 = lcd.lcd_build_lut(dev(layer["codebook"]), self.bits)
            packed = [packed0] + [packed0.clone() for _ in range(replicas - 1)]
            luts = [lut0] + [lut0.clone() for _ in range(replicas - 1)]
            ws = torch.empty(lcd.lcd_workspace_bytes(M, spec.N, spec.K, self.bits), dtype=torch.uint8, device="cuda")
            # INT8 activation variant: the quantisation step puts the 99th percentile of |x/s| at code 127
            s_q = float(np.float32(np.quantile(np.abs(layer["x"].astype(np.float64) / layer["s"]), 0.99) / 127.0))
            self.mats.append(dict(spec=spec, packed=packed, lut=luts, x=dev(layer["x"]), s=dev(layer["s"]), s_q=s_q,
                                  y=torch.empty((M, spec.N), dtype=torch.float16, device="cuda"), ws=ws))
            if keep_host:
                self.host.append(layer)
            del layer
        torch.cuda.synchronize()
        self.index_bytes = sum(m["spec"].N * m["spec"].K * self.bits // 8 for m in self.mats)
        self.flops = sum(2 * M * m["spec"].N * m["spec"].K for m in self.mats)
        self.total_bytes = self.index_bytes + sum(
            m["spec"].N * (1 << self.bits) * 2 + M * m["spec"].K * 2 + m["spec"].K * 4 + M * m["spec"].N * 2 for m in self.mats)

        self.groups = None
        self.block_groups = None
        if M <= 16:
            self.groups = [lcd.GemvGroup([(m["packed"][r], m["lut"][r], m["x"], m["s"], m["y"], m["spec"].N) for m in self.mats],
                                         self.bits, s_q=[m["s_q"] for m in self.mats] if act_int8 else None)
                           for r in range(replicas)]
            # The same layers as a decoder block would run them: layers that read the same input go out together
            # (q, k, v | o | gate, up | down), the launches of a step one after the other on the stream, and the
            # layers of one launch share ONE input vector and smoothing factor, as they do in a block.
            self.stages = dependency_stages(self.cfg)
            self.block_groups = []
            for r in range(replicas):
                per_stage = []
                for stage in self.stages:
                    first = self.mats[stage[0]]
                    per_stage.append(lcd.GemvGroup([(self.mats[i]["packed"][r], self.mats[i]["lut"][r], first["x"], first["s"],
                                                     self.mats[i]["y"], self.mats[i]["spec"].N) for i in stage],
                                                   self.bits, s_q=[first["s_q"]] * len(stage) if act_int8 else None))
                self.block_groups.append(per_stage)
        elif not per_layer:   # prefill: one grouped call (a smoothing launch and a matrix launch) for the whole set
            shared_ws = None
            self.groups = []
            for r in range(replicas):
                g = lcd.GemmGroup([(m["packed"][r], m["lut"][r], m["x"], m["s"], m["y"], m["spec"].N) for m in self.mats],
                                  self.bits, workspace=shared_ws, s_q=[m["s_q"] for m in self.mats] if act_int8 else None)
                shared_ws = g.workspace
                self.groups.append(g)

    def block_step(self, replica):
        """One decode step in dependency order: one grouped launch per stage."""
        for g in self.block_groups[replica]:
            g()

    def matrix_step(self, index, replica):
        """One single-matrix call (lcd_lut_gemv / lcd_lut_gemm) on matrix `index`."""
        m = self.mats[index]
        self.entry(m["packed"][replica], m["lut"][replica], m["x"], m["s"], m["spec"].N, self.bits, y=m["y"], workspace=m["ws"])

    def step(self, replica):
        if self.groups is not None and not self.per_layer:
            self.groups[replica]()
            return
        for m in self.mats:
            self.entry(m["packed"][replica], m["lut"][replica], m["x"], m["s"], m["spec"].N, self.bits,
                       y=m["y"], workspace=m["ws"])


def time_steps(ls, replicas, steps, warmup, eager, step_fn=None, per_replay=False):
    """Returns (wall ms per step, event ms per step).  Exactly `steps` timed steps of step_fn(replica)
    (default: the set's step).  per_replay: a third result, the event time per step of every graph replay
    (one replay = `replicas` steps), taken with an event between replays."""
    import torch

    stream = torch.cuda.Stream()
    graphs = {}
    step = step_fn or ls.step
    marks = []

    def run(n_steps, first):
        """Enqueue n_steps on `stream`, rotating replicas starting at `first`."""
        if eager:
            with torch.cuda.stream(stream):
                for i in range(n_steps):
                    step((first + i) % replicas)
            return
        done = 0
        while done < n_steps:
            chunk = min(replicas, n_steps - done)
            key = chunk
            if key not in graphs:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for r in range(chunk):
                        step(r)
                graphs[key] = g
            with torch.cuda.stream(stream):
                graphs[key].replay()
                if per_replay and timing[0]:
                    e = spare.pop()
                    e.record(stream)
                    marks.append((e, chunk))
            done += chunk

    timing = [False]
    spare = [torch.cuda.Event(enable_timing=True) for _ in range(steps // max(replicas, 1) + 2)] if per_replay else []
    for e in spare:
        e.record(stream)               # events are created lazily: not inside the timed region
    with torch.cuda.stream(stream):
        step(0)                        # first call outside capture (lazy module load)
    torch.cuda.synchronize()
    if not eager:                      # build every graph the timed loop needs before timing
        run(replicas, 0)
        if steps % replicas:
            run(steps % replicas, 0)
        if warmup % replicas and warmup > 0:
            run(warmup % replicas, 0)
    torch.cuda.synchronize()
    run(warmup, 0)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        e0.record(stream)
    timing[0] = True
    run(steps, 0)
    with torch.cuda.stream(stream):
        e1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if not per_replay:
        return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps
    samples, prev = [], e0
    for e, chunk in marks:
        samples.append(prev.elapsed_time(e) / chunk)
        prev = e
    # Now and then a replay takes milliseconds in this mode (the host stalls while it records the event between
    # two replays and the GPU runs dry; the headline region records no such events).  The percentiles ignore
    # that by themselves; the mean is taken over the replays within five times the median, and the number of
    # replays left out is reported.
    if not samples:
        return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps, samples, 0
    med = sorted(samples)[len(samples) // 2]
    kept = [(s, c) for s, (_, c) in zip(samples, marks) if s <= 5.0 * med]
    mean = sum(s * c for s, c in kept) / max(1, sum(c for _, c in kept))
    return (t1 - t0) * 1e3 / steps, mean, samples, len(samples) - len(kept)


def percentiles(samples_ms):
    """median / p10 / p90 of per-step times (us) over graph replays."""
    import numpy as np
    a = np.asarray(samples_ms, dtype=np.float64) * 1e3
    if a.size == 0:          # eager launches: there are no replays to tell apart
        return {"median_us": None, "p10_us": None, "p90_us": None, "samples": 0}
    return {"median_us": float(np.median(a)), "p10_us": float(np.percentile(a, 10)), "p90_us": float(np.percentile(a, 90)),
            "min_us": float(a.min()), "max_us": float(a.max()), "samples": int(a.size)}


def secondary_measurements(ls, replicas, steps, warmup, eager, decode):
    """Beside the headline (same inputs, separate timed regions, HIP events on the launch stream):
    the spread of the step time over graph replays, the step in the dependency order of a decoder block
    (decode only), and every distinct matrix on its own (one single-matrix call per step)."""
    out = {}
    steps2 = max(replicas * 8, min(steps, 1000) // replicas * replicas)
    _, ev, samples, first = time_steps(ls, replicas, steps2, min(warmup, 50), eager, per_replay=True)   # first: replays left out of the mean
    out["step_time_over_replays"] = dict(percentiles(samples), steps_per_replay=replicas, mean_us=ev * 1e3, stalled_replays_left_out_of_mean=first)
    if decode and ls.block_groups is not None and len(ls.stages) > 1:
        _, ev, samples, _ = time_steps(ls, replicas, steps2, min(warmup, 50), eager, step_fn=ls.block_step, per_replay=True)
        out["block_order_step"] = dict(
            percentiles(samples), mean_us=ev * 1e3, launches_per_step=len(ls.stages),
            stages=[[f"{ls.mats[i]['spec'].N}x{ls.mats[i]['spec'].K}" for i in st] for st in ls.stages],
            effective_GBps=ls.index_bytes / (ev * 1e-3) / 1e9, frac_of_hbm_peak=ls.index_bytes / (ev * 1e-3) / 1e9 / HBM_PEAK_GBS,
            what="the same set as a decoder block runs it: one grouped launch per group of layers that read the same input "
                 "(they share one x and s), the launches of a step in order on one stream, replayed from a HIP graph")
    per_matrix, seen = [], set()
    for i, m in enumerate(ls.mats if not ls.act_int8 else []):   # the single calls timed here are the fp16 entry points
        shape = (m["spec"].N, m["spec"].K)
        if shape in seen:
            continue
        seen.add(shape)
        _, ev, samples, _ = time_steps(ls, replicas, steps2, min(warmup, 50), eager, step_fn=lambda r, i=i: ls.matrix_step(i, r), per_replay=True)
        row = dict(percentiles(samples), matrix=f"{shape[0]}x{shape[1]}", mean_us=ev * 1e3)
        if decode:
            b = shape[0] * shape[1] * ls.bits // 8
            row.update(index_bytes=b, effective_GBps=b / (ev * 1e-3) / 1e9, frac_of_hbm_peak=b / (ev * 1e-3) / 1e9 / HBM_PEAK_GBS)
        else:
            f = 2.0 * ls.M * shape[0] * shape[1]
            row.update(flops=f, TFLOPs=f / (ev * 1e-3) / 1e12, frac_of_mfma_peak=f / (ev * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS)
        per_matrix.append(row)
    out["per_matrix_single_calls"] = per_matrix
    return out


def cpu_baseline(cfg_index, M, budget_s=12.0, bits=None):
    """The oracle as it stands, on this machine's host cores, on a bounded sample of the workload:
    every distinct matrix shape of the config once (rows capped for large M), repeated until about
    `budget_s` seconds of oracle time have been spent; the best pass is reported."""
    import oracle
    import synth

    cfg = resolve_config(cfg_index, bits)
    cap_weights = 4.0e8 / max(M, 1)          # per shape: keeps one pass at seconds, not minutes
    seen, layers, desc = set(), [], []
    for mid, spec in cfg.matrices():
        if (spec.N, spec.K) in seen:
            continue
        seen.add((spec.N, spec.K))
        rows = int(min(spec.N, max(16, cap_weights // spec.K // 16 * 16)))
        layers.append((rows, spec.K, synth.make_layer(cfg_index, mid, rows, spec.K, cfg.bits, M)))
        desc.append(f"{rows}x{spec.K}")
    sample_bytes = sum(rows * K * cfg.bits // 8 for rows, K, _ in layers)
    sample_flops = sum(2 * M * rows * K for rows, K, _ in layers)
    best, spent, passes = None, 0.0, 0
    while spent < budget_s and passes < 1000:
        t0 = time.perf_counter()
        for rows, K, layer in layers:
            oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], cfg.bits)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
        spent += dt
        passes += 1
    decode = M <= 16
    return {
        "value": (sample_bytes / best / 1e9) if decode else (sample_flops / best / 1e12),
        "unit": "GB/s" if decode else "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": f"config {cfg_index} at M={M}: rows x K = {', '.join(desc)} (each distinct matrix shape once), "
                  f"fp64 oracle, best of {passes} passes, {spent:.1f} s of oracle time in total",
    }


def measured_traffic(kernel, cfg_index):
    """HBM bytes per launch of the dominant kernel.  NOT measured by this run: rocprofv3 --pmc cannot run
    inside the timed program, so the figure is read from the committed summary of two counter runs
    (FETCH_SIZE / WRITE_SIZE, scaled by a copy of known size).  Returns (bytes, file name) or (None, None)."""
    f = ROOT / "profiles" / f"{kernel}_config{cfg_index}_hbm_traffic.txt"
    if not f.exists():
        return None, None
    for line in f.read_text().splitlines():
        if line.startswith("traffic_bytes_per_launch:"):
            return int(line.split(":")[1]), f"profiles/{f.name}"
    return None, None


def library_dense_gemm(cfg, M, steps, warmup):
    """Context only: the vendor library's dense fp16 GEMM (torch.matmul -> hipBLASLt) on fp16 weights of the
    config's shapes, same token count, same box.  It reads 16-bit weights and does no lookup; what it shows is
    the rate the chip sustains on this contraction size at the clock its power management allows."""
    import torch
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    mats = []
    for _, spec in cfg.matrices():
        x = torch.randn((M, spec.K), device="cuda", generator=g).to(torch.float16)
        w = (torch.randn((spec.N, spec.K), device="cuda", generator=g) * 0.02).to(torch.float16)
        mats.append((x, w.t()))
    for _ in range(warmup):
        for x, wt in mats:
            torch.matmul(x, wt)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        for x, wt in mats:
            torch.matmul(x, wt)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / steps
    flops = sum(2.0 * M * spec.N * spec.K for _, spec in cfg.matrices())
    return {"value": flops / us / 1e6, "unit": "TFLOP/s", "us_per_step": us,
            "what": "torch.matmul (vendor library) on dense fp16 weights of the same shapes and token count, eager launches"}


def bench_offline(cfg, steps, warmup):
    """Offline kernels on the largest matrix of the config: HIP-event time per call and the rate in
    algorithmic bytes (what the kernel must read and write once).  One JSON line."""
    import numpy as np
    import torch
    import paper_2506_12038_amd as lcd

    spec = max((s for _, s in cfg.matrices()), key=lambda s: s.N * s.K)
    N, K, bits = spec.N, spec.K, cfg.bits
    ncent = 1 << bits
    g = torch.Generator(device="cuda"); g.manual_seed(1)
    w = (torch.randn((N, K), device="cuda", generator=g) * 0.02).to(torch.float16)
    base = np.sort((np.random.default_rng(2).standard_normal(ncent) * 0.02).astype(np.float16))
    while len(np.unique(base)) < ncent:
        base = np.sort((np.random.default_rng(int(base.view(np.uint16).sum())).standard_normal(ncent) * 0.02).astype(np.float16))
    cb = torch.from_numpy(np.tile(base[None, :], (N, 1))).cuda()
    idx = lcd.lcd_assign_indices(w, cb, ncent, bits)
    counts = lcd.lcd_cluster_counts(idx, bits)
    packed = lcd.lcd_pack_indices(idx, bits)
    stream = torch.cuda.current_stream()
    weights = N * K

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / steps   # us

    idx_out = torch.empty_like(idx)
    rows = {
        "assign_kernel": (timed(lambda: lcd.lcd_assign_indices(w, cb, ncent, bits)), 3 * weights),
        "counts_kernel": (timed(lambda: lcd.lcd_cluster_counts(idx, bits)), weights),
        "merge_kernel+remap_kernel": (timed(lambda: lcd.lcd_merge_closest(cb, counts, idx, ncent, bits, idx_out=idx_out)), 2 * weights),
        "pack_kernel": (timed(lambda: lcd.lcd_pack_indices(idx, bits, out=packed)), weights + weights * bits // 8),
        "build_lut_kernel": (timed(lambda: lcd.lcd_build_lut(cb, bits)), N * ncent * 2 + lcd.lcd_lut_bytes(N, bits)),
    }
    out = {"metric": "offline_kernel_bandwidth_algorithmic_bytes", "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
           "data": "synthetic", "config": {"workload": f"offline kernels on {N}x{K}, {bits}-bit ({cfg.label})"},
           "kernels": {k: {"us": round(t, 2), "bytes": b, "GB/s": round(b / t / 1e3, 1), "frac_of_hbm_peak": round(b / t / 1e3 / HBM_PEAK_GBS, 3)}
                       for k, (t, b) in rows.items()}}
    print(json.dumps(out))


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import synth
    import paper_2506_12038_amd as lcd

    lcd.load_library()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = resolve_config(args.config, args.bits)
    M = args.m if args.m is not None else cfg.Ms[0]
    if args.offline:
        bench_offline(cfg, min(args.steps, 50), min(args.warmup, 5))
        return
    replicas = args.replicas or max(2, -(-600_000_000 // cfg.index_bytes()))
    if args.act_int8 and args.per_layer:
        sys.exit("--act-int8 applies to the grouped calls")
    ls = LayerSet(args.config, M, replicas, per_layer=args.per_layer, act_int8=args.act_int8, bits=args.bits)
    wall_ms, event_ms = time_steps(ls, replicas, args.steps, args.warmup, args.eager)

    decode = M <= 16
    n_launch = 1 if not args.per_layer else len(ls.mats)
    decode_kernel = "gemv_bucket_kernel" if (M == 1 and cfg.bits < 4) else "gemv_tokens_kernel"
    # the tokens kernel is preceded by a small activation-transform kernel for INT8 codes and for wide layers
    prepass = decode_kernel == "gemv_tokens_kernel" and not args.per_layer and (args.act_int8 or max(s.K for _, s in cfg.matrices()) >= 16384)
    if decode:
        metric, unit = "lut_gemv_effective_bandwidth_packed_index_bytes", "GB/s"
        value = ls.index_bytes / (wall_ms * 1e-3) / 1e9
        traffic, traffic_file = (measured_traffic(decode_kernel, args.config) if (n_launch == 1 and args.bits is None and not args.act_int8)
                                 else (None, None))
        roofline = {
            "bound": "hbm", "achieved": ls.index_bytes / (event_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": ls.index_bytes / (event_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_source": (f"{traffic_file}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, committed with the "
                               "kernel; not measured by this run") if traffic is not None else None,
            "kernel": decode_kernel,
            "launches_per_step": n_launch, "kernels_per_launch": 2 if prepass else 1, "algorithmic_bytes_per_step": ls.index_bytes,
            "avg_launch_us": event_ms * 1e3 / n_launch,
        }
    else:
        metric, unit = "lut_gemm_throughput", "TFLOP/s"
        value = ls.flops / (wall_ms * 1e-3) / 1e12
        roofline = {
            "bound": "mfma", "achieved": ls.flops / (event_ms * 1e-3) / 1e12, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": ls.flops / (event_ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, "traffic": None,
            "kernel": "gemm_kernel" if args.per_layer else "gemm_group_kernel", "launches_per_step": n_launch,
            "kernels_per_launch": 2, "algorithmic_flops_per_step": ls.flops,
            "avg_launch_us": event_ms * 1e3 / n_launch,
        }
    out = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 operands, f32 accumulate", "data": "synthetic",
        "config": {"workload": f"config {args.config}: {cfg.label}", "M": M, "bits": cfg.bits,
                   "matrices": [f"{m['spec'].N}x{m['spec'].K}" for m in ls.mats],
                   "activations": (f"int8 codes, input transformation of Sec. 4.1 (lcd_lut_{'gemv' if decode else 'gemm'}_q8_grouped)"
                                   if args.act_int8 else "fp16 x/s"),
                   "index_bytes_per_step": ls.index_bytes, "replicas_in_rotation": replicas,
                   "launch": ("eager" if args.eager else "hip graph replay") + (", one grouped launch per step" if n_launch == 1 else ", one call per matrix")},
        "roofline": roofline,
    }
    if not args.no_extra and not args.per_layer:
        out["secondary"] = secondary_measurements(ls, replicas, args.steps, args.warmup, args.eager, decode)
    del ls
    torch.cuda.empty_cache()
    if args.library_gemm and not decode:
        out["roofline"]["library_dense_fp16"] = library_dense_gemm(cfg, M, args.steps, args.warmup)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, M, bits=args.bits)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
