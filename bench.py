#!/usr/bin/env python3
"""Benchmark of the fused INT3/INT4 + low-rank linear layer on one MI355X.

A step is one pass of the whole hot path (down-projection + fused kernel for every layer of the
configuration) over one batch of seeded synthetic input.  Default workload: the Llama2-7B-shaped
decode layer set at M = 1 (q/k/v/o 4096x4096, gate/up 4096->11008, down 11008->4096, INT4, group
128, rank 64).  Weights are quantized on the GPU by the library's own feedback quantizer; every
step works on a different copy of the packed layer set so that neither L2 nor the 256 MB
Infinity Cache can serve the weights (the copies rotate over > 2 GB).

Prints ONE JSON line (see the design doc for the meaning of every field).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import fbq_synth  # noqa: E402

HBM_PEAK_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=1, help="index into the benchmark configurations")
    ap.add_argument("--M", type=int, default=0, help="tokens (default: first M of the configuration)")
    ap.add_argument("--copies", type=int, default=0, help="distinct copies of the layer set (default: > 2 GB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    return ap.parse_args()


def build_layer_set(specs, config, M, torch, fbq):
    """Seeded tensors -> GPU feedback quantizer -> packed device layers (+ x per layer)."""
    layers, xs = [], []
    for li, spec in enumerate(specs):
        W = fbq_synth.make_weight(spec, config, li)
        A, B = fbq_synth.make_branch(spec, config, li)
        t16 = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()
        d = fbq.Desc(spec.N, spec.K, spec.r, spec.bits, spec.group)
        Ad = t16(A.T) if spec.r else None
        Btd = t16(B.T) if spec.r else None
        Wd = t16(W)
        layers.append(fbq.quantize_feedback(d, Wd, Ad, Btd))
        torch.cuda.synchronize()
        del Wd
        xs.append(t16(fbq_synth.make_x(spec, M, config, li)))
    return layers, xs


def clone_layer(layer, fbq):
    c = lambda t: None if t is None else t.clone()
    return fbq.DeviceLayer(layer.desc, c(layer.qweight), c(layer.scales), c(layer.zeros), c(layer.At), c(layer.Bt))


class Launcher:
    """Pre-marshalled ctypes arguments of one fbq_linear call (keeps Python overhead off the stream)."""

    def __init__(self, fbq, layer, x, y, ws, M, stream_ptr):
        self.fn = fbq.load().fbq_linear
        d = layer.desc
        self.desc = d.c()
        p = lambda t: ctypes.c_void_p(0 if t is None else t.data_ptr())
        self.args = (ctypes.byref(self.desc), M, p(x), p(layer.qweight), p(layer.scales), p(layer.zeros), p(layer.At),
                     p(layer.Bt), p(y), p(ws), ctypes.c_size_t(0 if ws is None else ws.numel()), stream_ptr)

    def __call__(self):
        rc = self.fn(*self.args)
        if rc:
            raise RuntimeError(f"fbq_linear failed with status {rc}")


def cpu_baseline(specs, config, M, seconds):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    from oracle import fbq_oracle as orc
    spec = specs[0]
    rows = min(spec.N, 512)
    sub = fbq_synth.LayerSpec(spec.name, rows, spec.K, spec.r, spec.bits, spec.group, spec.w_std, spec.ab_std,
                              spec.outlier_p, spec.outlier_mul)
    W = fbq_synth.make_weight(sub, config, 0)
    A, B = fbq_synth.make_branch(sub, config, 0)
    x = fbq_synth.make_x(sub, M, config, 0)
    Aa, Bb = (A, B) if sub.r else (None, None)
    codes, s, z = orc.quantize(W, Aa, Bb, sub.bits, sub.group)
    words = orc.pack(codes, sub.bits)
    orc.linear(x, words, s, z, Aa, Bb, sub.bits, sub.group)          # warm-up
    reps, t0 = 0, time.perf_counter()
    while True:
        orc.linear(x, words, s, z, Aa, Bb, sub.bits, sub.group)
        reps += 1
        el = time.perf_counter() - t0
        if el >= seconds or reps >= 2000:
            break
    nbytes = fbq_synth.algorithmic_bytes(rows, sub.K, sub.r, sub.bits, M, sub.group)
    return {"value": round(nbytes * reps / el / 1e9, 4), "unit": "GB/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{reps} passes of the fp64 oracle over the first {rows} output rows of layer '{spec.name}' "
                      f"({spec.K}->{spec.N}, INT{spec.bits}, r={spec.r}, M={M}), {el:.1f} s",
            "us_per_layer_extrapolated": round(el / reps * 1e6 * spec.N / rows, 1)}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no collective); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2501_16385_amd as fbq
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        sys.exit(3)
    fbq.load()
    torch.cuda.set_device(0)

    specs, Ms = fbq_synth.config_layers(args.config)
    M = args.M or Ms[0]
    base_layers, xs = build_layer_set(specs, args.config, M, torch, fbq)
    set_bytes = sum(fbq_synth.algorithmic_bytes(s.N, s.K, s.r, s.bits, M, s.group) for s in specs)
    copies = args.copies or max(2, int(np.ceil(2.2e9 / set_bytes)))
    sets = [base_layers] + [[clone_layer(l, fbq) for l in base_layers] for _ in range(copies - 1)]

    stream = torch.cuda.current_stream()
    sp = ctypes.c_void_p(stream.cuda_stream)
    ys = [torch.empty((M, s.N), dtype=torch.float16, device="cuda") for s in specs]
    wss = [torch.zeros(max(16, fbq.workspace_bytes(l.desc, M)), dtype=torch.uint8, device="cuda") for l in base_layers]
    steps_fused = [[Launcher(fbq, l, xs[i], ys[i], wss[i] if l.desc.r else None, M, sp) for i, l in enumerate(ls)]
                   for ls in sets]

    # branch-free twins (r = 0) of the same packed layers: the comparator of "branch overhead %"
    def twin(l):
        d = fbq.Desc(l.desc.N, l.desc.K, 0, l.desc.bits, l.desc.group)
        return fbq.DeviceLayer(d, l.qweight, l.scales, l.zeros, None, None)
    steps_plain = [[Launcher(fbq, twin(l), xs[i], ys[i], None, M, sp) for i, l in enumerate(ls)] for ls in sets]

    def run(step_list, n, first=0):
        for s in range(n):
            for call in step_list[(first + s) % len(step_list)]:
                call()

    def timed(step_list, n, first):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)
        run(step_list, n, first)
        e1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return e0.elapsed_time(e1) / n, wall / n * 1e3      # ms per step: device events, host wall clock

    run(steps_fused, args.warmup)
    ms_fused, wall_fused = timed(steps_fused, args.steps, args.warmup)
    run(steps_plain, args.warmup)
    ms_plain, _ = timed(steps_plain, args.steps, args.warmup)

    # per-layer timings of the fused kernel alone (dominant kernel): events around each launch of a
    # dedicated pass, r = 0 twin launches so that exactly one kernel sits between the two events
    per_layer = []
    for i, spec in enumerate(specs):
        calls = [st[i] for st in steps_fused]
        for c in calls[: min(len(calls), 20)]:
            c()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        n = max(args.steps, 100)
        e0.record(stream)
        for s in range(n):
            calls[s % len(calls)]()
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / n * 1e3
        nbytes = fbq_synth.algorithmic_bytes(spec.N, spec.K, spec.r, spec.bits, M, spec.group)
        per_layer.append({"layer": spec.name, "N": spec.N, "K": spec.K, "us": round(us, 3),
                          "GBps": round(nbytes / us / 1e3, 1)})

    n_layers = len(specs)
    gbps = set_bytes / (ms_fused * 1e-3) / 1e9
    floor = sum(2 * s.r * (s.K + s.N) for s in specs) / sum(
        fbq_synth.algorithmic_bytes(s.N, s.K, 0, s.bits, M, s.group) for s in specs)
    # dominant kernel: the fused GEMV.  Its algorithmic bytes per launch = everything the layer must
    # move except A (read by the down-projection kernel): codes, scale+zero, Bt, x, y.
    fused_bytes = sum(fbq_synth.algorithmic_bytes(s.N, s.K, s.r, s.bits, M, s.group) - 2 * s.r * s.K for s in specs)
    plain_bytes = sum(fbq_synth.algorithmic_bytes(s.N, s.K, 0, s.bits, M, s.group) for s in specs)
    launches = n_layers
    avg_us_plain = ms_plain * 1e3 / launches
    out = {
        "metric": "fused W4/W3+low-rank linear: effective HBM GB/s (with us/layer and branch overhead %)",
        "value": round(gbps, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_fused, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": f"int{specs[0].bits} codes, f16 in/out, f32 accumulate", "data": "synthetic",
        "config": {"workload": f"config {args.config}: " + ", ".join(sorted({f'{s.K}->{s.N}' for s in specs})) +
                   f"; {n_layers} layers/step, INT{specs[0].bits}, group 128, rank {specs[0].r}, M={M}",
                   "layers_per_step": n_layers, "copies_rotated": copies, "launch_mode": "per-layer (2 launches each)"},
        "us_per_layer": round(ms_fused * 1e3 / n_layers, 3),
        "us_per_layer_branch_free": round(ms_plain * 1e3 / n_layers, 3),
        "branch_overhead_pct": round((ms_fused / ms_plain - 1) * 100, 2),
        "branch_overhead_byte_floor_pct": round(floor * 100, 2),
        "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBS, 4),
        "wall_ms_per_step": round(wall_fused, 6),
        "per_layer": per_layer,
        "roofline": {"bound": "hbm", "kernel": "fbq_gemv_kernel (branch-free launches, one kernel per event interval)",
                     "achieved": round(plain_bytes / launches / avg_us_plain / 1e3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(plain_bytes / launches / avg_us_plain / 1e3 / HBM_PEAK_GBS, 4), "traffic": None,
                     "avg_launch_us": round(avg_us_plain, 3), "bytes_per_launch": plain_bytes // launches},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(specs, args.config, M, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
