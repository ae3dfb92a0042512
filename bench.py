#!/usr/bin/env python3
"""Benchmark of the fused INT3/INT4 + low-rank linear layer on one MI355X.

A step is one pass of the whole hot path (in-launch down-projection + fused kernel, every layer of
the configuration) over one batch of seeded synthetic input.  Default workload: the
Llama2-7B-shaped decode layer set at M = 1 (q/k/v/o 4096x4096, gate/up 4096->11008,
down 11008->4096; INT4, group 128, rank 64).  Weights are quantized on the GPU by the library's
own feedback quantizer; every step works on a different copy of the packed layer set, so that
neither the L2s nor the 256 MB Infinity Cache can serve the weights (the copies rotate over > 2 GB).

Three launch schedules are timed (all produce identical y):
  staged     layers that can run together in a decoder share a launch: {q,k,v} {o} {gate,up} {down}
             -> 4 launches per step.  This is `value`.
  per_layer  one fbq_linear launch per layer -> 7 launches per step.
  merged     every layer with the same K in one launch -> 2 launches per step (the layers of the
             benchmark have independent inputs, so this is legal here; a decoder cannot do it).
Prints ONE JSON line (the design doc explains every field).
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
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=1, help="index into the benchmark configurations")
    ap.add_argument("--M", type=int, default=0, help="tokens (default: first M of the configuration)")
    ap.add_argument("--copies", type=int, default=0, help="distinct copies of the layer set (default: > 2 GB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-kernels", action="store_true", help="skip the context timings of the few-token and prefill kernels")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    return ap.parse_args()


def stages_of(specs):
    """Indices of layers that may run together in a decoder: same input, no dependency between them."""
    names = [s.name for s in specs]
    want = [["q_proj", "k_proj", "v_proj"], ["o_proj"], ["gate_proj", "up_proj"], ["down_proj"]]
    if all(n in names for grp in want for n in grp) and len(names) == 7:
        return [[names.index(n) for n in grp] for grp in want]
    return [[i] for i in range(len(specs))]


def build_layer_set(specs, config, M, torch, fbq):
    """Seeded tensors -> GPU feedback quantizer -> packed device layers (+ x per layer)."""
    layers, xs = [], []
    t16 = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()
    for li, spec in enumerate(specs):
        W = fbq_synth.make_weight(spec, config, li)
        A, B = fbq_synth.make_branch(spec, config, li)
        d = fbq.Desc(spec.N, spec.K, spec.r, spec.bits, spec.group)
        Atd = t16(A.T) if spec.r else None
        Btd = t16(B.T) if spec.r else None
        Wd = t16(W)
        layers.append(fbq.quantize_feedback(d, Wd, Atd, Btd))
        torch.cuda.synchronize()
        del Wd
        xs.append(t16(fbq_synth.make_x(spec, M, config, li)))
    return layers, xs


def clone_layer(layer, fbq):
    c = lambda t: None if t is None else t.clone()
    return fbq.DeviceLayer(layer.desc, c(layer.qweight), c(layer.scales), c(layer.zeros), c(layer.At), c(layer.Bt))


class GroupCall:
    """Pre-marshalled fbq_linear_group call (keeps Python off the critical path)."""

    def __init__(self, fbq, layers, xs, ys, wss, M, stream_ptr):
        self.fn = fbq.load().fbq_linear_group
        self.arr = fbq.make_group(layers, xs, ys, wss)
        self.args = (self.arr, len(layers), M, stream_ptr)

    def __call__(self):
        rc = self.fn(*self.args)
        if rc:
            raise RuntimeError(f"fbq_linear_group failed with status {rc}")


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
        if el >= seconds or reps >= 20000:
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
    if M > 16:
        print("bench.py: the default benchmark times the decode path (M <= 16)", file=sys.stderr)
        sys.exit(2)
    base_layers, xs = build_layer_set(specs, args.config, M, torch, fbq)
    # the layers of a stage read the same activations, as in a decoder (q/k/v: the normalised hidden state; gate/up alike)
    for grp in stages_of(specs):
        for i in grp[1:]:
            xs[i] = xs[grp[0]]
    nbytes = [fbq_synth.algorithmic_bytes(s.N, s.K, s.r, s.bits, M, s.group) for s in specs]
    nbytes_plain = [fbq_synth.algorithmic_bytes(s.N, s.K, 0, s.bits, M, s.group) for s in specs]
    set_bytes = sum(nbytes)
    copies = args.copies or max(2, int(np.ceil(2.2e9 / set_bytes)))
    sets = [base_layers] + [[clone_layer(l, fbq) for l in base_layers] for _ in range(copies - 1)]

    stream = torch.cuda.current_stream()
    sp = ctypes.c_void_p(stream.cuda_stream)
    ys = [torch.empty((M, s.N), dtype=torch.float16, device="cuda") for s in specs]
    wss = [torch.zeros(max(16, fbq.workspace_bytes(l.desc, M)), dtype=torch.uint8, device="cuda") for l in base_layers]

    def twin(l):     # branch-free twin (r = 0) of the same packed layer: the comparator of "branch overhead %"
        return fbq.DeviceLayer(fbq.Desc(l.desc.N, l.desc.K, 0, l.desc.bits, l.desc.group), l.qweight, l.scales, l.zeros,
                               None, None)

    def schedule(groups, plain=False):
        """One list of GroupCalls per copy of the layer set."""
        out = []
        for ls in sets:
            calls = []
            for grp in groups:
                lay = [twin(ls[i]) if plain else ls[i] for i in grp]
                calls.append(GroupCall(fbq, lay, [xs[i] for i in grp], [ys[i] for i in grp],
                                       [None if plain else wss[i] for i in grp], M, sp))
            out.append(calls)
        return out

    def timed(sched, n, warm):
        for s in range(warm):
            for call in sched[s % len(sched)]:
                call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)
        for s in range(n):
            for call in sched[(warm + s) % len(sched)]:
                call()
        e1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return e0.elapsed_time(e1) / n, wall / n * 1e3      # ms per step: device events, host wall clock

    def timed_graphs(sched, n, warm, steps_per_graph):
        """The same launches replayed from HIP graphs of steps_per_graph consecutive steps each."""
        graphs = []
        side = torch.cuda.Stream()
        gsp = ctypes.c_void_p(side.cuda_stream)
        for g0 in range(0, len(sched), steps_per_graph):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for calls in sched[g0:g0 + steps_per_graph]:
                    for call in calls:
                        rc = call.fn(call.arr, call.args[1], call.args[2], gsp)
                        if rc:
                            raise RuntimeError(f"fbq_linear_group failed with status {rc} during capture")
            graphs.append((g, len(sched[g0:g0 + steps_per_graph])))
        for i in range(max(1, warm // steps_per_graph)):
            graphs[i % len(graphs)][0].replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        done, i = 0, 0
        while done < n:
            g, k = graphs[i % len(graphs)]
            g.replay()
            done += k
            i += 1
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / done, done

    staged = stages_of(specs)
    per_layer = [[i] for i in range(len(specs))]
    merged = [list(range(len(specs)))]                       # the library splits it by kernel variant itself

    ms_staged, wall_staged = timed(schedule(staged), args.steps, args.warmup)
    ms_staged_plain, _ = timed(schedule(staged, plain=True), args.steps, args.warmup)
    ms_graph_all, graph_steps = timed_graphs(schedule(staged), args.steps, args.warmup, copies)
    ms_layer, _ = timed(schedule(per_layer), args.steps, args.warmup)
    ms_layer_plain, _ = timed(schedule(per_layer, plain=True), args.steps, args.warmup)
    ms_merged, _ = timed(schedule(merged), args.steps, args.warmup)
    ms_merged_plain, _ = timed(schedule(merged, plain=True), args.steps, args.warmup)

    # dominant kernel: the fused GEMV launch that serves the widest stage (most bytes per launch).
    # Its launches alone, back to back on the stream, bracketed by events: average duration per launch
    # (this includes the ~1.5 us the command processor needs between two dependent launches).
    dom = max(staged, key=lambda grp: sum(nbytes[i] for i in grp))
    dom_bytes = sum(nbytes[i] for i in dom)
    ms_dom, _ = timed(schedule([dom]), args.steps, args.warmup)
    dom_gbps = dom_bytes / (ms_dom * 1e-3) / 1e9

    # HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (config 1 only)
    traffic = None
    prof = os.path.join(ROOT, "profiles", "decode_gemv_llama7b_int4_m1.md")
    if args.config == 1 and M == 1 and os.path.exists(prof):
        for line in open(prof):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])

    n_layers = len(specs)
    gbps = set_bytes / (ms_staged * 1e-3) / 1e9
    floor = sum(2 * s.r * (s.K + s.N) for s in specs) / sum(nbytes_plain)
    mode = lambda ms, ms_plain, launches: {
        "launches_per_step": launches, "us_per_step": round(ms * 1e3, 3), "us_per_layer": round(ms * 1e3 / n_layers, 3),
        "GBps": round(set_bytes / ms / 1e6, 1), "frac_of_hbm_peak": round(set_bytes / ms / 1e6 / HBM_PEAK_GBS, 4),
        "us_per_layer_branch_free": round(ms_plain * 1e3 / n_layers, 3),
        "branch_overhead_pct": round((ms / ms_plain - 1) * 100, 2)}
    out = {
        "metric": "fused W4/W3+low-rank linear: effective HBM GB/s (us/layer and branch overhead % alongside)",
        "value": round(gbps, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_staged, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": f"int{specs[0].bits} codes, f16 in/out, f32 accumulate", "data": "synthetic",
        "config": {"workload": f"config {args.config}: " + ", ".join(sorted({f'{s.K}->{s.N}' for s in specs})) +
                   f"; {n_layers} layers/step, INT{specs[0].bits}, group 128, rank {specs[0].r}, M={M}",
                   "layers_per_step": n_layers, "bytes_per_step": set_bytes, "copies_rotated": copies,
                   "launch_schedule": "staged: " + " ".join("{" + ",".join(specs[i].name for i in g) + "}" for g in staged)},
        "us_per_layer": round(ms_staged * 1e3 / n_layers, 3),
        "branch_overhead_pct": round((ms_staged / ms_staged_plain - 1) * 100, 2),
        "branch_overhead_byte_floor_pct": round(floor * 100, 2),
        "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBS, 4),
        "wall_ms_per_step": round(wall_staged, 6),
        "schedules": {"staged": mode(ms_staged, ms_staged_plain, len(staged)),
                      "staged_graph_of_all_copies": {"us_per_step": round(ms_graph_all * 1e3, 3), "steps_timed": graph_steps,
                                                     "GBps": round(set_bytes / ms_graph_all / 1e6, 1)},
                      "per_layer": mode(ms_layer, ms_layer_plain, len(per_layer)),
                      "merged": mode(ms_merged, ms_merged_plain, 2)},
        "roofline": {"bound": "hbm", "kernel": ("fbq_gemv_kernel" if M <= 2 else "fbq_small_m_kernel") + ", the launch serving {" +
                     ",".join(specs[i].name for i in dom) + "}", "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(dom_gbps / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "avg_launch_us": round(ms_dom * 1e3, 3), "bytes_per_launch": dom_bytes},
    }
    if not args.no_other_kernels:
        # Context, not part of `value`: the other two kernel families on the widest layer shape of the set
        # (random packed words, same rotation protocol; see paper_2501_16385_amd/perf.py).
        from paper_2501_16385_amd import perf
        wide = max(specs, key=lambda s: s.N * s.K)
        fam = {}
        if len(staged) < len(specs):
            # the same staged layer set with 16 tokens: the layers of a stage share their activations, as in a decoder
            M16 = 16
            xs16 = {}
            for grp in staged:
                shared = torch.randn((M16, specs[grp[0]].K), device="cuda").half()
                for i in grp:
                    xs16[i] = shared
            ys16 = [torch.empty((M16, s.N), dtype=torch.float16, device="cuda") for s in specs]
            ws16 = [torch.zeros(max(16, fbq.workspace_bytes(l.desc, M16)), dtype=torch.uint8, device="cuda") for l in base_layers]
            sched16 = [[GroupCall(fbq, [ls[i] for i in grp], [xs16[i] for i in grp], [ys16[i] for i in grp],
                                  [ws16[i] for i in grp], M16, sp) for grp in staged] for ls in sets]
            ms16, _ = timed(sched16, max(50, args.steps // 4), max(5, args.warmup // 4))
            bytes16 = sum(fbq_synth.algorithmic_bytes(s.N, s.K, s.r, s.bits, M16, s.group) for s in specs)
            fam["few_token_M16_staged_layer_set"] = {"launches_per_step": len(staged), "us_per_step": round(ms16 * 1e3, 2),
                                                     "us_per_layer": round(ms16 * 1e3 / n_layers, 3),
                                                     "GBps": round(bytes16 / ms16 / 1e6, 1),
                                                     "frac_of_hbm_peak": round(bytes16 / ms16 / 1e6 / HBM_PEAK_GBS, 4)}
            del sched16
        del sets
        torch.cuda.empty_cache()
        for name, m in (("few_token_M16", 16), ("few_token_M4", 4), ("prefill_M1024", 1024)):
            t = perf.time_layer(wide.N, wide.K, wide.r, wide.bits, m, iters=200 if m <= 16 else 50, warmup=20)
            fam[name] = {"shape": f"{wide.K}->{wide.N}", "us": t["us"], "GBps": t["GBps"], "TFLOPps": t["TFLOPps"],
                         "frac_of_hbm_peak": round(t["GBps"] / HBM_PEAK_GBS, 4),
                         "frac_of_fp16_mfma_peak": round(t["TFLOPps"] / 2500.0, 4)}
        # layer-wise reconstruction (Alg. 1) on the 4096 x 4096 shape of the set, 2048 calibration tokens
        sq = min(specs, key=lambda s: s.N * s.K)
        fam["reconstruction_step"] = perf.time_train_step(sq.N, sq.K, sq.r, sq.bits, 2048, iters=20, warmup=3)
        out["other_kernel_families"] = fam
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(specs, args.config, M, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
