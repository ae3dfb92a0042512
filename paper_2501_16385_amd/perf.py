"""Times fbq_linear on one layer shape: `python -m paper_2501_16385_amd.perf --N 11008 --K 4096 --r 64 --bits 4 --M 16`.

Random packed words, scales, zeros and sub-branch stand in for a quantized layer (the kernels' time
does not depend on the values).  Enough distinct copies of the layer rotate that no cache holds the
weights.  Prints one JSON line: microseconds per call, effective GB/s over the algorithmic bytes and
TFLOP/s over the algorithmic flops (packed codes, scale/zero, A, B, x and y once; 2MNK + 2Mr(K+N)).
"""
from __future__ import annotations

import argparse
import ctypes
import json

import os
import sys

import torch

from . import fbq
from .random_layers import branch_free_twin, random_layer

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import fbq_synth  # noqa: E402  (byte and flop accounting: the one copy, pinned by the tests against the paper's MAC ratio)


kHostBoundUs = 9.0     # below this a Python loop of ctypes calls may not keep the stream fed: such launches are also timed from a HIP graph


def event_stats(run, iters, warmup, repeats=5):
    """run(n) enqueues n calls on the current stream.  Times `repeats` batches of `iters` calls each with HIP
    events; returns microseconds per call: mean over all batches, median and minimum over the batches."""
    run(warmup)
    torch.cuda.synchronize()
    per_call = []
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run(iters)
        e1.record()
        torch.cuda.synchronize()
        per_call.append(e0.elapsed_time(e1) / iters * 1e3)
    per_call.sort()
    return {"us_mean": round(sum(per_call) / len(per_call), 3), "us_median": round(per_call[len(per_call) // 2], 3),
            "us_min": round(per_call[0], 3), "batches": repeats, "calls_per_batch": iters}


def time_layer(N, K, r, bits, M, iters=100, warmup=10, rotate_bytes=1.0e9, repeats=3, with_twin=False, graph=False):
    """One layer shape, isolated: the same call back to back on the stream, every call on another copy of the
    packed layer.  with_twin also times the branch-free twin (r = 0) on the same packed weights.  graph: the calls
    are replayed from one HIP graph over all copies (for launches shorter than the host needs to enqueue one);
    "auto": eager first, and where that comes out below kHostBoundUs the graph as well, the faster of the two counts."""
    lib = fbq.load()
    d = fbq.Desc(N, K, r, bits)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    copies = max(2, int(rotate_bytes // fbq.packed_bytes(d)))
    layers = [random_layer(d, gen) for _ in range(copies)]
    x = torch.randn(M, K, device="cuda", generator=gen).half()
    y = torch.empty(M, N, dtype=torch.float16, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ptr = lambda t: ctypes.c_void_p(0 if t is None else t.data_ptr())

    def timed(ls):
        dd = ls[0].desc
        ws = torch.zeros(max(16, fbq.workspace_bytes(dd, M)), dtype=torch.uint8, device="cuda")
        descs = [l.desc.c() for l in ls]
        calls = [(ctypes.byref(descs[i]), M, ptr(x), ptr(l.qweight), ptr(l.scales), ptr(l.zeros), ptr(l.At), ptr(l.Bt),
                  ptr(y), ptr(ws), ctypes.c_size_t(ws.numel()), stream) for i, l in enumerate(ls)]

        def run(n):
            for i in range(n):
                rc = lib.fbq_linear(*calls[i % copies])
                if rc != 0:
                    raise RuntimeError(f"fbq_linear: {fbq.status_string(rc)}")
        eager = None
        if graph != True:
            eager = event_stats(run, iters, warmup, repeats)
            if not graph or eager["us_median"] > kHostBoundUs:
                return eager
        # one HIP graph holding a call on every copy: the host enqueues one graph instead of a call every few microseconds
        side = torch.cuda.Stream()
        gstream = ctypes.c_void_p(side.cuda_stream)
        run(2)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for c in calls:
                rc = lib.fbq_linear(*(c[:-1] + (gstream,)))
                if rc != 0:
                    raise RuntimeError(f"fbq_linear: {fbq.status_string(rc)} during capture")
        replays = max(1, -(-iters // copies))
        st = event_stats(lambda n: [g.replay() for _ in range(n)], replays, max(1, warmup // copies), repeats)
        for k in ("us_mean", "us_median", "us_min"):
            st[k] = round(st[k] / copies, 3)
        return st if eager is None or st["us_median"] < eager["us_median"] else eager

    st = timed(layers)
    us = st["us_median"]
    out = {"N": N, "K": K, "r": r, "bits": bits, "M": M, "us": us, "us_min": st["us_min"], "us_mean": st["us_mean"],
           "GBps": round(fbq_synth.algorithmic_bytes(N, K, r, bits, M) / us / 1e3, 1),
           "TFLOPps": round(fbq_synth.algorithmic_flops(N, K, r, M) / us / 1e6, 2), "copies": copies, "iters": iters,
           "batches": repeats}
    if with_twin and r:
        tw = timed([branch_free_twin(l) for l in layers])
        out["us_branch_free"] = tw["us_median"]
        out["branch_overhead_pct"] = round((us / tw["us_median"] - 1) * 100, 2)
    return out


def time_group(shapes, r, bits, M, iters=100, warmup=10, rotate_bytes=1.0e9, repeats=3):
    """Several layers (N, K) that read the same activations, served by one fbq_linear_group call (q/k/v, gate/up):
    the call back to back on the stream, every call on another copy of the packed layers."""
    lib = fbq.load()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    descs = [fbq.Desc(N, K, r, bits) for (N, K) in shapes]
    set_bytes = sum(fbq.packed_bytes(d) for d in descs)
    copies = max(2, int(rotate_bytes // set_bytes))
    sets = [[random_layer(d, gen) for d in descs] for _ in range(copies)]
    xs = {}
    for (N, K) in shapes:
        if K not in xs:
            xs[K] = torch.randn(M, K, device="cuda", generator=gen).half()
    ys = [torch.empty(M, N, dtype=torch.float16, device="cuda") for (N, K) in shapes]
    wss = [torch.zeros(max(16, fbq.workspace_bytes(d, M)), dtype=torch.uint8, device="cuda") for d in descs]
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    arrs = [fbq.make_group(ls, [xs[K] for (_, K) in shapes], ys, wss) for ls in sets]

    def run(n):
        for i in range(n):
            rc = lib.fbq_linear_group(arrs[i % copies], len(shapes), M, stream)
            if rc != 0:
                raise RuntimeError(f"fbq_linear_group: {fbq.status_string(rc)}")
    st = event_stats(run, iters, warmup, repeats)
    nbytes = sum(fbq_synth.algorithmic_bytes(N, K, r, bits, M) for (N, K) in shapes)
    return {"layers": [f"{K}->{N}" for (N, K) in shapes], "r": r, "bits": bits, "M": M, "us": st["us_median"], "us_min": st["us_min"],
            "bytes": nbytes, "GBps": round(nbytes / st["us_median"] / 1e3, 1), "copies": copies, "iters": iters}


def time_read_stream(nbytes, iters=200, warmup=20, pool_bytes=3 << 30, repeats=3):
    """The read-only yardstick kernel on launches of nbytes each, back to back, every launch on another part of
    a pool no cache holds.  Returns microseconds per launch (median of the batches) and GB/s."""
    lib = fbq.load()
    nbytes = (int(nbytes) + 4095) // 4096 * 4096
    pool = _read_pool(max(pool_bytes, 2 * nbytes))
    copies = pool.numel() // nbytes
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    base = pool.data_ptr()

    def run(n):
        for i in range(n):
            rc = lib.fbq_measure_read_stream(ctypes.c_void_p(base + (i % copies) * nbytes), ctypes.c_size_t(nbytes), stream)
            if rc != 0:
                raise RuntimeError(f"fbq_measure_read_stream: {fbq.status_string(rc)}")
    st = event_stats(run, iters, warmup, repeats)
    return {"bytes": nbytes, "us": st["us_median"], "us_min": st["us_min"], "GBps": round(nbytes / st["us_median"] / 1e3, 1)}


_POOL = None


def _read_pool(nbytes):
    global _POOL
    if _POOL is None or _POOL.numel() < nbytes:
        _POOL = None
        _POOL = torch.empty(int(nbytes), dtype=torch.uint8, device="cuda")
        _POOL.view(torch.int32).random_()
    return _POOL


def free_read_pool():
    global _POOL
    _POOL = None


def time_train_step(N, K, r, bits, T, iters=20, warmup=3):
    """Times fbq_gram and fbq_train_step (with and without the loss) on synthetic W ~ N(0, 0.02), X ~ N(0, 1).
    Flops: gram 2 K^2 T; gradients 8 N K r + 4 r K^2 (products with r rows only); the loss 2 N K^2 more."""
    d = fbq.Desc(N, K, r, bits)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    W = (torch.randn(N, K, device="cuda", generator=gen) * 0.02).half()
    X = torch.randn(T, K, device="cuda", generator=gen).half()
    At32 = torch.randn(r, K, device="cuda", generator=gen) * 0.01
    Bt32 = torch.randn(N, r, device="cuda", generator=gen) * 0.01
    st = fbq.train_state(d, At32, Bt32)
    ws = torch.empty(fbq.train_workspace_bytes(d, T), dtype=torch.uint8, device="cuda")
    hs = 1.0 / T
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn):
        for _ in range(warmup):
            fn()
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e3

    H16 = fbq.gram(d, X, hs, ws)
    us_gram = timed(lambda: fbq.gram(d, X, hs, ws))
    lr = 0.0        # the masters stay put: every timed iteration does the same work on the same values
    us_loss = timed(lambda: fbq.train_step(st, W, H16, hs, lr))
    us_grad = timed(lambda: fbq.train_step(st, W, H16, hs, lr, want_loss=False))
    fl_grad = 8.0 * N * K * r + 4.0 * r * K * K
    fl_loss = 2.0 * N * K * K
    return {"N": N, "K": K, "r": r, "bits": bits, "T": T, "gram_us": round(us_gram, 1),
            "gram_TFLOPps": round(2.0 * K * K * T / us_gram / 1e6, 1),
            "step_us": round(us_grad, 1), "step_with_loss_us": round(us_loss, 1),
            "loss_contraction_TFLOPps": round(fl_loss / max(us_loss - us_grad, 1e-3) / 1e6, 1),
            "step_TFLOPps": round(fl_grad / us_grad / 1e6, 1), "loss": float(st.loss.cpu()[0])}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--N", type=int, default=4096)
    ap.add_argument("--K", type=int, default=4096)
    ap.add_argument("--r", type=int, default=0)
    ap.add_argument("--bits", type=int, default=4)
    ap.add_argument("--M", type=int, default=1)
    ap.add_argument("--iters", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--train-tokens", type=int, default=0, help="time the reconstruction step on this many calibration tokens instead")
    ap.add_argument("--rotate-bytes", type=float, default=1.0e9, help="distinct copies of the layer rotate over at least this many bytes")
    ap.add_argument("--group", type=str, default="", help="several layers in one fbq_linear_group call, as NxK,NxK,... (they share x where K is equal)")
    ap.add_argument("--graph", action="store_true", help="replay the calls from one HIP graph over all copies")
    ap.add_argument("--twin", action="store_true", help="also time the branch-free twin (r = 0) on the same packed weights")
    ap.add_argument("--read-bytes", type=float, default=0, help="time the read-only yardstick kernel on launches of this many bytes instead")
    a = ap.parse_args()
    if a.train_tokens:
        print(json.dumps(time_train_step(a.N, a.K, a.r, a.bits, a.train_tokens, a.iters, a.warmup)), flush=True)
        return
    if a.group:
        shapes = [tuple(int(v) for v in item.split("x")) for item in a.group.split(",")]
        print(json.dumps(time_group(shapes, a.r, a.bits, a.M, a.iters, a.warmup, a.rotate_bytes)), flush=True)
        return
    if a.read_bytes:
        print(json.dumps(time_read_stream(a.read_bytes, a.iters, a.warmup)), flush=True)
        return
    print(json.dumps(time_layer(a.N, a.K, a.r, a.bits, a.M, a.iters, a.warmup, rotate_bytes=a.rotate_bytes, with_twin=a.twin, graph=a.graph)), flush=True)


if __name__ == "__main__":
    main()
