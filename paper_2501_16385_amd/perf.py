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

import torch

from . import fbq


def algorithmic_bytes(N, K, r, bits, M):
    return N * K * bits // 8 + 4 * N * (K // 128) + 2 * r * (K + N) + 2 * M * (K + N)


def algorithmic_flops(N, K, r, M):
    return 2 * M * N * K + 2 * M * r * (K + N)


def random_layer(d: fbq.Desc, gen, gain=None) -> fbq.DeviceLayer:
    """Uniformly random codes; gain: if given, scales are chosen so that |y| is about gain * |x| for random x."""
    words = fbq.packed_bytes(d) // 4 // d.N
    qmax = 2**d.bits - 1
    qw = torch.randint(-2**31, 2**31 - 1, (d.N, words), dtype=torch.int32, device="cuda", generator=gen)
    s = torch.rand(d.N, d.K // 128, device="cuda", generator=gen) * 0.01 + 0.001
    if gain is not None:                  # codes uniform on 0..qmax around a zero point near the middle: std (qmax + 1) / sqrt(12)
        s = s * (gain / (0.006 * (qmax + 1) / 12 ** 0.5 * d.K ** 0.5))
    s = s.half().view(torch.int16)
    z = (torch.rand(d.N, d.K // 128, device="cuda", generator=gen) + 0.5 * (qmax - 1)).half().view(torch.int16)
    At = Bt = None
    if d.r:
        At = (torch.randn(d.r, d.K, device="cuda", generator=gen) * 0.01).half().view(torch.int16)
        Bt = (torch.randn(d.N, d.r, device="cuda", generator=gen) * 0.01).half().view(torch.int16)
    return fbq.DeviceLayer(d, qw, s, z, At, Bt)


def time_layer(N, K, r, bits, M, iters=100, warmup=10, rotate_bytes=1.0e9):
    lib = fbq.load()
    d = fbq.Desc(N, K, r, bits)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    copies = max(2, int(rotate_bytes // fbq.packed_bytes(d)))
    layers = [random_layer(d, gen) for _ in range(copies)]
    x = torch.randn(M, K, device="cuda", generator=gen).half()
    y = torch.empty(M, N, dtype=torch.float16, device="cuda")
    ws = torch.zeros(max(16, fbq.workspace_bytes(d, M)), dtype=torch.uint8, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ptr = lambda t: ctypes.c_void_p(0 if t is None else t.data_ptr())
    descs = [l.desc.c() for l in layers]
    calls = [(ctypes.byref(descs[i]), M, ptr(x), ptr(l.qweight), ptr(l.scales), ptr(l.zeros), ptr(l.At), ptr(l.Bt),
              ptr(y), ptr(ws), ctypes.c_size_t(ws.numel()), stream) for i, l in enumerate(layers)]

    def run(n):
        for i in range(n):
            rc = lib.fbq_linear(*calls[i % copies])
            if rc != 0:
                raise RuntimeError(f"fbq_linear: {fbq.status_string(rc)}")

    run(warmup)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    run(iters)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) / iters * 1e3
    return {"N": N, "K": K, "r": r, "bits": bits, "M": M, "us": round(us, 2),
            "GBps": round(algorithmic_bytes(N, K, r, bits, M) / us / 1e3, 1),
            "TFLOPps": round(algorithmic_flops(N, K, r, M) / us / 1e6, 2), "copies": copies, "iters": iters}


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
    ap.add_argument("--N", type=int, required=True)
    ap.add_argument("--K", type=int, required=True)
    ap.add_argument("--r", type=int, default=0)
    ap.add_argument("--bits", type=int, default=4)
    ap.add_argument("--M", type=int, default=1)
    ap.add_argument("--iters", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--train-tokens", type=int, default=0, help="time the reconstruction step on this many calibration tokens instead")
    a = ap.parse_args()
    if a.train_tokens:
        print(json.dumps(time_train_step(a.N, a.K, a.r, a.bits, a.train_tokens, a.iters, a.warmup)), flush=True)
        return
    print(json.dumps(time_layer(a.N, a.K, a.r, a.bits, a.M, a.iters, a.warmup)), flush=True)


if __name__ == "__main__":
    main()
