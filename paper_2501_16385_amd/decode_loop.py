"""Token-by-token decode over a stack of decoder layers whose seven linear layers (q, k, v, o, gate, up,
down) are fused sub-branched quantized linears, replayed from one HIP graph per token.

    python -m paper_2501_16385_amd.decode_loop --layers 32 --hidden 4096 --inter 11008 --r 128 --bits 4

The paper reports whole-model decode speed for this configuration (Sec. 5.3: batch 1, rank 128);
--batch B decodes B independent sequences per step (B rows through every linear: from three rows on
the matrix-core kernel streams the weights once for all of them).  Only
the linear layers are the paper's method, so only they are real here; the glue between them is the
least that keeps the data flow of a decoder layer and the values bounded:

    q, k, v = x Wq, x Wk, x Wv        one grouped launch (they share x)
    a       = v                        attention over a single position returns v; q and k are computed and dropped
    h       = (x + a Wo) / 2           residual, halved instead of normalised (no reduction kernels in the graph)
    g, u    = h Wg, h Wu               one grouped launch
    x'      = (h + (silu(g) * u) Wd) / 2

Four fused launches and four element-wise kernels (two lerp, silu, mul) per layer.  Weights are random packed words (speed
does not depend on the values) unless a list of quantized layers is passed in.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys

import torch

from . import fbq
from .random_layers import random_layer

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import fbq_synth  # noqa: E402  (byte accounting)

NAMES = ("q", "k", "v", "o", "gate", "up", "down")


def layer_shapes(hidden: int, inter: int):
    """(N, K) of the seven linears of one decoder layer."""
    return {"q": (hidden, hidden), "k": (hidden, hidden), "v": (hidden, hidden), "o": (hidden, hidden),
            "gate": (inter, hidden), "up": (inter, hidden), "down": (hidden, inter)}


class DecoderStack:
    """layers: list (one per decoder layer) of dicts name -> fbq.DeviceLayer."""

    def __init__(self, layers, hidden: int, inter: int, keep_per_layer_buffers: bool = False, batch: int = 1,
                 share_workspaces: bool = False):
        self.layers, self.hidden, self.inter, self.batch = layers, hidden, inter, batch
        self.lib = fbq.load()
        dev = "cuda"
        f16 = lambda n: torch.zeros((batch, n), dtype=torch.float16, device=dev)
        self.x = f16(hidden)
        n_buf = len(layers) if keep_per_layer_buffers else 1
        self.buf = [{"q": f16(hidden), "k": f16(hidden), "v": f16(hidden), "o": f16(hidden), "h": f16(hidden),
                     "gate": f16(inter), "up": f16(inter), "act": f16(inter), "down": f16(hidden), "x_in": f16(hidden)}
                    for _ in range(n_buf)]
        # one zero-filled workspace per linear: launches of one token never share one.  A prompt pass of hundreds of rows
        # needs megabytes per linear (the re-ordered activations): its layers, which run one after the other, share a set.
        if share_workspaces:
            one = {n: self._workspace(layers[0][n].desc) for n in NAMES}
            self.ws = [one for _ in layers]
        else:
            self.ws = [{n: self._workspace(l[n].desc) for n in NAMES} for l in layers]
        self.graph = None

    def _workspace(self, desc):
        need = fbq.workspace_bytes(desc, self.batch)
        return torch.zeros(need, dtype=torch.uint8, device="cuda") if need else None

    def _group(self, li, names, xs, ys, stream_ptr):
        l, ws = self.layers[li], self.ws[li]
        arr = fbq.make_group([l[n] for n in names], xs, ys, [ws[n] for n in names])
        rc = self.lib.fbq_linear_group(arr, len(names), self.batch, stream_ptr)
        if rc:
            raise RuntimeError(f"fbq_linear_group: {fbq.status_string(rc)}")

    def step(self, stream=None):
        """One token through all layers: reads and overwrites self.x."""
        stream = stream or torch.cuda.current_stream()
        sp = ctypes.c_void_p(stream.cuda_stream)
        x = self.x
        for li in range(len(self.layers)):
            b = self.buf[li % len(self.buf)]
            if len(self.buf) > 1:
                b["x_in"].copy_(x)                      # kept for inspection only
            self._group(li, ("q", "k", "v"), [x, x, x], [b["q"], b["k"], b["v"]], sp)
            self._group(li, ("o",), [b["v"]], [b["o"]], sp)
            torch.lerp(x, b["o"], 0.5, out=b["h"])      # (x + o) / 2
            self._group(li, ("gate", "up"), [b["h"], b["h"]], [b["gate"], b["up"]], sp)
            torch.mul(torch.nn.functional.silu(b["gate"]), b["up"], out=b["act"])
            self._group(li, ("down",), [b["act"]], [b["down"]], sp)
            torch.lerp(b["h"], b["down"], 0.5, out=x)   # (h + down) / 2
        return x

    def capture(self):
        """Records step() into a HIP graph (after one eager step on a side stream, as capture requires)."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.step(side)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph, stream=side):
            self.step(side)
        return self.graph


def random_stack(n_layers, hidden, inter, r, bits, seed=1):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    shapes = layer_shapes(hidden, inter)
    return [{n: random_layer(fbq.Desc(shapes[n][0], shapes[n][1], r, bits), gen, gain=0.5) for n in NAMES} for _ in range(n_layers)]


def prompt_then_decode(layers, hidden, inter, prompt=256, new_tokens=64, warmup=2):
    """The shape of the paper's end-to-end measurement (Sec. 5.3: batch 1, a prompt of 256 tokens, then 64 generated):
    one pass of `prompt` rows through the stack (the prefill GEMM in every linear), then `new_tokens` single-row steps
    replayed from a HIP graph.  Returns milliseconds for each leg and tokens per second over the whole run."""
    pre = DecoderStack(layers, hidden, inter, batch=prompt, share_workspaces=True)
    dec = DecoderStack(layers, hidden, inter, batch=1)
    pre.x.copy_(torch.randn(prompt, hidden, device="cuda").half())
    dec.x.copy_(torch.randn(1, hidden, device="cuda").half())
    g = dec.capture()
    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    best = None
    for it in range(warmup + 3):
        torch.cuda.synchronize()
        e[0].record()
        pre.step()
        e[1].record()
        for _ in range(new_tokens):
            g.replay()
        e[2].record()
        torch.cuda.synchronize()
        t = (e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2]))
        if it >= warmup and (best is None or sum(t) < sum(best)):
            best = t
    total_s = sum(best) * 1e-3
    return {"prompt_tokens": prompt, "generated_tokens": new_tokens, "prompt_ms": round(best[0], 3),
            "decode_ms_per_token": round(best[1] / new_tokens, 4), "total_ms": round(sum(best), 3),
            "generated_tokens_per_s": round(new_tokens / total_s, 1),
            "all_tokens_per_s": round((prompt + new_tokens) / total_s, 1),
            "finite": bool(torch.isfinite(pre.x).all() and torch.isfinite(dec.x).all())}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--hidden", type=int, default=4096)
    ap.add_argument("--inter", type=int, default=11008)
    ap.add_argument("--r", type=int, default=128)
    ap.add_argument("--bits", type=int, default=4)
    ap.add_argument("--tokens", type=int, default=64, help="decode steps to time")
    ap.add_argument("--batch", type=int, default=1, help="sequences decoded together (rows per step)")
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--prompt", type=int, default=0, help="run a prompt pass of this many tokens first and report the whole run (Sec. 5.3: 256)")
    a = ap.parse_args()
    if a.prompt:
        out = prompt_then_decode(random_stack(a.layers, a.hidden, a.inter, a.r, a.bits), a.hidden, a.inter, a.prompt, a.tokens)
        out.update({"layers": a.layers, "bits": a.bits, "r": a.r, "hidden": a.hidden, "inter": a.inter})
        print(json.dumps(out), flush=True)
        return
    stack = DecoderStack(random_stack(a.layers, a.hidden, a.inter, a.r, a.bits), a.hidden, a.inter, batch=a.batch)
    stack.x.copy_(torch.randn(a.batch, a.hidden, device="cuda").half())
    g = stack.capture()
    for _ in range(a.warmup):
        g.replay()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(a.tokens):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) / a.tokens * 1e3
    shapes = layer_shapes(a.hidden, a.inter)
    nbytes = a.layers * sum(fbq_synth.algorithmic_bytes(N, K, a.r, a.bits, a.batch) for N, K in shapes.values())
    print(json.dumps({"tokens_per_s": round(a.batch * 1e6 / us, 1), "us_per_step": round(us, 1), "batch": a.batch, "layers": a.layers,
                      "fused_launches_per_step": 4 * a.layers, "GBps_over_linear_layers": round(nbytes / us / 1e3, 1),
                      "bits": a.bits, "r": a.r, "hidden": a.hidden, "inter": a.inter, "tokens_timed": a.tokens,
                      "finite": bool(torch.isfinite(stack.x).all())}), flush=True)


if __name__ == "__main__":
    main()
