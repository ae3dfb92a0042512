"""Layer-wise reconstruction of one layer (Alg. 1, Sec. 4.2) as a loop over fbq_train_step.

    python -m paper_2501_16385_amd.reconstruction --N 4096 --K 4096 --r 64 --bits 4 --tokens 2048 --steps 50

Synthetic W ~ N(0, 0.02) with 1 % outliers x10 and X ~ N(0, 1) stand in for a checkpoint and its
calibration activations.  A starts as N(0, sigma^2), B as zeros (Alg. 1, initialisation); every
iteration quantizes with feedback, evaluates the loss, and moves A and B down the detached gradient.
Prints one JSON line: the loss before the first and after the last iteration, and the time per
iteration.  Everything on the GPU runs in the library's kernels; torch holds the buffers.
"""
from __future__ import annotations

import argparse
import json

import torch

from . import fbq


def reconstruct_layer(d: fbq.Desc, W, X, steps: int, lr: float, a_std: float = 0.01, seed: int = 0, h_scale=None,
                      loss_every: int = 1):
    """Runs `steps` iterations of Alg. 1 on W [N,K] fp16 with calibration activations X [T,K] fp16.

    Returns (layer, losses): the DeviceLayer the last call wrote (codes, scales, zeros and fp16 branch of
    the final masters, ready for fbq.linear) and the list of (iteration, loss) pairs that were evaluated.
    lr is the plain gradient-descent step; it has to stay below 1 / (lambda_max(X^T X) * max(|A|_2^2, |B|_2^2)) for
    the norms A and B reach on the way, not only for the initial ones.
    """
    T = int(X.shape[0])
    hs = 1.0 / T if h_scale is None else float(h_scale)
    gen = torch.Generator(device=W.device)
    gen.manual_seed(seed)
    At32 = torch.randn(d.r, d.K, device=W.device, generator=gen) * a_std
    Bt32 = torch.zeros(d.N, d.r, device=W.device)
    st = fbq.train_state(d, At32, Bt32)
    ws = torch.empty(max(256, fbq.train_workspace_bytes(d, T)), dtype=torch.uint8, device=W.device)
    H16 = fbq.gram(d, X, hs, ws)
    losses = []
    for it in range(steps):
        want = loss_every > 0 and it % loss_every == 0
        fbq.train_step(st, W, H16, hs, lr, want_loss=want)
        if want:
            losses.append((it, st.loss.clone()))
    fbq.train_step(st, W, H16, hs, 0.0)          # lr = 0: the layer and the loss of the final masters
    losses.append((steps, st.loss.clone()))
    return st.layer, [(i, float(l.cpu()[0])) for i, l in losses]


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--N", type=int, default=4096)
    ap.add_argument("--K", type=int, default=4096)
    ap.add_argument("--r", type=int, default=64)
    ap.add_argument("--bits", type=int, default=4)
    ap.add_argument("--tokens", type=int, default=2048)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--lr", type=float, default=0.0, help="0: 0.05 / (lambda_max(X^T X) * |A|_2^2), by power iteration")
    a = ap.parse_args()
    d = fbq.Desc(a.N, a.K, a.r, a.bits)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    W = torch.randn(a.N, a.K, device="cuda", generator=gen) * 0.02
    W = (W * torch.where(torch.rand(a.N, a.K, device="cuda", generator=gen) < 0.01, 10.0, 1.0)).half()
    X = torch.randn(a.tokens, a.K, device="cuda", generator=gen).half()
    lr = a.lr
    if lr == 0.0:
        v = torch.randn(a.K, device="cuda", generator=gen)
        Xf = X.float()
        for _ in range(30):
            v = Xf.T @ (Xf @ v)
            v = v / v.norm()
        lam = float((Xf @ v).norm() ** 2)
        lr = 0.05 / (lam * (0.01 ** 2) * (a.K ** 0.5 + a.r ** 0.5) ** 2)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    layer, losses = reconstruct_layer(d, W, X, a.steps, lr)
    e1.record()
    torch.cuda.synchronize()
    print(json.dumps({"N": a.N, "K": a.K, "r": a.r, "bits": a.bits, "tokens": a.tokens, "steps": a.steps, "lr": lr,
                      "loss_first": losses[0][1], "loss_last": losses[-1][1],
                      "ms_per_step_with_loss": round(e0.elapsed_time(e1) / (a.steps + 1), 3)}), flush=True)


if __name__ == "__main__":
    main()
