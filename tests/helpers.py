"""Shared test plumbing: build one layer on both sides from the same seeded tensors."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

import fbq_synth
from oracle import fbq_oracle as orc


@dataclass
class OracleLayer:
    spec: fbq_synth.LayerSpec
    W: np.ndarray
    A: Optional[np.ndarray]
    B: Optional[np.ndarray]
    codes: np.ndarray
    scales: np.ndarray
    zeros: np.ndarray
    words: np.ndarray


def make_oracle_layer(spec: fbq_synth.LayerSpec, config: int = 7, layer_index: int = 0) -> OracleLayer:
    """Seeded W, A, B; codes, scales, zeros from the oracle's feedback quantizer."""
    W = fbq_synth.make_weight(spec, config, layer_index)
    A, B = fbq_synth.make_branch(spec, config, layer_index)
    Aa, Bb = (A, B) if spec.r else (None, None)
    codes, s, z = orc.quantize(W, Aa, Bb, spec.bits, spec.group)
    return OracleLayer(spec, W, Aa, Bb, codes, s, z, orc.pack(codes, spec.bits))


def oracle_y(L: OracleLayer, x: np.ndarray) -> np.ndarray:
    return orc.linear(x, L.words, L.scales, L.zeros, L.A, L.B, L.spec.bits, L.spec.group)


def rel_l2(got: np.ndarray, want: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def to_device_layer(L: OracleLayer):
    """Through the product's own fbq_pack, then to the GPU."""
    import paper_2501_16385_amd as fbq
    d = fbq.Desc(L.spec.N, L.spec.K, L.spec.r, L.spec.bits, L.spec.group)
    return fbq.upload_layer(fbq.pack(d, L.codes, L.scales, L.zeros, L.A, L.B))


def framed_in_nan(t):
    """The same device tensor inside a larger buffer filled with an fp16 NaN pattern (0x7D7D), 16-byte aligned: whatever
    a kernel reads from beyond the tensor and lets into its arithmetic - even multiplied by zero - shows as a NaN."""
    import torch
    if t is None:
        return None
    flat = t.contiguous().view(torch.uint8).reshape(-1)
    pad = 4096
    big = torch.full((flat.numel() + 2 * pad,), 0x7D, dtype=torch.uint8, device=t.device)
    big[pad:pad + flat.numel()] = flat
    return big[pad:pad + flat.numel()].view(t.dtype).view(t.shape)


def framed_layer(dev_layer):
    import paper_2501_16385_amd as fbq
    return fbq.DeviceLayer(dev_layer.desc, *(framed_in_nan(t) for t in (dev_layer.qweight, dev_layer.scales, dev_layer.zeros, dev_layer.At, dev_layer.Bt)))


GUARD = 256            # elements (y) / bytes (workspace) of sentinel on either side of a buffer the library writes
Y_SENTINEL = 0x7D7D    # an fp16 NaN: nothing the kernels compute, and visible if an output is never written
WS_SENTINEL = 0xA5


def gpu_y(dev_layer, x: np.ndarray) -> np.ndarray:
    """fbq_linear on x.  y and the workspace sit between guard bands filled with a sentinel: the call must leave the
    bands untouched, and must have overwritten every element of y."""
    import torch
    import paper_2501_16385_amd as fbq
    M, N = int(x.shape[0]), dev_layer.desc.N
    xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
    y_all = torch.full((M * N + 2 * GUARD,), Y_SENTINEL, dtype=torch.int16, device="cuda")
    y = y_all[GUARD:GUARD + M * N].view(M, N).view(torch.float16)
    need = fbq.workspace_bytes(dev_layer.desc, M)
    ws_all = torch.full((need + 2 * GUARD,), WS_SENTINEL, dtype=torch.uint8, device="cuda")
    ws = ws_all[GUARD:GUARD + need]
    ws.zero_()
    fbq.linear(dev_layer, xd, y=y, workspace=ws if need else None)
    torch.cuda.synchronize()
    y_host = y_all.cpu().numpy()
    assert np.all(y_host[:GUARD] == Y_SENTINEL) and np.all(y_host[GUARD + M * N:] == Y_SENTINEL), "y written out of bounds"
    ws_host = ws_all.cpu().numpy()
    assert np.all(ws_host[:GUARD] == WS_SENTINEL) and np.all(ws_host[GUARD + need:] == WS_SENTINEL), "workspace written out of bounds"
    got = y_host[GUARD:GUARD + M * N].view(np.float16).reshape(M, N).copy()
    assert not np.any(got.view(np.uint16) == Y_SENTINEL), "an element of y was never written"
    return got


# Element-wise bound beside the relative L2 norms (a single wrong output hardly moves a layer's norm).  Every path
# rounds y once to fp16 (half an ulp: 2^-11 |y|; 2^-10 |y| leaves room for a value next to a binade edge).  On top of
# that, relative to the rms of the outputs compared, by kernel family (chosen by the token count, as the dispatch does):
#   gemv    (1-2 tokens)   fp32 accumulation of exact products only: about 1e-6 sqrt(K)
#   few     (3-64 tokens)  the matrix cores sum q.x' on top of the offset 1024 sum(x') per group, about 40 times the
#                          signal, in fp32, and the offset is subtracted afterwards: about 5e-5 rms(y) per output
#   prefill (> 64 tokens)  every de-quantized weight is rounded to fp16 (2^-11 relative, independent): about 3e-4 rms(y)
# The slack is about ten standard deviations of that noise; a dropped or doubled term of the sum is 1e-2 rms(y) or more.
ELEMENT_SLACK = {"gemv": 2e-4, "few": 1e-3, "prefill": 3e-3}


def family_of(tokens: int) -> str:
    return "gemv" if tokens <= 2 else "few" if tokens <= 64 else "prefill"


def assert_matches_oracle(got: np.ndarray, want: np.ndarray, what: str, family: str = "", tol: float = 1e-3) -> None:
    """got, want [M, n]: relative L2 over all outputs and per token within tol (1e-3), and every single output within
    2^-10 |y| + ELEMENT_SLACK[family] * rms(y of its token); the family follows from the token count M unless named."""
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == want.shape, what
    slack = ELEMENT_SLACK[family if family in ELEMENT_SLACK else family_of(want.shape[0])]
    err = rel_l2(got, want)
    assert err <= tol, f"{what}: rel L2 {err:.3e}"
    for m in range(want.shape[0]):
        e = rel_l2(got[m], want[m])
        assert e <= tol, f"{what}, token {m}: rel L2 {e:.3e}"
        rms = float(np.sqrt(np.mean(want[m] ** 2)))
        bound = 2.0 ** -10 * np.abs(want[m]) + slack * rms
        worst = np.max(np.abs(got[m] - want[m]) - bound)
        assert worst <= 0, f"{what}, token {m}: an output is {worst:.3e} beyond its element-wise bound"
