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


def gpu_y(dev_layer, x: np.ndarray) -> np.ndarray:
    import torch
    import paper_2501_16385_amd as fbq
    xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
    y = fbq.linear(dev_layer, xd)
    torch.cuda.synchronize()
    return y.cpu().numpy()
