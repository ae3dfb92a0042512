"""Seeded synthetic inputs for the sub-branched quantized linear layer.

This module only draws random numbers and names shapes.  It contains none of
the method's arithmetic (no quantizer, no packing, no matmul): the CPU oracle
and the HIP library are both fed from here and share nothing else.

The tensors stand in for the Llama2-7B / 13B / 70B-shaped linear layers the
paper measures on (Sec. 3.2, Sec. 5.1 "Implementation Details"): the paper's
checkpoints and trained sub-branches are not available, and the kernel's cost
depends on shapes only.

Value recipe (all tensors are rounded once to fp16 and handed over as fp16):
  W  [N, K]  ~ N(0, w_std^2), and an independent Bernoulli(outlier_p) mask
             multiplies the selected entries by outlier_mul (default 1 % x10)
  A  [K, r]  ~ N(0, ab_std^2)      (down-projection, y = x.A.B convention)
  B  [r, N]  ~ N(0, ab_std^2)      (up-projection)
  x  [M, K]  ~ N(0, 1)
Seeds: base 20250116 + 1000*config + 10*layer_index + tensor_index
(tensor_index: W 0, A 1, B 2, x 3, outlier mask 4), each tensor from its own
Philox stream so that one tensor can be regenerated without the others.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

SEED_BASE = 20250116
GROUP = 128


@dataclass(frozen=True)
class LayerSpec:
    """One linear layer K -> N with a rank-r sub-branch, quantized to `bits`."""
    name: str
    N: int
    K: int
    r: int
    bits: int
    group: int = GROUP
    w_std: float = 0.02
    ab_std: float = 0.01
    outlier_p: float = 0.01
    outlier_mul: float = 10.0


def _rng(config: int, layer_index: int, tensor_index: int) -> np.random.Generator:
    seed = SEED_BASE + 1000 * config + 10 * layer_index + tensor_index
    return np.random.Generator(np.random.Philox(seed))


def _normal_f16(rng: np.random.Generator, shape: Tuple[int, ...], std: float) -> np.ndarray:
    # draw in fp32 in row blocks to bound peak memory on the large layers
    out = np.empty(shape, dtype=np.float16)
    rows = shape[0]
    step = max(1, (1 << 22) // max(1, int(np.prod(shape[1:]))))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        blk = rng.standard_normal((r1 - r0,) + tuple(shape[1:]), dtype=np.float32)
        out[r0:r1] = (blk * np.float32(std)).astype(np.float16)
    return out


def make_weight(spec: LayerSpec, config: int, layer_index: int) -> np.ndarray:
    """W [N, K] fp16 with sparse x`outlier_mul` outliers."""
    rng_w = _rng(config, layer_index, 0)
    rng_m = _rng(config, layer_index, 4)
    out = np.empty((spec.N, spec.K), dtype=np.float16)
    step = max(1, (1 << 22) // spec.K)
    for r0 in range(0, spec.N, step):
        r1 = min(spec.N, r0 + step)
        blk = rng_w.standard_normal((r1 - r0, spec.K), dtype=np.float32) * np.float32(spec.w_std)
        mask = rng_m.random((r1 - r0, spec.K), dtype=np.float32) < np.float32(spec.outlier_p)
        blk[mask] *= np.float32(spec.outlier_mul)
        out[r0:r1] = blk.astype(np.float16)
    return out


def make_branch(spec: LayerSpec, config: int, layer_index: int) -> Tuple[np.ndarray, np.ndarray]:
    """A [K, r], B [r, N] fp16.  r == 0 gives empty arrays."""
    A = _normal_f16(_rng(config, layer_index, 1), (spec.K, spec.r), spec.ab_std) if spec.r else \
        np.zeros((spec.K, 0), np.float16)
    B = _normal_f16(_rng(config, layer_index, 2), (spec.r, spec.N), spec.ab_std) if spec.r else \
        np.zeros((0, spec.N), np.float16)
    return A, B


def make_x(spec: LayerSpec, M: int, config: int, layer_index: int) -> np.ndarray:
    """x [M, K] fp16 ~ N(0,1)."""
    return _normal_f16(_rng(config, layer_index, 3), (M, spec.K), 1.0)


def make_random_quantized(spec: LayerSpec, config: int, layer_index: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Stand-in for a quantized layer that is too large to push through the fp64 quantizer in a test:
    uniformly random codes [N, K] (uint8, 0 .. 2^bits - 1), fp16 scales in the range the quantizer
    produces for N(0, w_std^2) weights with outliers, fp16 zero points around the middle of the code
    range.  (The kernels' work does not depend on how the codes came about.)"""
    qmax = (1 << spec.bits) - 1
    rng_c, rng_s, rng_z = _rng(config, layer_index, 5), _rng(config, layer_index, 6), _rng(config, layer_index, 7)
    G = spec.K // spec.group
    codes = np.empty((spec.N, spec.K), dtype=np.uint8)
    step = max(1, (1 << 24) // spec.K)
    for r0 in range(0, spec.N, step):
        r1 = min(spec.N, r0 + step)
        codes[r0:r1] = rng_c.integers(0, qmax + 1, (r1 - r0, spec.K), dtype=np.uint8)
    span = np.float32(spec.w_std) * (5.0 + 25.0 * rng_s.random((spec.N, G), dtype=np.float32) ** 8)   # mostly ~5 sigma, some outlier groups
    scales = (span / np.float32(qmax)).astype(np.float16)
    zeros = (np.float32(0.5 * qmax) + (rng_z.random((spec.N, G), dtype=np.float32) - 0.5) * np.float32(0.5 * qmax)).astype(np.float16)
    return codes, scales, zeros


def make_layer(spec: LayerSpec, M: int, config: int = 0, layer_index: int = 0) -> Dict[str, np.ndarray]:
    A, B = make_branch(spec, config, layer_index)
    return {"W": make_weight(spec, config, layer_index), "A": A, "B": B,
            "x": make_x(spec, M, config, layer_index)}


# --------------------------------------------------------------------------
# The benchmark configurations (index = position in the configs list).
# --------------------------------------------------------------------------

def _llama7b(bits: int, r: int) -> List[LayerSpec]:
    sq = [LayerSpec(n, 4096, 4096, r, bits) for n in ("q_proj", "k_proj", "v_proj", "o_proj")]
    mlp = [LayerSpec("gate_proj", 11008, 4096, r, bits), LayerSpec("up_proj", 11008, 4096, r, bits),
           LayerSpec("down_proj", 4096, 11008, r, bits)]
    return sq + mlp


def config_layers(config: int) -> Tuple[List[LayerSpec], List[int]]:
    """Layer list and token counts M of benchmark configuration `config`."""
    if config == 0:      # single 4096x4096 INT4 layer, rank 32, one token
        return [LayerSpec("linear", 4096, 4096, 32, 4)], [1]
    if config == 1:      # Llama2-7B decode layer set, INT4, rank 64
        return _llama7b(4, 64), [1]
    if config == 2:      # same shapes, INT3, small batches
        return _llama7b(3, 64), [1, 4, 8, 16]
    if config == 3:      # prefill through the MLP shapes
        return [LayerSpec("gate_proj", 11008, 4096, 64, 4), LayerSpec("down_proj", 4096, 11008, 64, 4)], [1024]
    if config == 4:      # large-layer sweep, both bit widths, rank 128
        shapes = [(13824, 5120), (5120, 13824), (28672, 8192), (8192, 28672)]
        out = []
        for bits in (4, 3):
            for (n, k) in shapes:
                out.append(LayerSpec(f"l{k}x{n}_w{bits}", n, k, 128, bits, w_std=0.015))
        return out, [1, 16, 256]
    raise ValueError(f"unknown config {config}")


def algorithmic_bytes(N: int, K: int, r: int, bits: int, M: int, group: int = GROUP) -> int:
    """Bytes the method itself must move once: codes, scale+zero, A, B, x, y."""
    return N * K * bits // 8 + 2 * N * (K // group) * 2 + 2 * r * (K + N) + 2 * M * (K + N)


def algorithmic_flops(N: int, K: int, r: int, M: int) -> int:
    """2 flops per MAC: main projection plus both sub-branch projections."""
    return 2 * M * N * K + 2 * M * r * (K + N)
