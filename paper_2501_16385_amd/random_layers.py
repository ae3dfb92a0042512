"""Random packed layers for timing: the kernels' speed does not depend on the values, so uniformly random
packed words with plausible scales, zero points and sub-branch stand in for a quantized layer."""
from __future__ import annotations

import torch

from . import fbq


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


def branch_free_twin(layer: fbq.DeviceLayer) -> fbq.DeviceLayer:
    """The same packed weights without the sub-branch (r = 0): the comparator of "branch overhead %"."""
    d = layer.desc
    return fbq.DeviceLayer(fbq.Desc(d.N, d.K, 0, d.bits, d.group), layer.qweight, layer.scales, layer.zeros, None, None)
