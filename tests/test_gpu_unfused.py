"""fbq_linear_unfused, the conventional arrangement of Sec. 3.2 (main path, down-projection and a
read-modify-write up-projection as three launches), against the oracle and against fbq_linear.
It rounds t = x.A to fp16 between its launches, as a stand-alone kernel's output is; the fused path
does not, so the two may differ by that rounding: about 2^-11 of the sub-branch's share of y."""
import ctypes

import numpy as np
import pytest

import fbq_synth
from helpers import make_oracle_layer, oracle_y, rel_l2, to_device_layer

pytestmark = pytest.mark.gpu

CASES = [(1024, 4096, 64, 1), (300, 1408, 24, 2), (640, 8192, 128, 5), (512, 11008, 64, 16), (257, 128, 8, 1)]


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K,r,M", CASES)
def test_unfused_composition_matches_oracle_and_fused(bits, N, K, r, M):
    import torch
    import paper_2501_16385_amd as fbq
    spec = fbq_synth.LayerSpec(f"u{N}x{K}", N, K, r, bits)
    L = make_oracle_layer(spec, config=37)
    x = fbq_synth.make_x(spec, M, 37, 0)
    dev = to_device_layer(L)
    xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
    y_u = fbq.linear_unfused(dev, xd)
    y_f = fbq.linear(dev, xd)
    torch.cuda.synchronize()
    got_u = y_u.cpu().numpy().astype(np.float64)
    got_f = y_f.cpu().numpy().astype(np.float64)
    want = oracle_y(L, x)
    # the oracle's bar, with room for the fp16 rounding of t: each of the r products t_j B_jn carries 2^-11 relative
    assert rel_l2(got_u, want) <= 1.5e-3, rel_l2(got_u, want)
    assert rel_l2(got_f, want) <= 1e-3
    # against the fused path: nothing but that rounding and the final fp16 rounding of y
    assert rel_l2(got_u, got_f) <= 1.5e-3, rel_l2(got_u, got_f)


def test_unfused_rejects_more_than_sixteen_tokens():
    import torch
    import paper_2501_16385_amd as fbq
    spec = fbq_synth.LayerSpec("u", 256, 256, 8, 4)
    L = make_oracle_layer(spec, config=37)
    dev = to_device_layer(L)
    x = torch.zeros((17, 256), dtype=torch.float16, device="cuda")
    with pytest.raises(fbq.FbqError) as e:
        fbq.linear_unfused(dev, x)
    assert "unsupported" in str(e.value).lower() or e.value.code != 0
