"""fbq_linear_static (the entry point that allocates nothing: its hand-over scratch is a device array
inside the library) against fbq_linear, through the C ABI, on two calls in a row, the second on a
smaller layer with fewer tokens.  Both entry points run the same kernels with the same fixed
summation orders, so the outputs must agree bit for bit; the oracle's bar is checked as well."""
import ctypes

import numpy as np
import pytest

import fbq_synth
from helpers import make_oracle_layer, oracle_y, rel_l2, to_device_layer

pytestmark = pytest.mark.gpu

Y_TOL = 1e-3

# (N, K, r, M) pairs: a call and a smaller one right behind it, through both decode kernel families
PAIRS = [
    ((1024, 4096, 64, 16), (300, 1408, 24, 1)),      # few-token kernel, then the one-token GEMV
    ((512, 11008, 128, 2), (257, 128, 8, 1)),        # GEMV with two K slices of t, then a single group
    ((640, 8192, 256, 9), (96, 2048, 32, 4)),        # widest sub-branch, then a narrow one, both few-token
]


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("first,second", PAIRS)
def test_static_scratch_entry_matches_fbq_linear(bits, first, second):
    import torch
    import paper_2501_16385_amd as fbq
    lib = fbq.load()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ptr = lambda t: ctypes.c_void_p(0 if t is None else t.data_ptr())
    cases = []
    for (N, K, r, M) in (first, second):
        spec = fbq_synth.LayerSpec(f"s{N}x{K}", N, K, r, bits)
        L = make_oracle_layer(spec, config=31)
        x = fbq_synth.make_x(spec, M, 31, 0)
        dev = to_device_layer(L)
        xd = torch.from_numpy(x.view(np.int16)).cuda()
        y_ws = torch.full((M, N), -1, dtype=torch.int16, device="cuda")
        y_st = torch.full((M, N), -2, dtype=torch.int16, device="cuda")
        ws = torch.zeros(max(16, fbq.workspace_bytes(dev.desc, M)), dtype=torch.uint8, device="cuda")
        cases.append((L, x, dev, xd, y_ws, y_st, ws, M))
    torch.cuda.synchronize()
    # the two static calls go out back to back on one stream, with nothing in between
    for (L, x, dev, xd, y_ws, y_st, ws, M) in cases:
        d = dev.desc.c()
        rc = lib.fbq_linear_static(ctypes.byref(d), M, ptr(xd), ptr(dev.qweight), ptr(dev.scales), ptr(dev.zeros), ptr(dev.At),
                                   ptr(dev.Bt), ptr(y_st), stream)
        assert rc == 0, fbq.status_string(rc)
    for (L, x, dev, xd, y_ws, y_st, ws, M) in cases:
        d = dev.desc.c()
        rc = lib.fbq_linear(ctypes.byref(d), M, ptr(xd), ptr(dev.qweight), ptr(dev.scales), ptr(dev.zeros), ptr(dev.At), ptr(dev.Bt),
                            ptr(y_ws), ptr(ws), ctypes.c_size_t(ws.numel()), stream)
        assert rc == 0, fbq.status_string(rc)
    torch.cuda.synchronize()
    for (L, x, dev, xd, y_ws, y_st, ws, M) in cases:
        got_st = y_st.cpu().numpy().view(np.float16)
        got_ws = y_ws.cpu().numpy().view(np.float16)
        want = oracle_y(L, x)
        assert np.array_equal(got_st.view(np.uint16), got_ws.view(np.uint16)), "static-scratch call differs from fbq_linear"
        assert rel_l2(got_st, want) <= Y_TOL
        for m in range(M):
            assert rel_l2(got_st[m], want[m]) <= Y_TOL


def test_static_scratch_entry_refuses_what_it_cannot_serve():
    import torch
    import paper_2501_16385_amd as fbq
    lib = fbq.load()
    d = fbq.Desc(64, 256, 8, 4)
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p = ctypes.c_void_p(buf.data_ptr())
    call = lambda M, x: lib.fbq_linear_static(ctypes.byref(d.c()), M, x, p, p, p, p, p, p, None)
    assert call(17, p) == 3      # more tokens than the static scratch serves
    assert call(0, p) == 2
    assert call(1, None) == 1
    assert call(1, ctypes.c_void_p(buf.data_ptr() + 4)) == 4
