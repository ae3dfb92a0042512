"""CPU-side checks of the C ABI: the library loads, exports what include/fbq.h declares, rejects bad
arguments before any launch, and its host-side fbq_pack writes the documented device layout."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2501_16385_amd as fbq
from oracle import fbq_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "fbq.h")).read()
    declared = sorted(set(re.findall(r"\b(fbq_[a-z_]+)\s*\(", header)))
    assert declared == sorted(fbq.EXPORTED_SYMBOLS)
    lib = fbq.load()
    for name in declared:
        assert getattr(lib, name) is not None


def test_sizes_and_status_strings():
    d = fbq.Desc(4096, 4096, 64, 4)
    assert fbq.packed_bytes(d) == 4096 * 4096 // 2
    assert fbq.packed_bytes(fbq.Desc(4096, 4096, 64, 3)) == 4096 * 4096 * 3 // 8
    assert fbq.workspace_bytes(d, 1) > 0 and fbq.workspace_bytes(fbq.Desc(4096, 4096, 0, 4), 1) == 0
    assert fbq.workspace_bytes(d, 16) >= 16 * 64 * 4
    assert fbq.workspace_bytes(fbq.Desc(4096, 4096, 0, 4), 100) >= 128 * 4096 * 2   # prefill keeps a copy of x
    assert fbq.workspace_bytes(d, 40) == 3 * fbq.workspace_bytes(d, 9)                # 17..64 tokens: the few-token kernel, every 16 tokens with words of their own
    assert fbq.workspace_bytes(d, 64) == 4 * fbq.workspace_bytes(d, 16) and fbq.workspace_bytes(d, 17) == 2 * fbq.workspace_bytes(d, 16)
    assert fbq.workspace_bytes(d, 9) >= 4 * 16 * d.r * 8                               # tagged partial sums of t, one set per K slice
    assert fbq.workspace_bytes(fbq.Desc(4096, 4096, 0, 4), 9) == 0                      # nothing to hand over without a sub-branch
    assert fbq.workspace_bytes(d, 2) == 2 * fbq.workspace_bytes(d, 1)        # one set of tagged words per token
    assert fbq.status_string(0) == "ok"
    assert all(fbq.status_string(c) for c in range(8))


@pytest.mark.parametrize("desc,code", [
    (fbq.Desc(16, 256, 8, 5), 3), (fbq.Desc(16, 256, 8, 4, 64), 3), (fbq.Desc(16, 200, 8, 4), 2),
    (fbq.Desc(0, 256, 8, 4), 2), (fbq.Desc(16, 256, 7, 4), 2), (fbq.Desc(16, 256, 264, 4), 3),
    (fbq.Desc(16, 65536, 8, 4), 3), (fbq.Desc(16, 256, -8, 4), 2)])
def test_bad_descriptors_are_rejected(desc, code):
    lib = fbq.load()
    assert lib.fbq_check_desc(ctypes.byref(desc.c())) == code
    assert fbq.packed_bytes(desc) == 0 and fbq.workspace_bytes(desc, 1) == 0
    # fbq_linear refuses before touching the GPU (bogus but aligned pointers are never dereferenced)
    p = ctypes.c_void_p(0x1000)
    assert lib.fbq_linear(ctypes.byref(desc.c()), 1, p, p, p, p, p, p, p, p, 1 << 20, None) == code


def test_linear_argument_errors_without_launch():
    lib = fbq.load()
    d = fbq.Desc(16, 256, 8, 4)
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    call = lambda M, x, ws, wb: lib.fbq_linear(ctypes.byref(d.c()), M, x, ok, ok, ok, ok, ok, ok, ws, wb, None)
    assert call(0, ok, ok, 1 << 20) == 2            # M < 1
    assert call(1, None, ok, 1 << 20) == 1          # null x
    assert call(1, odd, ok, 1 << 20) == 4           # misaligned x
    assert call(1, ok, None, 1 << 20) == 1          # workspace needed but null
    assert call(1, ok, ok, 8) == 5                  # workspace too small
    assert lib.fbq_linear(None, 1, ok, ok, ok, ok, ok, ok, ok, ok, 1 << 20, None) == 1
    # the entry point with the library's own scratch checks the same things, and its token limit, before it touches the GPU
    static = lambda M, x: lib.fbq_linear_static(ctypes.byref(d.c()), M, x, ok, ok, ok, ok, ok, ok, None)
    assert static(0, ok) == 2 and static(17, ok) == 3 and static(1, None) == 1 and static(1, odd) == 4
    assert lib.fbq_linear_static(None, 1, ok, ok, ok, ok, ok, ok, ok, None) == 1
    # the comparator (conventional three-launch sub-branch) validates like fbq_linear and stops at 16 tokens
    unfused = lambda M, x, ws, wb: lib.fbq_linear_unfused(ctypes.byref(d.c()), M, x, ok, ok, ok, ok, ok, ok, ws, wb, None)
    assert unfused(0, ok, ok, 1 << 20) == 2 and unfused(1, None, ok, 1 << 20) == 1 and unfused(1, odd, ok, 1 << 20) == 4
    assert unfused(1, ok, ok, 8) == 5 and unfused(17, ok, ok, 1 << 20) == 3
    assert lib.fbq_unpack_codes(ctypes.byref(d.c()), None, ok, None) == 1
    assert lib.fbq_reconstruct(ctypes.byref(d.c()), ok, ok, ok, None, ok, ok, None) == 1
    assert lib.fbq_quantize_feedback(ctypes.byref(d.c()), ok, ok, ok, odd, ok, ok, None) == 4


def test_group_rejects_overlapping_workspaces_and_the_test_hook_clamps():
    lib = fbq.load()
    d = fbq.Desc(16, 256, 8, 4)
    need = fbq.workspace_bytes(d, 1)
    assert need > 0
    ok = 0x10000
    layer = lambda ws: fbq.fbq._CLayerCall(d.c(), ok, ok, ok, ok, ok, ok, ok, ws, need)
    arr = (fbq.fbq._CLayerCall * 2)(layer(0x20000), layer(0x20000 + need - 16))
    assert lib.fbq_linear_group(arr, 2, 1, None) == 5            # the second workspace starts inside the first
    arr = (fbq.fbq._CLayerCall * 2)(layer(0x20000), layer(0x20000))
    assert lib.fbq_linear_group(arr, 2, 1, None) == 5
    # the poll limit: clamped to the default from above, any negative value means "fall back at once"
    default = lib.fbq_test_set_spin_limit(1 << 30)
    assert default == 1 << 15
    assert lib.fbq_test_set_spin_limit(-7) == 1 << 15            # the huge value was clamped
    assert lib.fbq_test_set_spin_limit(default) == -1
    assert lib.fbq_test_set_spin_limit(default) == default


def test_training_argument_errors_without_launch():
    lib = fbq.load()
    d = fbq.Desc(256, 512, 16, 4)
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    need = fbq.train_workspace_bytes(d, 100)
    assert need >= 2 * 256 * 512 * 2 and need % 256 == 0
    assert fbq.train_workspace_bytes(fbq.Desc(256, 512, 0, 4), 100) == 0 and fbq.train_workspace_bytes(d, 0) == 0
    assert fbq.train_workspace_bytes(d, 1 << 16) >= 512 * (1 << 16) * 2       # x transposed
    gram = lambda T, X, hs, ws, wb: lib.fbq_gram(ctypes.byref(d.c()), T, X, hs, ok, ws, wb, None)
    assert gram(0, ok, 1.0, ok, need) == 2
    assert gram(100, ok, 0.0, ok, need) == 2         # h_scale must be positive
    assert gram(100, None, 1.0, ok, need) == 1
    assert gram(100, odd, 1.0, ok, need) == 4
    assert gram(100, ok, 1.0, ok, 64) == 5
    step = lambda dd, W, hs, lr, wb: lib.fbq_train_step(ctypes.byref(dd.c()), W, ok, hs, ok, ok, lr, ok, ok, ok, ok, ok, ok, ok, ok,
                                                        ok, wb, None)
    assert step(fbq.Desc(256, 512, 0, 4), ok, 1.0, 0.1, need) == 2      # no branch to train
    assert step(d, ok, 1.0, -1.0, need) == 2
    assert step(d, None, 1.0, 0.1, need) == 1
    assert step(d, odd, 1.0, 0.1, need) == 4
    assert step(d, ok, 1.0, 0.1, 1024) == 5


@pytest.mark.parametrize("bits", [3, 4])
def test_host_pack_writes_the_documented_layout(bits):
    rng = np.random.Generator(np.random.Philox(900 + bits))
    N, K, r = 7, 384, 16
    d = fbq.Desc(N, K, r, bits)
    codes = rng.integers(0, 2 ** bits, (N, K), dtype=np.uint8)
    s = rng.random((N, K // 128)).astype(np.float16)
    z = (rng.random((N, K // 128)) * 8).astype(np.float16)
    A = rng.standard_normal((K, r)).astype(np.float16)
    B = rng.standard_normal((r, N)).astype(np.float16)
    p = fbq.pack(d, codes, s, z, A, B)
    assert np.array_equal(p.qweight, orc.pack(codes, bits))           # same words as the oracle's packer
    assert np.array_equal(orc.unpack(p.qweight, K, bits), codes)      # and the oracle reads them back
    assert np.array_equal(p.scales, s) and np.array_equal(p.zeros, z)
    assert np.array_equal(p.At, A.T) and np.array_equal(p.Bt, B.T)
    bad = codes.copy()
    bad[3, 5] = 2 ** bits
    with pytest.raises(fbq.FbqError) as e:
        fbq.pack(d, bad, s, z, A, B)
    assert e.value.code == 2


def test_loading_the_library_first_still_leaves_one_hip_runtime():
    """The binding hands torch's streams and pointers to the library, so both must sit on the same HIP runtime; torch's
    wheel has a copy of its own.  In a fresh process that touches this package before torch, only one copy may end
    up mapped (with two, every launch on a torch stream failed)."""
    import subprocess
    import sys
    code = (
        "import paper_2501_16385_amd as fbq\n"
        "fbq.load()\n"
        "import torch\n"
        "paths = {line.split()[-1] for line in open('/proc/self/maps') if 'libamdhip64' in line}\n"
        "print(len(paths), sorted(paths))\n"
        "assert len(paths) == 1, paths\n"
    )
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
