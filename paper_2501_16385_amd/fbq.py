"""ctypes binding of the C ABI in include/fbq.h: argument marshalling only.

Device buffers are torch tensors (torch is used for device memory and streams, nothing else);
every step of the path runs in the library's own kernels.  There is no CPU fallback: if
libfbq.so is missing or the GPU is absent the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfbq.so")
_lib: Optional[ctypes.CDLL] = None

EXPORTED_SYMBOLS = ["fbq_status_string", "fbq_check_desc", "fbq_packed_bytes", "fbq_workspace_bytes", "fbq_pack",
                    "fbq_linear", "fbq_linear_static", "fbq_linear_unfused", "fbq_linear_group", "fbq_reconstruct", "fbq_unpack_codes", "fbq_quantize_feedback",
                    "fbq_train_workspace_bytes", "fbq_gram", "fbq_train_step", "fbq_test_set_spin_limit",
                    "fbq_measure_read_stream"]


class FbqError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {status_string(code)} (fbq_status {code})")


class _CDesc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("K", ctypes.c_int32), ("r", ctypes.c_int32), ("bits", ctypes.c_int32),
                ("group", ctypes.c_int32)]


class _CLayerCall(ctypes.Structure):
    _fields_ = [("desc", _CDesc), ("x", ctypes.c_void_p), ("qweight", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("zeros", ctypes.c_void_p), ("At", ctypes.c_void_p), ("Bt", ctypes.c_void_p), ("y", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


@dataclass(frozen=True)
class Desc:
    N: int
    K: int
    r: int
    bits: int
    group: int = 128

    def c(self) -> _CDesc:
        return _CDesc(self.N, self.K, self.r, self.bits, self.group)


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Loads libfbq.so (built by paper_2501_16385_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(f"{_LIB_PATH} not built: run `python -m paper_2501_16385_amd.build`")
        # The library and torch must share ONE HIP runtime: the streams and device pointers this binding hands over are
        # torch's.  torch's wheel brings its own copy of the runtime; loaded first, it also serves this library, but
        # when this library came first the process ended up with two runtimes and every launch on a torch stream
        # failed with a launch error.
        import torch  # noqa: F401
        lib = ctypes.CDLL(_LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        dp = ctypes.POINTER(_CDesc)
        lib.fbq_status_string.restype = ctypes.c_char_p
        lib.fbq_status_string.argtypes = [i32]
        lib.fbq_check_desc.restype = i32
        lib.fbq_check_desc.argtypes = [dp]
        lib.fbq_packed_bytes.restype = sz
        lib.fbq_packed_bytes.argtypes = [dp]
        lib.fbq_workspace_bytes.restype = sz
        lib.fbq_workspace_bytes.argtypes = [dp, i32]
        lib.fbq_pack.restype = i32
        lib.fbq_pack.argtypes = [dp] + [vp] * 10
        lib.fbq_linear.restype = i32
        lib.fbq_linear.argtypes = [dp, i32] + [vp] * 8 + [sz, vp]
        lib.fbq_linear_static.restype = i32
        lib.fbq_linear_static.argtypes = [dp, i32] + [vp] * 8
        lib.fbq_linear_unfused.restype = i32
        lib.fbq_linear_unfused.argtypes = [dp, i32] + [vp] * 8 + [sz, vp]
        lib.fbq_measure_read_stream.restype = i32
        lib.fbq_measure_read_stream.argtypes = [vp, sz, vp]
        lib.fbq_test_set_spin_limit.restype = i32
        lib.fbq_test_set_spin_limit.argtypes = [i32]
        lib.fbq_linear_group.restype = i32
        lib.fbq_linear_group.argtypes = [ctypes.POINTER(_CLayerCall), i32, i32, vp]
        lib.fbq_reconstruct.restype = i32
        lib.fbq_reconstruct.argtypes = [dp] + [vp] * 7
        lib.fbq_unpack_codes.restype = i32
        lib.fbq_unpack_codes.argtypes = [dp] + [vp] * 3
        lib.fbq_quantize_feedback.restype = i32
        lib.fbq_quantize_feedback.argtypes = [dp] + [vp] * 7
        f32 = ctypes.c_float
        lib.fbq_train_workspace_bytes.restype = sz
        lib.fbq_train_workspace_bytes.argtypes = [dp, i32]
        lib.fbq_gram.restype = i32
        lib.fbq_gram.argtypes = [dp, i32, vp, f32, vp, vp, sz, vp]
        lib.fbq_train_step.restype = i32
        lib.fbq_train_step.argtypes = [dp, vp, vp, f32, vp, vp, f32] + [vp] * 9 + [sz, vp]
        _lib = lib
    return _lib


def status_string(code: int) -> str:
    return load().fbq_status_string(int(code)).decode()


def _check(code: int, what: str) -> None:
    if code != 0:
        raise FbqError(code, what)


def packed_bytes(d: Desc) -> int:
    return int(load().fbq_packed_bytes(ctypes.byref(d.c())))


def workspace_bytes(d: Desc, M: int) -> int:
    return int(load().fbq_workspace_bytes(ctypes.byref(d.c()), int(M)))


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _dev_ptr(t) -> Optional[ctypes.c_void_p]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("expected a device tensor")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream=None) -> ctypes.c_void_p:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


@dataclass
class PackedLayer:
    """Host-side arrays in the device layout (outputs of fbq_pack)."""
    desc: Desc
    qweight: np.ndarray   # uint32 [N, K*bits/32]
    scales: np.ndarray    # float16 [N, G]
    zeros: np.ndarray     # float16 [N, G]
    At: Optional[np.ndarray]   # float16 [r, K]
    Bt: Optional[np.ndarray]   # float16 [N, r]


def pack(d: Desc, codes: np.ndarray, scales: np.ndarray, zeros: np.ndarray, A: Optional[np.ndarray],
         B: Optional[np.ndarray]) -> PackedLayer:
    """fbq_pack: canonical host tensors -> device-layout host tensors."""
    G = d.K // d.group
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float16)
    zeros = np.ascontiguousarray(zeros, dtype=np.float16)
    if codes.shape != (d.N, d.K) or scales.shape != (d.N, G) or zeros.shape != (d.N, G):
        raise ValueError("shape mismatch")
    nbytes = packed_bytes(d)
    if nbytes == 0:
        _check(int(load().fbq_check_desc(ctypes.byref(d.c()))), "fbq_pack")
    qw = np.empty((d.N, nbytes // 4 // d.N), np.uint32)
    s_out, z_out = np.empty_like(scales), np.empty_like(zeros)
    if d.r:
        A = np.ascontiguousarray(A, dtype=np.float16)
        B = np.ascontiguousarray(B, dtype=np.float16)
        if A.shape != (d.K, d.r) or B.shape != (d.r, d.N):
            raise ValueError("shape mismatch")
        A_out, Bt_out = np.empty((d.r, d.K), np.float16), np.empty((d.N, d.r), np.float16)
    else:
        A = B = A_out = Bt_out = None
    rc = load().fbq_pack(ctypes.byref(d.c()), _np_ptr(codes), _np_ptr(scales), _np_ptr(zeros), _np_ptr(A), _np_ptr(B),
                         _np_ptr(qw), _np_ptr(s_out), _np_ptr(z_out), _np_ptr(A_out), _np_ptr(Bt_out))
    _check(rc, "fbq_pack")
    return PackedLayer(d, qw, s_out, z_out, A_out, Bt_out)


@dataclass
class DeviceLayer:
    """Device tensors of one layer plus its scratch."""
    desc: Desc
    qweight: "object"
    scales: "object"
    zeros: "object"
    At: "object"
    Bt: "object"


def upload_layer(p: PackedLayer, device="cuda") -> DeviceLayer:
    import torch
    t = lambda a: None if a is None else torch.from_numpy(a.view(np.int16) if a.dtype == np.float16 else a.view(np.int32)).to(device)
    return DeviceLayer(p.desc, t(p.qweight), t(p.scales), t(p.zeros), t(p.At), t(p.Bt))


def linear(layer: DeviceLayer, x, y=None, workspace=None, stream=None):
    """fbq_linear: x [M, K] fp16 device tensor -> y [M, N] fp16 device tensor."""
    import torch
    d = layer.desc
    M = int(x.shape[0])
    if y is None:
        y = torch.empty((M, d.N), dtype=torch.float16, device=x.device)
    need = workspace_bytes(d, M)
    if workspace is None and need:
        workspace = torch.zeros(need, dtype=torch.uint8, device=x.device)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().fbq_linear(ctypes.byref(d.c()), M, _dev_ptr(x), _dev_ptr(layer.qweight), _dev_ptr(layer.scales),
                           _dev_ptr(layer.zeros), _dev_ptr(layer.At), _dev_ptr(layer.Bt), _dev_ptr(y), _dev_ptr(workspace),
                           wbytes, _stream(stream))
    _check(rc, "fbq_linear")
    return y


def linear_unfused(layer: DeviceLayer, x, y=None, workspace=None, stream=None):
    """fbq_linear_unfused: the comparator of Sec. 3.2 - main path, down-projection and read-modify-write
    up-projection as three launches (up to 16 tokens)."""
    import torch
    d = layer.desc
    M = int(x.shape[0])
    if y is None:
        y = torch.empty((M, d.N), dtype=torch.float16, device=x.device)
    need = workspace_bytes(d, M)
    if workspace is None and need:
        workspace = torch.zeros(need, dtype=torch.uint8, device=x.device)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().fbq_linear_unfused(ctypes.byref(d.c()), M, _dev_ptr(x), _dev_ptr(layer.qweight), _dev_ptr(layer.scales),
                                   _dev_ptr(layer.zeros), _dev_ptr(layer.At), _dev_ptr(layer.Bt), _dev_ptr(y), _dev_ptr(workspace),
                                   wbytes, _stream(stream))
    _check(rc, "fbq_linear_unfused")
    return y


def linear_static(layer: DeviceLayer, x, y=None, stream=None):
    """fbq_linear_static: fbq_linear for up to 16 tokens with the library's own scratch (nothing is allocated
    by the call; pass y to keep this wrapper from allocating the output)."""
    import torch
    d = layer.desc
    M = int(x.shape[0])
    if y is None:
        y = torch.empty((M, d.N), dtype=torch.float16, device=x.device)
    rc = load().fbq_linear_static(ctypes.byref(d.c()), M, _dev_ptr(x), _dev_ptr(layer.qweight), _dev_ptr(layer.scales),
                                  _dev_ptr(layer.zeros), _dev_ptr(layer.At), _dev_ptr(layer.Bt), _dev_ptr(y), _stream(stream))
    _check(rc, "fbq_linear_static")
    return y


def make_group(layers, xs, ys, workspaces):
    """Marshals a list of (layer, x, y, workspace) into the array fbq_linear_group takes (reusable)."""
    arr = (_CLayerCall * len(layers))()
    ptr = lambda t: None if t is None else t.data_ptr()
    for i, (l, x, y, ws) in enumerate(zip(layers, xs, ys, workspaces)):
        arr[i] = _CLayerCall(l.desc.c(), ptr(x), ptr(l.qweight), ptr(l.scales), ptr(l.zeros), ptr(l.At), ptr(l.Bt), ptr(y),
                             ptr(ws), 0 if ws is None else ws.numel() * ws.element_size())
    return arr


def linear_group(layers, xs, ys=None, workspaces=None, stream=None):
    """fbq_linear_group: several independent layers, same token count, as few launches as possible."""
    import torch
    M = int(xs[0].shape[0])
    if ys is None:
        ys = [torch.empty((M, l.desc.N), dtype=torch.float16, device=x.device) for l, x in zip(layers, xs)]
    if workspaces is None:
        workspaces = []
        for l, x in zip(layers, xs):
            need = workspace_bytes(l.desc, M)
            workspaces.append(torch.zeros(need, dtype=torch.uint8, device=x.device) if need else None)
    arr = make_group(layers, xs, ys, workspaces)
    _check(load().fbq_linear_group(arr, len(layers), M, _stream(stream)), "fbq_linear_group")
    return ys


def reconstruct(layer: DeviceLayer, stream=None):
    """fbq_reconstruct: W_F [N, K] fp32 device tensor."""
    import torch
    d = layer.desc
    out = torch.empty((d.N, d.K), dtype=torch.float32, device=layer.qweight.device)
    rc = load().fbq_reconstruct(ctypes.byref(d.c()), _dev_ptr(layer.qweight), _dev_ptr(layer.scales), _dev_ptr(layer.zeros),
                                _dev_ptr(layer.At), _dev_ptr(layer.Bt), _dev_ptr(out), _stream(stream))
    _check(rc, "fbq_reconstruct")
    return out


def unpack_codes(layer: DeviceLayer, stream=None):
    """fbq_unpack_codes: integer codes [N, K] uint8 device tensor."""
    import torch
    d = layer.desc
    out = torch.empty((d.N, d.K), dtype=torch.uint8, device=layer.qweight.device)
    rc = load().fbq_unpack_codes(ctypes.byref(d.c()), _dev_ptr(layer.qweight), _dev_ptr(out), _stream(stream))
    _check(rc, "fbq_unpack_codes")
    return out


def quantize_feedback(d: Desc, W, At=None, Bt=None, stream=None) -> DeviceLayer:
    """fbq_quantize_feedback: W [N, K] fp16, At [r, K], Bt [N, r] device tensors -> packed device layer."""
    import torch
    dev = W.device
    nbytes = packed_bytes(d)
    if nbytes == 0:
        _check(int(load().fbq_check_desc(ctypes.byref(d.c()))), "fbq_quantize_feedback")
    qw = torch.empty((d.N, nbytes // 4 // d.N), dtype=torch.int32, device=dev)
    G = d.K // d.group
    s = torch.empty((d.N, G), dtype=torch.int16, device=dev)
    z = torch.empty((d.N, G), dtype=torch.int16, device=dev)
    rc = load().fbq_quantize_feedback(ctypes.byref(d.c()), _dev_ptr(W), _dev_ptr(At), _dev_ptr(Bt), _dev_ptr(qw), _dev_ptr(s),
                                      _dev_ptr(z), _stream(stream))
    _check(rc, "fbq_quantize_feedback")
    return DeviceLayer(d, qw, s, z, At, Bt)


def train_workspace_bytes(d: Desc, T: int) -> int:
    return int(load().fbq_train_workspace_bytes(ctypes.byref(d.c()), int(T)))


def gram(d: Desc, X, h_scale: float, workspace=None, stream=None):
    """fbq_gram: X [T, K] fp16 device tensor -> fp16(h_scale * X^T X) [K, K] device tensor."""
    import torch
    T = int(X.shape[0])
    if workspace is None:
        workspace = torch.empty(max(256, train_workspace_bytes(d, T)), dtype=torch.uint8, device=X.device)
    H16 = torch.empty((d.K, d.K), dtype=torch.float16, device=X.device)
    rc = load().fbq_gram(ctypes.byref(d.c()), T, _dev_ptr(X), float(h_scale), _dev_ptr(H16), _dev_ptr(workspace),
                         workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "fbq_gram")
    return H16


@dataclass
class TrainState:
    """Device tensors one reconstruction iteration reads and writes (allocated once, reused every step)."""
    desc: Desc
    At32: "object"        # [r, K] fp32 master, updated in place
    Bt32: "object"        # [N, r] fp32 master, updated in place
    layer: DeviceLayer    # the layer as it was BEFORE the last step's update (fp16 branch, codes, scales, zeros)
    grad_At: "object"
    grad_Bt: "object"
    loss: "object"        # 1 fp32
    workspace: "object"


def train_state(d: Desc, At32, Bt32) -> TrainState:
    import torch
    dev = At32.device
    G = d.K // d.group
    layer = DeviceLayer(d, torch.empty((d.N, packed_bytes(d) // 4 // d.N), dtype=torch.int32, device=dev),
                        torch.empty((d.N, G), dtype=torch.int16, device=dev), torch.empty((d.N, G), dtype=torch.int16, device=dev),
                        torch.empty((d.r, d.K), dtype=torch.int16, device=dev), torch.empty((d.N, d.r), dtype=torch.int16, device=dev))
    return TrainState(d, At32, Bt32, layer, torch.empty((d.r, d.K), dtype=torch.float32, device=dev),
                      torch.empty((d.N, d.r), dtype=torch.float32, device=dev), torch.empty(1, dtype=torch.float32, device=dev),
                      torch.empty(max(256, train_workspace_bytes(d, 1)), dtype=torch.uint8, device=dev))


def train_step(st: TrainState, W, H16, h_scale: float, lr: float, stream=None, want_loss: bool = True) -> None:
    """fbq_train_step: one loop-body iteration of Alg. 1 on the state's masters (want_loss=False skips the
    one contraction only the loss needs)."""
    d, l = st.desc, st.layer
    rc = load().fbq_train_step(ctypes.byref(d.c()), _dev_ptr(W), _dev_ptr(H16), float(h_scale), _dev_ptr(st.At32),
                               _dev_ptr(st.Bt32), float(lr), _dev_ptr(l.qweight), _dev_ptr(l.scales), _dev_ptr(l.zeros),
                               _dev_ptr(l.At), _dev_ptr(l.Bt), _dev_ptr(st.grad_At), _dev_ptr(st.grad_Bt), _dev_ptr(st.loss) if want_loss else None,
                               _dev_ptr(st.workspace), st.workspace.numel() * st.workspace.element_size(), _stream(stream))
    _check(rc, "fbq_train_step")
