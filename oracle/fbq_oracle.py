"""ctypes front end of the CPU oracle in fbq_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product never imports this module and this
module never imports the product.  Argument marshalling only: every number is
computed by the C file, whose header states what is computed and how it is
pinned - with one exception, `gram` (H = X^T X), which is the plain numpy
product written out here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fbq_oracle.c")
_LIB = os.path.join(_HERE, "libfbq_oracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over output rows)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.fbqo_half_to_double.restype = ctypes.c_double
        lib.fbqo_half_to_double.argtypes = [ctypes.c_uint16]
        lib.fbqo_double_to_half.restype = ctypes.c_uint16
        lib.fbqo_double_to_half.argtypes = [ctypes.c_double]
        _lib = lib
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f16(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    if a.dtype == np.uint16:
        return a
    raise TypeError("expected fp16 (or its uint16 bit pattern)")


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def num_threads() -> int:
    return int(_load().fbqo_num_threads())


def half_to_double(bits: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(h.shape, np.float64)
    _load().fbqo_half_to_double_array(_p(h), _p(out), ctypes.c_long(h.size))
    return out


def double_to_half(d: np.ndarray) -> np.ndarray:
    d = np.ascontiguousarray(d, dtype=np.float64)
    out = np.empty(d.shape, np.uint16)
    _load().fbqo_double_to_half_array(_p(d), _p(out), ctypes.c_long(d.size))
    return out


def sigma(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """Sigma [N,K] fp64 from A [K,r], B [r,N] fp16."""
    K, r = A.shape
    N = B.shape[1]
    out = np.empty((N, K), np.float64)
    _check(_load().fbqo_sigma(N, K, r, _p(_f16(A)), _p(_f16(B)), _p(out)), "sigma")
    return out


def quantize(W: np.ndarray, A: Optional[np.ndarray], B: Optional[np.ndarray], bits: int, group: int
             ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Feedback quantizer Q(W - Sigma): codes [N,K] u8, scales [N,G] f16, zeros [N,G] f16."""
    N, K = W.shape
    r = 0 if A is None else A.shape[1]
    if K % group:
        raise ValueError("K must be a multiple of the group size")
    G = K // group
    codes = np.empty((N, K), np.uint8)
    s = np.empty((N, G), np.uint16)
    z = np.empty((N, G), np.uint16)
    a = _f16(A) if r else None
    b = _f16(B) if r else None
    _check(_load().fbqo_quantize(N, K, r, bits, group, _p(_f16(W)), _p(a), _p(b), _p(codes), _p(s), _p(z)),
           "quantize")
    return codes, s.view(np.float16), z.view(np.float16)


def packed_words(K: int, bits: int) -> int:
    return K * bits // 32


def pack(codes: np.ndarray, bits: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    words = np.empty((N, packed_words(K, bits)), np.uint32)
    _check(_load().fbqo_pack(N, K, bits, _p(codes), _p(words)), "pack")
    return words


def unpack(words: np.ndarray, K: int, bits: int) -> np.ndarray:
    words = np.ascontiguousarray(words, dtype=np.uint32)
    N = words.shape[0]
    codes = np.empty((N, K), np.uint8)
    _check(_load().fbqo_unpack(N, K, bits, _p(words), _p(codes)), "unpack")
    return codes


def dequant(words: np.ndarray, scales: np.ndarray, zeros: np.ndarray, K: int, bits: int, group: int) -> np.ndarray:
    words = np.ascontiguousarray(words, dtype=np.uint32)
    N = words.shape[0]
    out = np.empty((N, K), np.float64)
    _check(_load().fbqo_dequant(N, K, bits, group, _p(words), _p(_f16(scales)), _p(_f16(zeros)), _p(out)), "dequant")
    return out


def reconstruct(words: np.ndarray, scales: np.ndarray, zeros: np.ndarray, A: Optional[np.ndarray],
                B: Optional[np.ndarray], K: int, bits: int, group: int) -> np.ndarray:
    """W_F = Q(W - Sigma) + Sigma, [N,K] fp64."""
    words = np.ascontiguousarray(words, dtype=np.uint32)
    N = words.shape[0]
    r = 0 if A is None else A.shape[1]
    out = np.empty((N, K), np.float64)
    a = _f16(A) if r else None
    b = _f16(B) if r else None
    _check(_load().fbqo_reconstruct(N, K, r, bits, group, _p(words), _p(_f16(scales)), _p(_f16(zeros)), _p(a), _p(b),
                                    _p(out)), "reconstruct")
    return out


def linear(x: np.ndarray, words: np.ndarray, scales: np.ndarray, zeros: np.ndarray, A: Optional[np.ndarray],
           B: Optional[np.ndarray], bits: int, group: int) -> np.ndarray:
    """y [M,N] fp64 = x.Wq^T + (x.A).B, weights dequantized on the fly."""
    words = np.ascontiguousarray(words, dtype=np.uint32)
    M, K = x.shape
    N = words.shape[0]
    r = 0 if A is None else A.shape[1]
    y = np.empty((M, N), np.float64)
    a = _f16(A) if r else None
    b = _f16(B) if r else None
    _check(_load().fbqo_linear(M, N, K, r, bits, group, _p(_f16(x)), _p(words), _p(_f16(scales)), _p(_f16(zeros)),
                               _p(a), _p(b), _p(y)), "linear")
    return y


def dense_linear(x: np.ndarray, Wd: np.ndarray) -> np.ndarray:
    """y [M,N] fp64 = x.Wd^T for a materialised fp64 weight."""
    Wd = np.ascontiguousarray(Wd, dtype=np.float64)
    M, K = x.shape
    N = Wd.shape[0]
    y = np.empty((M, N), np.float64)
    _check(_load().fbqo_dense_linear(M, N, K, _p(_f16(x)), _p(Wd), _p(y)), "dense_linear")
    return y


def gram(X: np.ndarray) -> np.ndarray:
    """H = X^T X in fp64 for X [T,K] fp16: the matrix through which the loss and gradient of Sec. 4.2
    depend on the calibration activations."""
    Xd = np.ascontiguousarray(X).astype(np.float64)
    return Xd.T @ Xd


def train_step(W: np.ndarray, X: np.ndarray, A: np.ndarray, B: np.ndarray, lr: float, bits: int, group: int):
    """One loop-body iteration of Alg. 1.  A [K,r], B [r,N] fp64 masters, updated IN PLACE.
    Returns a dict describing the parameters before the update: codes, scales, zeros, A16, B16,
    loss, gradA, gradB."""
    N, K = W.shape
    T = X.shape[0]
    r = A.shape[1]
    if A.dtype != np.float64 or B.dtype != np.float64 or not A.flags.c_contiguous or not B.flags.c_contiguous:
        raise TypeError("A and B must be contiguous fp64 arrays (they are updated in place)")
    G = K // group
    codes = np.empty((N, K), np.uint8)
    s = np.empty((N, G), np.uint16)
    z = np.empty((N, G), np.uint16)
    A16 = np.empty((K, r), np.uint16)
    B16 = np.empty((r, N), np.uint16)
    gA = np.empty((K, r), np.float64)
    gB = np.empty((r, N), np.float64)
    loss = ctypes.c_double(0.0)
    lib = _load()
    lib.fbqo_train_step.argtypes = [ctypes.c_int] * 6 + [ctypes.c_void_p] * 4 + [ctypes.c_double] + [ctypes.c_void_p] * 7 + [
        ctypes.POINTER(ctypes.c_double)]
    _check(lib.fbqo_train_step(N, K, r, bits, group, T, _p(_f16(W)), _p(_f16(X)), _p(A), _p(B), float(lr), _p(codes), _p(s),
                               _p(z), _p(A16), _p(B16), _p(gA), _p(gB), ctypes.byref(loss)), "train_step")
    return {"codes": codes, "scales": s.view(np.float16), "zeros": z.view(np.float16), "A16": A16.view(np.float16),
            "B16": B16.view(np.float16), "loss": loss.value, "gradA": gA, "gradB": gB}
