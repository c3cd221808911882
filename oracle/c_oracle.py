"""ctypes front end of oracle/dz_oracle.c (test infrastructure only; see that file's header)."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dz_oracle.c")
_LIB = os.path.join(_HERE, "libdz_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no fp contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.dzo_num_threads.restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, shape=None):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def num_threads() -> int:
    return int(lib().dzo_num_threads())


def set_threads(n: int) -> None:
    lib().dzo_set_threads(ctypes.c_int(n))


def validate(codes, idx, scale, zero, bits: int, group: int) -> int:
    codes = _chk(codes, np.uint8)
    N, K = codes.shape[0], codes.shape[1] * 2
    idx = _chk(idx, np.uint8, (N, K // 2))
    scale = _chk(scale, np.float16, (N, K // group))
    zero = _chk(zero, np.float16, (N, K // group))
    return int(lib().dzo_validate(_p(codes), _p(idx), _p(scale), _p(zero), N, K, bits, group))


def dequant(codes, idx, scale, zero, bits: int, group: int) -> np.ndarray:
    """Dense fp32 [N][K] matrix the canonical tables stand for."""
    codes = _chk(codes, np.uint8)
    N, K = codes.shape[0], codes.shape[1] * 2
    idx = _chk(idx, np.uint8, (N, K // 2))
    scale = _chk(scale, np.float16, (N, K // group))
    zero = _chk(zero, np.float16, (N, K // group))
    out = np.empty((N, K), np.float32)
    lib().dzo_dequant(_p(codes), _p(idx), _p(scale), _p(zero), N, K, bits, group, _p(out))
    return out


def linear(x, W, dense_deltas: Optional[Sequence[np.ndarray]], token_to_delta,
           acc64: bool = False) -> np.ndarray:
    """y[t] = x[t] . (W + Delta_{token_to_delta[t]})^T as fp32 [T][N].
    W may be None (delta term only); dense_deltas may be None/empty (base term only)."""
    x = _chk(x, np.float16)
    T, K = x.shape
    D = 0 if not dense_deltas else len(dense_deltas)
    if W is not None:
        W = _chk(W, np.float16)
        N = W.shape[0]
        assert W.shape == (N, K)
    else:
        N = dense_deltas[0].shape[0]
    keep = []
    ptrs = None
    if D:
        keep = [_chk(d, np.float32, (N, K)) for d in dense_deltas]
        ptrs = (ctypes.c_void_p * D)(*[d.ctypes.data for d in keep])
    ids = None if token_to_delta is None else _chk(token_to_delta, np.int32, (T,))
    y = np.empty((T, N), np.float32)
    lib().dzo_linear(_p(x), _p(W), ptrs, D, _p(ids), T, N, K, 1 if acc64 else 0, _p(y))
    return y


def segment(token_to_delta, D: int):
    ids = _chk(token_to_delta, np.int32)
    T = ids.shape[0]
    counts = np.zeros(D, np.int32)
    offsets = np.zeros(D + 1, np.int32)
    perm = np.zeros(T, np.int32)
    lib().dzo_segment(_p(ids), T, D, _p(counts), _p(offsets), _p(perm))
    return counts, offsets, perm
