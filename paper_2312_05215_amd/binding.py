from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

__all__ = [
    "DZ_OK", "DZ_ERR_ARG", "DZ_ERR_SHAPE", "DZ_ERR_BITS", "DZ_ERR_ALIGN", "DZ_ERR_HIP", "DZ_ERR_INDEX", "DZ_ERR_LIMIT",
    "DZ_OPT_SPLIT_K", "DZ_OPT_WORKGROUPS", "DZ_OPT_ROUND_TILES", "DZ_OPT_LARGE_BATCH_STREAMING", "DZ_OPT_WIDE_TILE",
    "DZ_OPT_REUSE_SEGMENTS", "dz_set_option", "dz_linear_static", "dz_probe_read", "dz_probe_mfma", "dz_compress_delta", "dz_lora_sbmm",
    "dz_qpacked_bytes", "dz_qpack_delta", "dz_qunpack_delta", "dz_qsbmm", "dz_qlinear", "dz_merge_delta",
    "DZ_MAX_DELTAS", "DzError", "lib", "lib_path", "dz_strerror", "dz_create", "dz_destroy",
    "dz_packed_bytes", "dz_pack_delta", "dz_unpack_delta", "dz_segment", "dz_base_gemm", "dz_sbmm",
    "dz_linear", "dz_linear_group", "dz_check", "Context", "SYMBOLS", "DZ_MAX_GROUP",
    "dz_cache_create", "dz_cache_destroy", "dz_cache_acquire", "dz_cache_wait", "dz_cache_release", "dz_cache_stats",
]

DZ_OK, DZ_ERR_ARG, DZ_ERR_SHAPE, DZ_ERR_BITS, DZ_ERR_ALIGN, DZ_ERR_HIP, DZ_ERR_INDEX, DZ_ERR_LIMIT = 0, -1, -2, -3, -4, -5, -6, -7
(DZ_OPT_SPLIT_K, DZ_OPT_WORKGROUPS, DZ_OPT_ROUND_TILES, DZ_OPT_LARGE_BATCH_STREAMING, DZ_OPT_WIDE_TILE,
 DZ_OPT_REUSE_SEGMENTS) = 1, 2, 3, 4, 5, 6
DZ_MAX_DELTAS = 128
DZ_MAX_GROUP = 4

SYMBOLS = ["dz_strerror", "dz_last_hip_error", "dz_create", "dz_destroy", "dz_set_option", "dz_linear_static", "dz_probe_read", "dz_probe_mfma",
           "dz_compress_delta", "dz_lora_sbmm", "dz_qpacked_bytes", "dz_qpack_delta", "dz_qunpack_delta", "dz_qsbmm",
           "dz_qlinear", "dz_merge_delta", "dz_packed_bytes", "dz_pack_delta",
           "dz_unpack_delta", "dz_segment", "dz_base_gemm", "dz_sbmm", "dz_linear", "dz_linear_group", "dz_check",
           "dz_cache_create", "dz_cache_destroy", "dz_cache_acquire", "dz_cache_wait", "dz_cache_release",
           "dz_cache_stats"]

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


class DzError(RuntimeError):
    def __init__(self, rc: int, where: str, detail: str = ""):
        self.rc = rc
        super().__init__(f"{where}: {dz_strerror(rc)} (rc={rc}){(' -- ' + detail) if detail else ''}")


def lib_path() -> str:
    return os.path.join(_HERE, "libdz.so")


def lib() -> ctypes.CDLL:
    """The loaded libdz.so.  Raises if it is missing: there is no other implementation."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} not found: build it with `python -m paper_2312_05215_amd.build` "
                              "(or __graft_entry__.build()); libdz has no fallback path")
        L = ctypes.CDLL(path)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        L.dz_strerror.restype = ctypes.c_char_p
        L.dz_strerror.argtypes = [ci]
        L.dz_last_hip_error.restype = ctypes.c_char_p
        L.dz_last_hip_error.argtypes = [vp]
        L.dz_create.argtypes = [ctypes.POINTER(vp), ci]
        L.dz_destroy.argtypes = [vp]
        L.dz_packed_bytes.restype = ctypes.c_size_t
        L.dz_packed_bytes.argtypes = [ci, ci, ci, ci]
        L.dz_pack_delta.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, vp, vp]
        L.dz_unpack_delta.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
        L.dz_segment.argtypes = [vp, vp, ci, ci, vp, vp, vp, vp]
        L.dz_base_gemm.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp]
        L.dz_sbmm.argtypes = [vp, vp, ctypes.POINTER(vp), ci, vp, vp, ci, ci, ci, ci, ci, ci, vp]
        L.dz_linear.argtypes = [vp, vp, vp, ctypes.POINTER(vp), ci, vp, vp, ci, ci, ci, ci, ci, vp]
        L.dz_linear_group.argtypes = [vp, vp, ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ci, vp, ctypes.POINTER(vp),
                                      ctypes.POINTER(ci), ci, ci, ci, ci, vp]
        L.dz_check.argtypes = [vp, vp]
        L.dz_set_option.argtypes = [vp, ci, ci]
        L.dz_qpacked_bytes.restype = ctypes.c_size_t
        L.dz_qpacked_bytes.argtypes = [ci, ci, ci, ci]
        L.dz_qpack_delta.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp, vp]
        L.dz_qunpack_delta.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, vp, vp, vp]
        L.dz_qsbmm.argtypes = [vp, vp, ctypes.POINTER(vp), ci, vp, vp, ci, ci, ci, ci, ci, ci, vp]
        L.dz_qlinear.argtypes = [vp, vp, vp, ctypes.POINTER(vp), ci, vp, vp, ci, ci, ci, ci, ci, vp]
        L.dz_merge_delta.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp]
        L.dz_compress_delta.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, vp, vp, vp]
        L.dz_lora_sbmm.argtypes = [vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ci, ci, vp, vp, ci, ci, ci, ci, vp]
        L.dz_probe_read.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.dz_probe_mfma.argtypes = [vp, ci, ctypes.POINTER(ctypes.c_double), vp]
        L.dz_linear_static.argtypes = [ci, vp, vp, ctypes.POINTER(vp), ci, vp, vp, ci, ci, ci, ci, ci, vp]
        i64p, i32p = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32)
        L.dz_cache_create.argtypes = [ctypes.POINTER(vp), ci, ci, ctypes.c_size_t]
        L.dz_cache_destroy.argtypes = [vp]
        L.dz_cache_acquire.argtypes = [vp, ci, i64p, ctypes.POINTER(vp), ctypes.c_size_t, ctypes.POINTER(vp), i32p, i32p,
                                       vp, i64p]
        L.dz_cache_wait.argtypes = [vp, ctypes.c_int64, vp]
        L.dz_cache_release.argtypes = [vp, ctypes.c_int64, vp]
        L.dz_cache_stats.argtypes = [vp, i64p, i64p, i64p]
        for name in SYMBOLS:
            getattr(L, name)
        _lib = L
    return _lib


def dz_strerror(rc: int) -> str:
    return lib().dz_strerror(rc).decode()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):          # a raw device address (e.g. from dz_cache_acquire)
        return t
    if not t.is_cuda:
        raise ValueError("libdz takes device tensors")
    if not t.is_contiguous():
        raise ValueError("libdz takes contiguous tensors")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def _raise(ctx, rc: int, where: str, check: bool):
    if rc != DZ_OK and check:
        detail = lib().dz_last_hip_error(ctx).decode() if rc == DZ_ERR_HIP and ctx else ""
        raise DzError(rc, where, detail)
    return rc


def dz_create(device: int = 0) -> int:
    h = ctypes.c_void_p()
    rc = lib().dz_create(ctypes.byref(h), device)
    if rc != DZ_OK:
        raise DzError(rc, "dz_create")
    return h.value


def dz_destroy(ctx: int) -> int:
    return lib().dz_destroy(ctx)


def dz_set_option(ctx, key: int, value: int, check=True) -> int:
    return _raise(ctx, lib().dz_set_option(ctx, int(key), int(value)), "dz_set_option", check)


def dz_probe_read(ctx, buf, nbytes: int, stream=None, check=True) -> int:
    return _raise(ctx, lib().dz_probe_read(ctx, _ptr(buf), int(nbytes), _stream(stream)), "dz_probe_read", check)


def dz_probe_mfma(ctx, iters: int, stream=None):
    """Returns the floating point operations the launch performs."""
    flops = ctypes.c_double()
    _raise(ctx, lib().dz_probe_mfma(ctx, int(iters), ctypes.byref(flops), _stream(stream)), "dz_probe_mfma", True)
    return float(flops.value)


def dz_packed_bytes(N: int, K: int, bits: int, group: int) -> int:
    return int(lib().dz_packed_bytes(N, K, bits, group))


def dz_pack_delta(ctx, codes, idx, scale, zero, N, K, bits, group, packed_out, stream=None, check=True) -> int:
    rc = lib().dz_pack_delta(ctx, _ptr(codes), _ptr(idx), _ptr(scale), _ptr(zero), N, K, bits, group,
                             _ptr(packed_out), _stream(stream))
    return _raise(ctx, rc, "dz_pack_delta", check)


def dz_unpack_delta(ctx, packed, N, K, bits, group, codes=None, idx=None, scale=None, zero=None, dense_f32=None,
                    stream=None, check=True) -> int:
    rc = lib().dz_unpack_delta(ctx, _ptr(packed), N, K, bits, group, _ptr(codes), _ptr(idx), _ptr(scale),
                               _ptr(zero), _ptr(dense_f32), _stream(stream))
    return _raise(ctx, rc, "dz_unpack_delta", check)


def dz_qpacked_bytes(N: int, K: int, bits: int, group: int) -> int:
    return int(lib().dz_qpacked_bytes(N, K, bits, group))


def dz_qpack_delta(ctx, codes, scale, zero, N, K, bits, group, packed_out, stream=None, check=True) -> int:
    rc = lib().dz_qpack_delta(ctx, _ptr(codes), _ptr(scale), _ptr(zero), N, K, bits, group, _ptr(packed_out), _stream(stream))
    return _raise(ctx, rc, "dz_qpack_delta", check)


def dz_qunpack_delta(ctx, packed, N, K, bits, group, codes=None, scale=None, zero=None, dense_f32=None, stream=None,
                     check=True) -> int:
    rc = lib().dz_qunpack_delta(ctx, _ptr(packed), N, K, bits, group, _ptr(codes), _ptr(scale), _ptr(zero), _ptr(dense_f32),
                                _stream(stream))
    return _raise(ctx, rc, "dz_qunpack_delta", check)


def dz_qsbmm(ctx, x, qpacked_deltas, token_to_delta, out, T, N, K, bits, group, accumulate=0, stream=None, check=True) -> int:
    arr, D = _ptr_array(qpacked_deltas)
    rc = lib().dz_qsbmm(ctx, _ptr(x), arr, D, _ptr(token_to_delta), _ptr(out), T, N, K, bits, group, int(accumulate),
                        _stream(stream))
    return _raise(ctx, rc, "dz_qsbmm", check)


def dz_qlinear(ctx, x, W, qpacked_deltas, token_to_delta, out, T, N, K, bits, group, stream=None, check=True) -> int:
    arr, D = _ptr_array(qpacked_deltas)
    rc = lib().dz_qlinear(ctx, _ptr(x), _ptr(W), arr, D, _ptr(token_to_delta), _ptr(out), T, N, K, bits, group, _stream(stream))
    return _raise(ctx, rc, "dz_qlinear", check)


def dz_merge_delta(ctx, W, packed, N, K, bits, group, merged_out, stream=None, check=True) -> int:
    rc = lib().dz_merge_delta(ctx, _ptr(W), _ptr(packed), N, K, bits, group, _ptr(merged_out), _stream(stream))
    return _raise(ctx, rc, "dz_merge_delta", check)


def dz_compress_delta(ctx, delta, N, K, bits, group, codes, idx, scale, zero, stream=None, check=True) -> int:
    rc = lib().dz_compress_delta(ctx, _ptr(delta), N, K, bits, group, _ptr(codes), _ptr(idx), _ptr(scale), _ptr(zero),
                                 _stream(stream))
    return _raise(ctx, rc, "dz_compress_delta", check)


def dz_lora_sbmm(ctx, x, A_list, B_list, rank, token_to_adapter, out, T, N, K, accumulate=0, stream=None, check=True) -> int:
    aarr, D = _ptr_array(A_list)
    barr, Db = _ptr_array(B_list)
    if D != Db:
        raise ValueError("dz_lora_sbmm: one A and one B per adapter")
    rc = lib().dz_lora_sbmm(ctx, _ptr(x), aarr, barr, D, int(rank), _ptr(token_to_adapter), _ptr(out), T, N, K,
                            int(accumulate), _stream(stream))
    return _raise(ctx, rc, "dz_lora_sbmm", check)


def dz_segment(ctx, token_to_delta, T, D, counts=None, offsets=None, perm=None, stream=None, check=True) -> int:
    rc = lib().dz_segment(ctx, _ptr(token_to_delta), T, D, _ptr(counts), _ptr(offsets), _ptr(perm), _stream(stream))
    return _raise(ctx, rc, "dz_segment", check)


def dz_base_gemm(ctx, x, W, out, T, N, K, stream=None, check=True) -> int:
    rc = lib().dz_base_gemm(ctx, _ptr(x), _ptr(W), _ptr(out), T, N, K, _stream(stream))
    return _raise(ctx, rc, "dz_base_gemm", check)


def _ptr_array(packed_deltas: Sequence):
    D = len(packed_deltas)
    arr = (ctypes.c_void_p * max(D, 1))()
    for i, p in enumerate(packed_deltas):
        arr[i] = p if isinstance(p, int) else _ptr(p)
    return arr, D


def dz_sbmm(ctx, x, packed_deltas, token_to_delta, out, T, N, K, bits, group, accumulate=0, stream=None,
            check=True) -> int:
    arr, D = _ptr_array(packed_deltas)
    rc = lib().dz_sbmm(ctx, _ptr(x), arr, D, _ptr(token_to_delta), _ptr(out), T, N, K, bits, group,
                       int(accumulate), _stream(stream))
    return _raise(ctx, rc, "dz_sbmm", check)


def dz_linear(ctx, x, W, packed_deltas, token_to_delta, out, T, N, K, bits, group, stream=None, check=True) -> int:
    arr, D = _ptr_array(packed_deltas)
    rc = lib().dz_linear(ctx, _ptr(x), _ptr(W), arr, D, _ptr(token_to_delta), _ptr(out), T, N, K, bits, group,
                         _stream(stream))
    return _raise(ctx, rc, "dz_linear", check)


def dz_linear_static(device: int, x, W, packed_deltas, token_to_delta, out, T, N, K, bits, group, stream=None,
                     check=True) -> int:
    arr, D = _ptr_array(packed_deltas)
    rc = lib().dz_linear_static(int(device), _ptr(x), _ptr(W), arr, D, _ptr(token_to_delta), _ptr(out), T, N, K, bits,
                                group, _stream(stream))
    return _raise(None, rc, "dz_linear_static", check)


def dz_linear_group(ctx, x, W_list, packed_deltas_list, token_to_delta, out_list, T, N_list, K, bits, group,
                    stream=None, check=True) -> int:
    """W_list, out_list, N_list: one entry per projection; packed_deltas_list: per projection, its D packed deltas."""
    P = len(W_list)
    D = len(packed_deltas_list[0]) if P else 0
    if any(len(d) != D for d in packed_deltas_list) or len(out_list) != P or len(N_list) != P:
        raise ValueError("dz_linear_group: every projection needs W, out, N and the same number of deltas")
    warr, _ = _ptr_array(W_list)
    oarr, _ = _ptr_array(out_list)
    darr, _ = _ptr_array([d for ds in packed_deltas_list for d in ds])
    narr = (ctypes.c_int * max(P, 1))(*[int(n) for n in N_list])
    rc = lib().dz_linear_group(ctx, _ptr(x), P, warr, darr, D, _ptr(token_to_delta), oarr, narr, T, K, bits, group,
                               _stream(stream))
    return _raise(ctx, rc, "dz_linear_group", check)


def dz_check(ctx, stream=None) -> int:
    return lib().dz_check(ctx, _stream(stream))


def dz_cache_create(device: int, slots: int, slot_bytes: int) -> int:
    """device < 0: a cache that only takes the decisions (no device memory, nothing copied)."""
    h = ctypes.c_void_p()
    rc = lib().dz_cache_create(ctypes.byref(h), int(device), int(slots), int(slot_bytes))
    if rc != DZ_OK:
        raise DzError(rc, "dz_cache_create")
    return h.value


def dz_cache_destroy(cache: int) -> int:
    return lib().dz_cache_destroy(cache)


def dz_cache_acquire(cache, keys: Sequence[int], host_blobs: Optional[Sequence[Optional[torch.Tensor]]], nbytes: int,
                     copy_stream=None, check=True):
    """Returns (rc, device addresses, slots, hits, ticket).  host_blobs: host tensors (pinned for overlap), one per
    key; None for a cache created with device < 0.  copy_stream: a torch stream or raw handle; None = the current
    stream."""
    n = len(keys)
    karr = (ctypes.c_int64 * max(n, 1))(*[int(k) for k in keys])
    harr = (ctypes.c_void_p * max(n, 1))()
    if host_blobs is not None:
        if len(host_blobs) != n:
            raise ValueError("dz_cache_acquire: one host blob per key")
        for i, t in enumerate(host_blobs):
            if t is not None:
                if t.is_cuda or not t.is_contiguous():
                    raise ValueError("dz_cache_acquire takes contiguous host tensors")
                harr[i] = t.data_ptr()
    darr = (ctypes.c_void_p * max(n, 1))()
    sarr = (ctypes.c_int32 * max(n, 1))()
    hitarr = (ctypes.c_int32 * max(n, 1))()
    ticket = ctypes.c_int64()
    rc = lib().dz_cache_acquire(cache, n, karr, harr if host_blobs is not None else None, int(nbytes), darr, sarr, hitarr,
                                _stream(copy_stream) if host_blobs is not None else None, ctypes.byref(ticket))
    if rc != DZ_OK and check:
        raise DzError(rc, "dz_cache_acquire")
    return (rc, [int(darr[i] or 0) for i in range(n)], [int(sarr[i]) for i in range(n)],
            [int(hitarr[i]) for i in range(n)], int(ticket.value))


def dz_cache_wait(cache, ticket: int, compute_stream=None) -> int:
    rc = lib().dz_cache_wait(cache, int(ticket), _stream(compute_stream))
    if rc != DZ_OK:
        raise DzError(rc, "dz_cache_wait")
    return rc


def dz_cache_release(cache, ticket: int, compute_stream=None) -> int:
    rc = lib().dz_cache_release(cache, int(ticket), _stream(compute_stream))
    if rc != DZ_OK:
        raise DzError(rc, "dz_cache_release")
    return rc


def dz_cache_stats(cache):
    h, m, e = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    rc = lib().dz_cache_stats(cache, ctypes.byref(h), ctypes.byref(m), ctypes.byref(e))
    if rc != DZ_OK:
        raise DzError(rc, "dz_cache_stats")
    return int(h.value), int(m.value), int(e.value)


class Context:
    """Owns a dz_ctx handle (context manager); `.h` is the handle the dz_* functions take."""

    def __init__(self, device: int = 0):
        self.h = dz_create(device)

    def set_option(self, key: int, value: int) -> int:
        return dz_set_option(self.h, key, value)

    def close(self):
        if self.h:
            dz_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
