"""Thin ctypes binding of libmeft's C ABI (include/meft.h): argument marshalling only.

Function names and argument order follow the header.  Tensors are torch tensors on the GPU (the
binding takes their `data_ptr()`); torch is used for device memory and streams and for nothing
else.  There is no CPU fallback: if the library has not been built, importing this module fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmeft.so")

MEFT_OK, MEFT_ERR_INVALID_ARG, MEFT_ERR_UNSUPPORTED, MEFT_ERR_WORKSPACE, MEFT_ERR_DEVICE = range(5)
MEFT_F32, MEFT_BF16 = 0, 1
MEFT_FLAG_HOST_KV = 1
MEFT_FLAG_KEEP_STAGED = 2
MEFT_FLAG_PRESTAGED = 4
MEFT_FLAG_REUSE_FWD = 8

EXPORTS = ("meft_workspace_bytes", "meft_check_shape", "meft_status_string", "meft_route",
           "meft_sparse_fwd", "meft_sparse_bwd", "meft_profile_enable", "meft_profile_read",
           "meft_probe_copy", "meft_probe_mfma", "meft_adam_rows", "meft_last_device_error",
           "meft_union_workspace_bytes", "meft_union_fwd", "meft_union_bwd", "meft_hostkv_stage",
           "meft_debug_global_loads", "meft_route_static")
MEFT_ROUTE_STATIC_BYTES = 16 << 20


class MeftShape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d", ctypes.c_int32), ("N", ctypes.c_int32),
                ("n_blocks", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("top_e", ctypes.c_int32), ("top_k", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("activation", ctypes.c_int32), ("flags", ctypes.c_uint32)]


class MeftAdam(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("step", ctypes.c_int32)]


class MeftError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        detail = f": {last_device_error()}" if status == MEFT_ERR_DEVICE else ""
        super().__init__(f"{fn}: {status_string(status)} (status {status}){detail}")


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2406_04984_amd.build` "
                      "(there is no fallback path)")
# The library must bind to the HIP runtime that the caller's tensors and streams come from.  PyTorch ships its
# own copy; loading it first makes the loader resolve libmeft.so's dependency to that same copy (two runtimes
# in one process do not see each other's device memory, and the second one may not find the device at all).
import torch  # noqa: E402,F401

_lib = ctypes.CDLL(LIB_PATH)

_vp, _sz, _i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
_shape_p = ctypes.POINTER(MeftShape)
_lib.meft_workspace_bytes.restype = _sz
_lib.meft_workspace_bytes.argtypes = [_shape_p]
_lib.meft_check_shape.restype = ctypes.c_int
_lib.meft_check_shape.argtypes = [_shape_p]
_lib.meft_status_string.restype = ctypes.c_char_p
_lib.meft_status_string.argtypes = [ctypes.c_int]
_lib.meft_route.restype = ctypes.c_int
_lib.meft_route.argtypes = [_shape_p, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.meft_route_static.restype = ctypes.c_int
_lib.meft_route_static.argtypes = [_shape_p, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.meft_sparse_fwd.restype = ctypes.c_int
_lib.meft_sparse_fwd.argtypes = [_shape_p, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.meft_sparse_bwd.restype = ctypes.c_int
_lib.meft_sparse_bwd.argtypes = [_shape_p, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.meft_adam_rows.restype = ctypes.c_int
_lib.meft_adam_rows.argtypes = [_shape_p, ctypes.POINTER(MeftAdam), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.meft_union_workspace_bytes.restype = _sz
_lib.meft_union_workspace_bytes.argtypes = [_shape_p]
_lib.meft_union_fwd.restype = ctypes.c_int
_lib.meft_union_fwd.argtypes = [_shape_p, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.meft_union_bwd.restype = ctypes.c_int
_lib.meft_union_bwd.argtypes = [_shape_p, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.meft_hostkv_stage.restype = ctypes.c_int
_lib.meft_hostkv_stage.argtypes = [_shape_p, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.meft_last_device_error.restype = ctypes.c_char_p
_lib.meft_last_device_error.argtypes = []
_lib.meft_probe_copy.restype = ctypes.c_int
_lib.meft_probe_copy.argtypes = [_vp, _vp, _sz, _vp]
_lib.meft_probe_mfma.restype = ctypes.c_int
_lib.meft_probe_mfma.argtypes = [_vp, ctypes.c_int, ctypes.c_int, _vp]
_lib.meft_profile_enable.restype = None
_lib.meft_profile_enable.argtypes = [ctypes.c_int]
_lib.meft_debug_global_loads.restype = None
_lib.meft_debug_global_loads.argtypes = [ctypes.c_int]
_lib.meft_profile_read.restype = ctypes.c_int
_lib.meft_profile_read.argtypes = [ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(_i32),
                                   ctypes.POINTER(ctypes.c_float), ctypes.c_int]


def make_shape(T, d, n_blocks, block_size, top_e, top_k, dtype, flags=0, N=None, activation=0) -> MeftShape:
    dt = {"f32": MEFT_F32, "bf16": MEFT_BF16}.get(dtype, dtype)
    return MeftShape(T, d, n_blocks * block_size if N is None else N, n_blocks, block_size, top_e, top_k,
                     dt, activation, flags)


def last_device_error() -> str:
    return _lib.meft_last_device_error().decode()


def status_string(status: int) -> str:
    return _lib.meft_status_string(int(status)).decode()


def meft_check_shape(shape: MeftShape) -> int:
    return int(_lib.meft_check_shape(ctypes.byref(shape)))


def meft_workspace_bytes(shape: MeftShape) -> int:
    return int(_lib.meft_workspace_bytes(ctypes.byref(shape)))


def _p(x):
    """Device (or pinned host) address of a torch tensor, a raw integer address, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def meft_route(shape, h, Wg, bias, block_idx, block_score, ws, stream=None, check=True) -> int:
    wp, wb = _ws(ws)
    rc = _lib.meft_route(ctypes.byref(shape), _p(h), _p(Wg), _p(bias), _p(block_idx), _p(block_score),
                         wp, wb, _stream(stream))
    if check and rc:
        raise MeftError("meft_route", rc)
    return rc


def meft_route_static(shape, h, Wg, bias, block_idx, block_score, stream=None, check=True) -> int:
    rc = _lib.meft_route_static(ctypes.byref(shape), _p(h), _p(Wg), _p(bias), _p(block_idx), _p(block_score),
                                _stream(stream))
    if check and rc:
        raise MeftError("meft_route_static", rc)
    return rc


def meft_sparse_fwd(shape, h, K, V, block_idx, out, idx, act, ws, stream=None, check=True) -> int:
    wp, wb = _ws(ws)
    rc = _lib.meft_sparse_fwd(ctypes.byref(shape), _p(h), _p(K), _p(V), _p(block_idx), _p(out), _p(idx),
                              _p(act), wp, wb, _stream(stream))
    if check and rc:
        raise MeftError("meft_sparse_fwd", rc)
    return rc


def meft_sparse_bwd(shape, h, K, V, idx, act, dOut, dh, dK, dV, touched, n_touched, ws, stream=None,
                    check=True) -> int:
    wp, wb = _ws(ws)
    rc = _lib.meft_sparse_bwd(ctypes.byref(shape), _p(h), _p(K), _p(V), _p(idx), _p(act), _p(dOut), _p(dh),
                              _p(dK), _p(dV), _p(touched), _p(n_touched), wp, wb, _stream(stream))
    if check and rc:
        raise MeftError("meft_sparse_bwd", rc)
    return rc


def meft_hostkv_stage(shape, block_idx, K, V, ws, stream=None, check=True) -> int:
    wp, wb = _ws(ws)
    rc = _lib.meft_hostkv_stage(ctypes.byref(shape), _p(block_idx), _p(K), _p(V), wp, wb, _stream(stream))
    if check and rc:
        raise MeftError("meft_hostkv_stage", rc)
    return rc


def meft_union_workspace_bytes(shape: MeftShape) -> int:
    return int(_lib.meft_union_workspace_bytes(ctypes.byref(shape)))


def meft_union_fwd(shape, h, K, V, idx, out, S, n_S, ws, stream=None, check=True) -> int:
    wp, wb = _ws(ws)
    rc = _lib.meft_union_fwd(ctypes.byref(shape), _p(h), _p(K), _p(V), _p(idx), _p(out), _p(S), _p(n_S), wp, wb,
                             _stream(stream))
    if check and rc:
        raise MeftError("meft_union_fwd", rc)
    return rc


def meft_union_bwd(shape, h, K, V, S, n_S, dOut, dh, dK, dV, ws, stream=None, check=True) -> int:
    wp, wb = _ws(ws)
    rc = _lib.meft_union_bwd(ctypes.byref(shape), _p(h), _p(K), _p(V), _p(S), _p(n_S), _p(dOut), _p(dh), _p(dK),
                             _p(dV), wp, wb, _stream(stream))
    if check and rc:
        raise MeftError("meft_union_bwd", rc)
    return rc


def meft_adam_rows(shape, hp: MeftAdam, W, G, m, v, master, touched, n_touched, stream=None, check=True) -> int:
    rc = _lib.meft_adam_rows(ctypes.byref(shape), ctypes.byref(hp) if hp is not None else None, _p(W), _p(G),
                             _p(m), _p(v), _p(master), _p(touched), _p(n_touched), _stream(stream))
    if check and rc:
        raise MeftError("meft_adam_rows", rc)
    return rc


def meft_probe_copy(dst, src, nbytes: int, stream=None, check=True) -> int:
    rc = _lib.meft_probe_copy(_p(dst), _p(src), nbytes, _stream(stream))
    if check and rc:
        raise MeftError("meft_probe_copy", rc)
    return rc


def meft_probe_mfma(out, workgroups: int, iters: int, stream=None, check=True) -> int:
    rc = _lib.meft_probe_mfma(_p(out), workgroups, iters, _stream(stream))
    if check and rc:
        raise MeftError("meft_probe_mfma", rc)
    return rc


def meft_debug_global_loads(on: bool) -> None:
    _lib.meft_debug_global_loads(1 if on else 0)


def meft_profile_enable(on: bool) -> None:
    _lib.meft_profile_enable(1 if on else 0)


def meft_profile_read(cap: int = 64):
    """[(kernel name, launches, total milliseconds)] since profiling was enabled."""
    names = (ctypes.c_char_p * cap)()
    launches = (_i32 * cap)()
    ms = (ctypes.c_float * cap)()
    n = _lib.meft_profile_read(names, launches, ms, cap)
    return [(names[i].decode(), int(launches[i]), float(ms[i])) for i in range(n)]
