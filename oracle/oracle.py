"""ctypes front end of the C oracle (oracle/meft_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.
It marshals numpy arrays into the C functions; the arithmetic is all in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "meft_oracle.c")
_LIB = os.path.join(_HERE, "libmeft_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP, -O2, no fast-math so sums stay in index order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d", "n_blocks", "block_size", "top_e", "top_k")]


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for fn in ("meft_oracle_route", "meft_oracle_fwd", "meft_oracle_bwd", "meft_oracle_apply",
                   "meft_oracle_threads", "meft_oracle_adam_rows", "meft_oracle_union_fwd",
                   "meft_oracle_union_bwd"):
            getattr(_lib, fn).restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_load().meft_oracle_threads())


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _shape(T, d, n_blocks, block_size, top_e, top_k):
    return _Shape(T, d, n_blocks, block_size, top_e, top_k)


@dataclass
class Route:
    block_idx: np.ndarray    # [T, e] int32, ordered by (score desc, block asc)
    block_score: np.ndarray  # [T, e] float64
    p: np.ndarray            # [T, n_blocks] float64, every router score


@dataclass
class Forward:
    out: np.ndarray          # [T, d] float64
    idx: np.ndarray          # [T, k] int32, ordered by (score desc, id asc)
    score: np.ndarray        # [T, k] float64, pre-activation
    act: np.ndarray          # [T, k] float64 = max(score, 0)
    next_score: np.ndarray   # [T] float64: the (k+1)-th candidate score, -inf if none
    cand_id: Optional[np.ndarray]     # [T, C] int32 ascending, or None
    cand_score: Optional[np.ndarray]  # [T, C] float64, or None


@dataclass
class Backward:
    dh: np.ndarray           # [T, d] float64
    dK: np.ndarray           # [N, d] (or [n_rows, d]) float64
    dV: np.ndarray
    touched: np.ndarray      # ascending int32


def route(h, Wg, top_e, bias=None) -> Route:
    h, hp = _f32(h)
    Wg, wp = _f32(Wg)
    T, d = h.shape
    B = Wg.shape[0]
    bias_a = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    s = _shape(T, d, B, 1, top_e, 1)
    bi = np.empty((T, top_e), np.int32)
    bsc = np.empty((T, top_e), np.float64)
    p = np.empty((T, B), np.float64)
    rc = _load().meft_oracle_route(ctypes.byref(s), hp, wp, _ptr(bias_a), _ptr(bi), _ptr(bsc), _ptr(p))
    if rc:
        raise ValueError(f"meft_oracle_route: bad arguments ({rc})")
    return Route(bi, bsc, p)


def forward(h, K, V, block_idx, block_size, top_k, want_candidates=False) -> Forward:
    h, hp = _f32(h)
    K, kp = _f32(K)
    V, vp = _f32(V)
    T, d = h.shape
    N = K.shape[0]
    block_idx = np.ascontiguousarray(block_idx, dtype=np.int32)
    e = block_idx.shape[1]
    assert N % block_size == 0 and V.shape == K.shape
    s = _shape(T, d, N // block_size, block_size, e, top_k)
    C = e * block_size
    out = np.empty((T, d), np.float64)
    idx = np.empty((T, top_k), np.int32)
    sc = np.empty((T, top_k), np.float64)
    nxt = np.empty((T,), np.float64)
    cid = np.empty((T, C), np.int32) if want_candidates else None
    csc = np.empty((T, C), np.float64) if want_candidates else None
    rc = _load().meft_oracle_fwd(ctypes.byref(s), hp, kp, vp, _ptr(block_idx), _ptr(out), _ptr(idx),
                                 _ptr(sc), _ptr(nxt), _ptr(cid), _ptr(csc))
    if rc:
        raise ValueError(f"meft_oracle_fwd: bad arguments ({rc})")
    return Forward(out, idx, sc, np.maximum(sc, 0.0), nxt, cid, csc)


def backward(h, K, V, idx, score, dOut, block_size, rows=None, want_dh=True) -> Backward:
    h, hp = _f32(h)
    K, kp = _f32(K)
    V, vp = _f32(V)
    dOut, gp = _f32(dOut)
    T, d = h.shape
    N = K.shape[0]
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    score = np.ascontiguousarray(score, dtype=np.float64)
    k = idx.shape[1]
    B = N // block_size
    # the backward only needs N and k; top_e is set so that the shape check passes
    e = min(B, max(1, -(-k // block_size)))
    s = _shape(T, d, B, block_size, e, k)
    dh = np.empty((T, d), np.float64) if want_dh else None
    rows_a = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    n_out = N if rows_a is None else rows_a.shape[0]
    dK = np.empty((n_out, d), np.float64)
    dV = np.empty((n_out, d), np.float64)
    touched = np.empty((max(1, min(N, T * k)),), np.int32)
    nt = ctypes.c_int32(0)
    rc = _load().meft_oracle_bwd(ctypes.byref(s), hp, kp, vp, _ptr(idx), _ptr(score), gp, _ptr(dh),
                                 _ptr(dK), _ptr(dV), _ptr(touched), ctypes.byref(nt), _ptr(rows_a),
                                 ctypes.c_int32(0 if rows_a is None else rows_a.shape[0]))
    if rc:
        raise ValueError(f"meft_oracle_bwd: bad arguments ({rc})")
    return Backward(dh, dK, dV, touched[: nt.value].copy())


def apply_selection(h, K, V, idx, block_size) -> np.ndarray:
    """out[t,:] = sum_i max(h[t].K[idx[t,i]], 0) V[idx[t,i],:] for selections given from outside."""
    h, hp = _f32(h)
    K, kp = _f32(K)
    V, vp = _f32(V)
    T, d = h.shape
    N = K.shape[0]
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    k = idx.shape[1]
    B = N // block_size
    e = min(B, max(1, -(-k // block_size)))
    s = _shape(T, d, B, block_size, e, k)
    out = np.empty((T, d), np.float64)
    rc = _load().meft_oracle_apply(ctypes.byref(s), hp, kp, vp, _ptr(idx), _ptr(out))
    if rc:
        raise ValueError(f"meft_oracle_apply: bad arguments ({rc})")
    return out


def layer(t, want_candidates=False, rows=None):
    """route -> forward -> backward on a synth.Tensors bundle."""
    c = t.cfg
    r = route(t.h, t.Wg, c.top_e, t.bias)
    f = forward(t.h, t.K, t.V, r.block_idx, c.block_size, c.top_k, want_candidates)
    b = backward(t.h, t.K, t.V, f.idx, f.score, t.dOut, c.block_size, rows=rows)
    return r, f, b


def adam_rows(w, g, m, v, touched, step, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One row-sparse Adam step; returns new (w, m, v) as float64 arrays, inputs are not modified."""
    w = np.array(w, dtype=np.float64, order="C")
    m = np.array(m, dtype=np.float64, order="C")
    v = np.array(v, dtype=np.float64, order="C")
    g = np.ascontiguousarray(g, dtype=np.float64)
    touched = np.ascontiguousarray(touched, dtype=np.int32)
    N, d = w.shape
    assert g.shape == w.shape == m.shape == v.shape
    fn = _load().meft_oracle_adam_rows
    fn.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p,
                   ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double, ctypes.c_double,
                   ctypes.c_double, ctypes.c_double, ctypes.c_int32]
    rc = fn(N, d, _ptr(touched), len(touched), _ptr(g), _ptr(w), _ptr(m), _ptr(v), lr, beta1, beta2, eps, step)
    if rc:
        raise ValueError(f"meft_oracle_adam_rows: bad arguments ({rc})")
    return w, m, v


def union_of(idx) -> np.ndarray:
    """S of Algorithm 1: the sorted unique neuron ids over all tokens' selections."""
    return np.unique(np.asarray(idx)).astype(np.int32)


def union_forward(h, K, V, S) -> np.ndarray:
    """Batch-union evaluation: every token uses every neuron of S.  Returns out [T, d] float64."""
    h, hp = _f32(h)
    K, kp = _f32(K)
    V, vp = _f32(V)
    S = np.ascontiguousarray(S, dtype=np.int32)
    T, d = h.shape
    out = np.empty((T, d), np.float64)
    rc = _load().meft_oracle_union_fwd(T, d, K.shape[0], hp, kp, vp, _ptr(S), len(S), _ptr(out))
    if rc:
        raise ValueError(f"meft_oracle_union_fwd: bad arguments ({rc})")
    return out


def union_backward(h, K, V, S, dOut, want_dh=True):
    """Returns (dh [T, d] or None, dK [len(S), d], dV [len(S), d]) float64; row i of dK, dV is neuron S[i]."""
    h, hp = _f32(h)
    K, kp = _f32(K)
    V, vp = _f32(V)
    g, gp = _f32(dOut)
    S = np.ascontiguousarray(S, dtype=np.int32)
    T, d = h.shape
    dh = np.empty((T, d), np.float64) if want_dh else None
    dK = np.empty((len(S), d), np.float64)
    dV = np.empty((len(S), d), np.float64)
    rc = _load().meft_oracle_union_bwd(T, d, K.shape[0], hp, kp, vp, _ptr(S), len(S), gp, _ptr(dh), _ptr(dK),
                                       _ptr(dV))
    if rc:
        raise ValueError(f"meft_oracle_union_bwd: bad arguments ({rc})")
    return dh, dK, dV
