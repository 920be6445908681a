"""Brute-force dense parallel adapter in numpy fp64 -- TEST INFRASTRUCTURE ONLY.

The adapter term of the paper's Parallel Adapter equation (Section 2):
out = ReLU(h W_A) W_B with W_A = K^T, W_B = V, and the gradients of
L = sum(out * dOut).  Written with library matmuls and masks, independently of
the C oracle, so that the oracle's dense special case can be pinned to it.
"""
import numpy as np


def dense_adapter(h, K, V):
    h = np.asarray(h, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    s = h @ K.T
    return np.maximum(s, 0.0) @ V


def dense_adapter_grads(h, K, V, dOut):
    h = np.asarray(h, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    dOut = np.asarray(dOut, np.float64)
    s = h @ K.T                    # [T, N]
    a = np.maximum(s, 0.0)
    dV = a.T @ dOut                # [N, d]
    g = dOut @ V.T                 # [T, N]
    ds = g * (s > 0.0)
    dK = ds.T @ h
    dh = ds @ K
    return dh, dK, dV


def masked_adapter(h, K, V, mask):
    """Dense adapter restricted to the (token, neuron) pairs where mask is True."""
    h = np.asarray(h, np.float64)
    s = h @ np.asarray(K, np.float64).T
    return (np.maximum(s, 0.0) * mask) @ np.asarray(V, np.float64)
