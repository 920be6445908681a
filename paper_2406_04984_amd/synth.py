"""Seeded synthetic inputs for the MEFT sparse-adapter layer.

This module only draws random numbers and rounds them to the storage type.  It
holds none of the method's arithmetic (no scores, no selection, no sums), so
the CPU oracle's tests and the GPU tests can both import it without sharing
anything the parity comparison depends on.

Every tensor comes from a counter-based generator (numpy's Philox) keyed by
(base seed of the configuration, stream id of the tensor), so any tensor can be
regenerated on its own.  Values of a bf16 configuration are rounded to bf16
(round to nearest, ties to even) on the host and returned both as float32
arrays holding exactly those values (for the oracle) and as uint16 bit
patterns (for the device), so both sides start from identical bits.

The paper fine-tunes LLaMA-7B (hidden size 4096) with up to 6144 key/value
pairs per layer and 64 activated pairs per token (Section 4, implementation
details; Table 2).  Its datasets and weights are not available, so the
configurations below stand in for that workload at the shapes the benchmark
names: normal hidden states with a few large "outlier" channels, normal keys,
values and router rows with variance 1/d.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import numpy as np

BASE_SEED = 20240604

# stream ids: one per tensor
_STREAM = {"h": 1, "Wg": 2, "K": 3, "V": 4, "dOut": 5, "outlier": 6, "bias": 7}


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    dtype: str            # "f32" or "bf16"
    T: int                # tokens
    d: int                # hidden size
    n_blocks: int         # number of key experts (neuron blocks)
    block_size: int       # neurons per block
    top_e: int            # blocks activated per token
    top_k: int            # neurons activated per token
    outlier_frac: float = 0.0   # fraction of channels of h that are scaled
    outlier_scale: float = 1.0
    zipf_s: float = 0.0         # >0: router bias -s*ln(rank), rank a seeded permutation
    host_kv: bool = False       # K, V (and dK, dV) live in pinned host memory
    keep_staged: bool = False   # with host_kv: the backward reuses the device copies the forward staged
    reuse_fwd: bool = False     # the backward takes the forward's entry grouping and activation rows from the workspace
    seed: int = BASE_SEED

    @property
    def N(self) -> int:
        return self.n_blocks * self.block_size

    @property
    def C(self) -> int:
        return self.top_e * self.block_size

    def replace(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, Config] = {
    "tiny_f32": Config("tiny_f32", "f32", 256, 128, 16, 128, 2, 32, seed=BASE_SEED + 1),
    "small_bf16": Config("small_bf16", "bf16", 2048, 1024, 64, 256, 4, 128,
                         outlier_frac=0.01, outlier_scale=8.0, reuse_fwd=True, seed=BASE_SEED + 2),
    "llama7b_bf16": Config("llama7b_bf16", "bf16", 8192, 4096, 64, 1024, 4, 256,
                           outlier_frac=0.005, outlier_scale=10.0, reuse_fwd=True, seed=BASE_SEED + 3),
    # the paper's ablation without key experts (Section 4.3, "MEFT w/o KE"): one block holds every neuron
    "noke_bf16": Config("noke_bf16", "bf16", 2048, 4096, 1, 65536, 1, 256,
                        outlier_frac=0.005, outlier_scale=10.0, seed=BASE_SEED + 6),
    "wide_bf16": Config("wide_bf16", "bf16", 4096, 4096, 256, 1024, 8, 512,
                        zipf_s=1.1, reuse_fwd=True, seed=BASE_SEED + 4),
    "llama7b_hostkv_bf16": Config("llama7b_hostkv_bf16", "bf16", 8192, 4096, 128, 1024, 4, 256,
                                  outlier_frac=0.005, outlier_scale=10.0, host_kv=True, keep_staged=True,
                                  reuse_fwd=True, seed=BASE_SEED + 5),
}


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); returns uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to the float32 holding the same value."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def _normal(seed: int, stream: int, shape, std: float, chunk_rows: int = 8192) -> np.ndarray:
    g = _rng(seed, stream)
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(shape[0], -1) if len(shape) > 1 else out.reshape(-1, 1)
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        blk = g.standard_normal((r1 - r0, flat.shape[1]), dtype=np.float32)
        if std != 1.0:
            blk *= np.float32(std)
        flat[r0:r1] = blk
    return out


@dataclasses.dataclass
class Tensors:
    """Inputs of one layer.  Float arrays hold exactly the stored values."""
    cfg: Config
    h: np.ndarray                 # [T, d] float32
    Wg: np.ndarray                # [n_blocks, d] float32
    K: np.ndarray                 # [N, d] float32
    V: np.ndarray                 # [N, d] float32
    dOut: np.ndarray              # [T, d] float32
    bias: Optional[np.ndarray]    # [n_blocks] float32 or None
    outlier_channels: np.ndarray  # int64 ids of the scaled channels of h

    def storage(self, name: str) -> np.ndarray:
        """The array as the device stores it: float32, or uint16 bf16 bits."""
        a = getattr(self, name)
        if self.cfg.dtype == "bf16" and name in ("h", "Wg", "K", "V", "dOut"):
            return bf16_round(a)
        return a


def make_tensor(cfg: Config, name: str) -> np.ndarray:
    """One input tensor of `cfg` as float32 holding the stored (rounded) values."""
    d = cfg.d
    wstd = 1.0 / math.sqrt(d)
    if name == "h":
        a = _normal(cfg.seed, _STREAM["h"], (cfg.T, d), 1.0)
        ch = outlier_channels(cfg)
        if ch.size:
            a[:, ch] *= np.float32(cfg.outlier_scale)
    elif name == "dOut":
        a = _normal(cfg.seed, _STREAM["dOut"], (cfg.T, d), 1.0)
    elif name == "Wg":
        a = _normal(cfg.seed, _STREAM["Wg"], (cfg.n_blocks, d), wstd)
    elif name == "K":
        a = _normal(cfg.seed, _STREAM["K"], (cfg.N, d), wstd)
    elif name == "V":
        a = _normal(cfg.seed, _STREAM["V"], (cfg.N, d), wstd)
    else:
        raise KeyError(name)
    if cfg.dtype == "bf16":
        a = bf16_to_f32(bf16_round(a))
    return a


def outlier_channels(cfg: Config) -> np.ndarray:
    n = int(round(cfg.outlier_frac * cfg.d))
    if n <= 0:
        return np.zeros(0, dtype=np.int64)
    g = _rng(cfg.seed, _STREAM["outlier"])
    return np.sort(g.permutation(cfg.d)[:n]).astype(np.int64)


def router_bias(cfg: Config) -> Optional[np.ndarray]:
    """Zipf-like block popularity: bias[b] = -s * ln(rank_b), rank a seeded permutation of 1..B."""
    if cfg.zipf_s <= 0.0:
        return None
    g = _rng(cfg.seed, _STREAM["bias"])
    rank = g.permutation(cfg.n_blocks).astype(np.float64) + 1.0
    return (-cfg.zipf_s * np.log(rank)).astype(np.float32)


def make_inputs(cfg: Config) -> Tensors:
    return Tensors(cfg=cfg,
                   h=make_tensor(cfg, "h"), Wg=make_tensor(cfg, "Wg"),
                   K=make_tensor(cfg, "K"), V=make_tensor(cfg, "V"),
                   dOut=make_tensor(cfg, "dOut"), bias=router_bias(cfg),
                   outlier_channels=outlier_channels(cfg))


def small_case(T: int, d: int, n_blocks: int, block_size: int, top_e: int, top_k: int,
               dtype: str = "f32", seed: int = 7, **kw) -> Config:
    """An ad-hoc configuration for unit tests."""
    return Config(f"case_T{T}_d{d}_B{n_blocks}x{block_size}_e{top_e}_k{top_k}_{dtype}_s{seed}",
                  dtype, T, d, n_blocks, block_size, top_e, top_k, seed=seed, **kw)


@dataclasses.dataclass
class AdamCase:
    """Inputs of one optimizer step on a parameter matrix: weights, gradient, both moments, the rows to update.
    Float arrays hold exactly the stored values (bf16-representable where dtype is "bf16")."""
    dtype: str
    W: np.ndarray         # [N, d] float32
    G: np.ndarray         # [N, d] float32
    m: np.ndarray         # [N, d] float32
    v: np.ndarray         # [N, d] float32, >= 0
    touched: np.ndarray   # ascending int32 row ids


def adam_case(N: int, d: int, n_touched: int, dtype: str = "bf16", seed: int = 11, grad_std: float = 0.05) -> AdamCase:
    """Weights ~ N(0, 1/d) like the keys and values, gradient ~ N(0, grad_std^2), moments of the size a few
    earlier steps would have left, and a seeded subset of `n_touched` rows."""
    W = _normal(seed, 101, (N, d), 1.0 / math.sqrt(d))
    G = _normal(seed, 102, (N, d), grad_std)
    m = _normal(seed, 103, (N, d), 0.3 * grad_std)
    v = np.square(_normal(seed, 104, (N, d), 0.2 * grad_std)) + np.float32((0.1 * grad_std) ** 2)
    if dtype == "bf16":
        W, G = bf16_to_f32(bf16_round(W)), bf16_to_f32(bf16_round(G))
    touched = np.sort(_rng(seed, 105).choice(N, size=n_touched, replace=False)).astype(np.int32)
    return AdamCase(dtype, W, G, m, v, touched)
