"""Device buffers of one layer and the three ABI calls on them.

Used by the benchmark and by the GPU tests.  PyTorch is here for device memory and the stream only;
every step of the layer runs in libmeft through paper_2406_04984_amd.binding.  This module computes
nothing of the method and knows nothing of the CPU oracle.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from . import synth

SENTINEL_BF16 = 0x7FC1      # a NaN pattern no computation produces
SENTINEL_F32 = 0x7FC00001


def _torch():
    import torch
    return torch


def to_device(t: synth.Tensors, name: str):
    torch = _torch()
    a = t.storage(name)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_pinned(t: synth.Tensors, name: str):
    torch = _torch()
    a = t.storage(name)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).pin_memory()
    return torch.from_numpy(a).pin_memory()


def to_host(x) -> np.ndarray:
    torch = _torch()
    if x.dtype == torch.bfloat16:
        return x.float().cpu().numpy()
    return x.cpu().numpy()


class DeviceLayer:
    """Device buffers of one layer and the three ABI calls on them."""

    def __init__(self, t: synth.Tensors, binding=None):
        torch = _torch()
        if binding is None:
            from . import binding
        self.B = binding
        c = t.cfg
        self.cfg = c
        self.shape = binding.make_shape(c.T, c.d, c.n_blocks, c.block_size, c.top_e, c.top_k, c.dtype,
                                        flags=(binding.MEFT_FLAG_HOST_KV if c.host_kv else 0) |
                                              (binding.MEFT_FLAG_KEEP_STAGED if c.host_kv and c.keep_staged else 0) |
                                              (binding.MEFT_FLAG_REUSE_FWD if c.reuse_fwd else 0))
        self.dt = torch.bfloat16 if c.dtype == "bf16" else torch.float32
        dev = "cuda"
        self.h, self.Wg, self.dOut = (to_device(t, n) for n in ("h", "Wg", "dOut"))
        if c.host_kv:   # keys and values (and their gradients) stay in pinned host memory
            self.K, self.V = (to_pinned(t, n) for n in ("K", "V"))
        else:
            self.K, self.V = (to_device(t, n) for n in ("K", "V"))
        self.bias = None if t.bias is None else torch.from_numpy(t.bias).cuda()
        T, d, N, e, k = c.T, c.d, c.N, c.top_e, c.top_k
        self.block_idx = torch.full((T, e), -1, dtype=torch.int32, device=dev)
        self.block_score = torch.zeros((T, e), dtype=torch.float32, device=dev)
        self.out = torch.zeros((T, d), dtype=self.dt, device=dev)
        self.idx = torch.full((T, k), -1, dtype=torch.int32, device=dev)
        self.act = torch.zeros((T, k), dtype=torch.float32, device=dev)
        self.dh = torch.zeros((T, d), dtype=self.dt, device=dev)
        if c.host_kv:
            self.dK = torch.zeros((N, d), dtype=self.dt).pin_memory()
            self.dV = torch.zeros((N, d), dtype=self.dt).pin_memory()
        else:
            self.dK = torch.zeros((N, d), dtype=self.dt, device=dev)
            self.dV = torch.zeros((N, d), dtype=self.dt, device=dev)
        self.touched = torch.full((max(1, min(N, T * k)),), -1, dtype=torch.int32, device=dev)
        self.n_touched = torch.full((1,), -1, dtype=torch.int32, device=dev)
        nbytes = binding.meft_workspace_bytes(self.shape)
        assert nbytes > 0, "shape rejected"
        self.ws = torch.empty((nbytes,), dtype=torch.uint8, device=dev)

    def fill_grad_sentinel(self):
        torch = _torch()
        if self.dt == torch.bfloat16:
            self.dK.view(torch.int16).fill_(SENTINEL_BF16)
            self.dV.view(torch.int16).fill_(SENTINEL_BF16)
        else:
            self.dK.view(torch.int32).fill_(SENTINEL_F32)
            self.dV.view(torch.int32).fill_(SENTINEL_F32)

    def route(self):
        self.B.meft_route(self.shape, self.h, self.Wg, self.bias, self.block_idx, self.block_score, self.ws)

    def fwd(self):
        self.B.meft_sparse_fwd(self.shape, self.h, self.K, self.V, self.block_idx, self.out, self.idx,
                               self.act, self.ws)

    def bwd(self, want_dh=True):
        self.B.meft_sparse_bwd(self.shape, self.h, self.K, self.V, self.idx, self.act, self.dOut,
                               self.dh if want_dh else None, self.dK, self.dV, self.touched, self.n_touched,
                               self.ws)

    def step(self):
        self.route()
        self.fwd()
        self.bwd()

    def block_loads(self) -> np.ndarray:
        """Tokens routed to each block by the last route() (the realised load histogram)."""
        torch = _torch()
        torch.cuda.synchronize()
        return torch.bincount(self.block_idx.flatten().long(), minlength=self.cfg.n_blocks).cpu().numpy()

    def results(self, rows: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
        """Copies results to the host.  `rows`: fetch dK / dV only for these neuron ids (large shapes);
        the sentinel checks over all rows are evaluated where the gradients live either way."""
        torch = _torch()
        torch.cuda.synchronize()
        nt = int(self.n_touched.item())
        bf = self.dt == torch.bfloat16
        ibits = torch.int16 if bf else torch.int32
        sent = SENTINEL_BF16 if bf else SENTINEL_F32
        sent_signed = sent - (1 << 16) if (bf and sent >= (1 << 15)) else sent
        r = dict(block_idx=to_host(self.block_idx), block_score=to_host(self.block_score),
                 out=to_host(self.out), idx=to_host(self.idx), act=to_host(self.act), dh=to_host(self.dh),
                 touched=to_host(self.touched)[:max(nt, 0)], n_touched=nt)
        for name, x in (("dK", self.dK), ("dV", self.dV)):
            is_s = x.view(ibits) == sent_signed
            r[name + "_row_all_sentinel"] = is_s.all(dim=1).cpu().numpy()
            r[name + "_row_any_sentinel"] = is_s.any(dim=1).cpu().numpy()
            del is_s
            if rows is None:
                r[name] = to_host(x)
                r[name + "_bits"] = x.view(ibits).cpu().numpy()
            else:
                sel = torch.from_numpy(np.asarray(rows, np.int64)).to(x.device)
                r[name] = to_host(x.index_select(0, sel))
        r["grad_rows"] = None if rows is None else np.asarray(rows, np.int64)
        return r
