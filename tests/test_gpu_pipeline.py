"""Layer pipeline for host-resident keys and values: meft_hostkv_stage requests a layer's K, V blocks ahead of its
forward (MEFT_FLAG_PRESTAGED), so that the transfer overlaps the previous layer's compute.  Every layer's results
are compared with the CPU oracle under the usual parity rules; the kernels and the data are those of the
unpipelined calls, so the results must also be bit-identical to them."""
import numpy as np
import pytest

from paper_2406_04984_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu

NAMES = ("block_idx", "idx", "act", "out", "dh", "dK_bits", "dV_bits", "touched")


def _layers(n, dtype="bf16", d=128):
    out = []
    for l in range(n):
        cfg = synth.small_case(T=150 + 10 * l, d=d, n_blocks=6, block_size=32, top_e=2, top_k=12, dtype=dtype,
                               seed=820 + l, host_kv=True)
        out.append(synth.make_inputs(cfg))
    return out


def _flags(B, *names):
    f = 0
    for n in names:
        f |= getattr(B, "MEFT_FLAG_" + n)
    return f


def test_prestaged_forward_and_kept_backward_are_bit_identical():
    import torch
    from paper_2406_04984_amd import binding as B
    t = _layers(1)[0]
    ref = P.run_gpu(t)
    layer = P.DeviceLayer(t)
    c = t.cfg
    staged = B.make_shape(c.T, c.d, c.n_blocks, c.block_size, c.top_e, c.top_k, c.dtype,
                          flags=_flags(B, "HOST_KV", "PRESTAGED", "KEEP_STAGED"))
    layer.fill_grad_sentinel()
    layer.route()
    B.meft_hostkv_stage(layer.shape, layer.block_idx, layer.K, layer.V, layer.ws)
    B.meft_sparse_fwd(staged, layer.h, layer.K, layer.V, layer.block_idx, layer.out, layer.idx, layer.act, layer.ws)
    B.meft_sparse_bwd(staged, layer.h, layer.K, layer.V, layer.idx, layer.act, layer.dOut, layer.dh, layer.dK, layer.dV,
                      layer.touched, layer.n_touched, layer.ws)
    got = layer.results()
    from oracle import oracle
    r, f, _ = oracle.layer(t, want_candidates=True)
    rep = P.compare(t, got, r, f, None)
    print(rep.summary(), flush=True)
    rep.assert_ok()
    for n in NAMES:
        assert (ref[n] == got[n]).all(), n


def test_three_layers_pipelined():
    from paper_2406_04984_amd import binding as B
    ts = _layers(3)
    refs = [P.run_gpu(t) for t in ts]
    layers = [P.DeviceLayer(t) for t in ts]          # every layer in flight has a workspace of its own
    shapes = []
    for t in ts:
        c = t.cfg
        shapes.append(B.make_shape(c.T, c.d, c.n_blocks, c.block_size, c.top_e, c.top_k, c.dtype,
                                   flags=_flags(B, "HOST_KV", "PRESTAGED", "KEEP_STAGED")))
    for la in layers:
        la.fill_grad_sentinel()
        la.route()
    B.meft_hostkv_stage(layers[0].shape, layers[0].block_idx, layers[0].K, layers[0].V, layers[0].ws)
    for l, la in enumerate(layers):
        if l + 1 < len(layers):                      # the next layer's transfer starts before this layer's compute
            nx = layers[l + 1]
            B.meft_hostkv_stage(nx.shape, nx.block_idx, nx.K, nx.V, nx.ws)
        B.meft_sparse_fwd(shapes[l], la.h, la.K, la.V, la.block_idx, la.out, la.idx, la.act, la.ws)
    for l in reversed(range(len(layers))):           # backward in reverse order, on the copies the forwards kept
        la = layers[l]
        B.meft_sparse_bwd(shapes[l], la.h, la.K, la.V, la.idx, la.act, la.dOut, la.dh, la.dK, la.dV, la.touched,
                          la.n_touched, la.ws)
    from oracle import oracle
    for l, la in enumerate(layers):
        got = la.results()
        r, f, _ = oracle.layer(ts[l], want_candidates=True)
        rep = P.compare(ts[l], got, r, f, None)
        print(f"layer {l}:", rep.summary(), flush=True)
        rep.assert_ok()
        for n in NAMES:
            assert (refs[l][n] == got[n]).all(), (l, n)


def test_prestaged_without_a_stage_call_is_refused():
    import torch
    from paper_2406_04984_amd import binding as B
    t = _layers(1)[0]
    layer = P.DeviceLayer(t)
    c = t.cfg
    staged = B.make_shape(c.T, c.d, c.n_blocks, c.block_size, c.top_e, c.top_k, c.dtype,
                          flags=_flags(B, "HOST_KV", "PRESTAGED"))
    layer.route()
    rc = B.meft_sparse_fwd(staged, layer.h, layer.K, layer.V, layer.block_idx, layer.out, layer.idx, layer.act,
                           layer.ws, check=False)
    assert rc == B.MEFT_ERR_INVALID_ARG
    torch.cuda.synchronize()
