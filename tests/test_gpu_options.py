"""The optional arguments and the calling conventions of the three main entry points, on both formulations
(per-pair gather: f32, block-dense matrix-core: bf16): nullable outputs, a workspace full of garbage, a caller's
stream, one workspace shared by different shapes.  Everything is compared bit for bit with a plain run."""
import numpy as np
import pytest

from paper_2406_04984_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu

CASES = [dict(T=150, d=72, n_blocks=6, block_size=40, top_e=2, top_k=12, dtype="f32", seed=1101),
         dict(T=300, d=192, n_blocks=7, block_size=72, top_e=3, top_k=30, dtype="bf16", seed=1102)]
NAMES = ("block_idx", "block_score", "idx", "act", "out", "dh", "dK_bits", "dV_bits", "touched")


def _same(a, b, names=NAMES):
    for n in names:
        assert np.array_equal(a[n], b[n]), n


@pytest.mark.parametrize("kw", CASES, ids=["gather_f32", "dense_bf16"])
def test_workspace_contents_do_not_matter(kw):
    import torch
    t = synth.make_inputs(synth.small_case(**kw))
    ref = P.run_gpu(t)
    layer = P.DeviceLayer(t)
    layer.fill_grad_sentinel()
    for call in (layer.route, layer.fwd, layer.bwd):
        layer.ws.fill_(0xFF)          # NaN patterns and negative integers everywhere
        call()
    _same(ref, layer.results())
    for call in (layer.route, layer.fwd, layer.bwd):
        layer.ws.fill_(0x00)
        call()
    _same(ref, layer.results())


@pytest.mark.parametrize("kw", CASES, ids=["gather_f32", "dense_bf16"])
def test_nullable_outputs(kw):
    import torch
    t = synth.make_inputs(synth.small_case(**kw))
    ref = P.run_gpu(t)
    layer = P.DeviceLayer(t)
    layer.fill_grad_sentinel()
    B = layer.B
    B.meft_route(layer.shape, layer.h, layer.Wg, layer.bias, layer.block_idx, None, layer.ws)   # no block scores
    layer.fwd()
    layer.dh.fill_(7.0)
    layer.bwd(want_dh=False)                                                                     # no dh
    got = layer.results()
    _same(ref, got, [n for n in NAMES if n not in ("block_score", "dh")])
    assert bool((layer.dh == 7.0).all()), "dh was written although it was not asked for"


@pytest.mark.parametrize("kw", CASES, ids=["gather_f32", "dense_bf16"])
def test_on_a_stream_of_the_caller(kw):
    import torch
    t = synth.make_inputs(synth.small_case(**kw))
    ref = P.run_gpu(t)
    layer = P.DeviceLayer(t)
    layer.fill_grad_sentinel()
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):       # the binding passes torch's current stream
        layer.step()
    st.synchronize()
    _same(ref, layer.results())


def test_one_workspace_for_different_shapes():
    import torch
    ts = [synth.make_inputs(synth.small_case(**kw)) for kw in CASES]
    refs = [P.run_gpu(t) for t in ts]
    layers = [P.DeviceLayer(t) for t in ts]
    big = max(layers, key=lambda la: la.ws.numel()).ws
    for la in layers:
        la.ws = big
        la.fill_grad_sentinel()
    for _ in range(2):
        for la, ref in zip(layers, refs):
            la.step()
            _same(ref, la.results())


def test_everything_selected_on_the_matrix_core_path():
    """top_e = n_blocks, top_k = N in bf16: the block-dense kernels compute the dense parallel adapter (Section 2)."""
    from oracle import dense_ref
    cfg = synth.small_case(T=90, d=128, n_blocks=4, block_size=32, top_e=4, top_k=128, dtype="bf16", seed=1103)
    t = synth.make_inputs(cfg)
    g = P.run_gpu(t)
    assert (g["idx"] == np.arange(cfg.N)[None, :]).all()
    assert P.rel_l2(g["out"], dense_ref.dense_adapter(t.h, t.K, t.V)) <= 2e-2
    dh, dK, dV = dense_ref.dense_adapter_grads(t.h, t.K, t.V, t.dOut)
    assert P.rel_l2(g["dh"], dh) <= 2e-2 and P.rel_l2(g["dK"], dK) <= 2e-2 and P.rel_l2(g["dV"], dV) <= 2e-2


def test_global_load_kernels_match_the_buffer_load_kernels():
    """The matrix-core kernels load operands below 4 GB through buffer resources and larger ones through global
    pointers; meft_debug_global_loads(1) selects the latter at any size.  Both give the same bits."""
    from paper_2406_04984_amd import binding as B
    t = synth.make_inputs(synth.small_case(**CASES[1]))
    ref = P.run_gpu(t)
    B.meft_debug_global_loads(True)
    try:
        got = P.run_gpu(t)
    finally:
        B.meft_debug_global_loads(False)
    _same(ref, got)


def test_measurement_probes_run():
    """The streaming-copy probe copies; the matrix-instruction probe fills its output with finite sums."""
    import torch
    from paper_2406_04984_amd import binding as B
    a = torch.arange(1 << 16, dtype=torch.int32, device="cuda")
    b = torch.zeros_like(a)
    B.meft_probe_copy(b, a, a.numel() * 4)
    out = torch.full((8 * 256,), float("nan"), dtype=torch.float32, device="cuda")
    B.meft_probe_mfma(out, 8, 16)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    assert bool(torch.isfinite(out).all()) and bool((out != 0).any())


@pytest.mark.parametrize("kw", CASES + [dict(T=333, d=192, n_blocks=5, block_size=72, top_e=2, top_k=19, dtype="bf16",
                                             seed=1104),
                                        dict(T=200, d=128, n_blocks=12, block_size=64, top_e=8, top_k=70, dtype="bf16",
                                             seed=1105)],
                         ids=["gather_f32", "dense_bf16", "dense_ragged", "dense_top_e_8"])
def test_backward_on_the_forwards_tables_gives_the_same_bits(kw):
    """MEFT_FLAG_REUSE_FWD: the backward takes the grouping of the entries and the activation rows from the
    workspace, where the forward of the step left them, instead of rebuilding both from (idx, act).  Two steps in
    a row, each bit-identical to the plain run; the per-pair formulation ignores the flag."""
    t = synth.make_inputs(synth.small_case(**kw))
    ref = P.run_gpu(t)
    tr = synth.Tensors(t.cfg.replace(reuse_fwd=True), t.h, t.Wg, t.K, t.V, t.dOut, t.bias, t.outlier_channels)
    layer = P.DeviceLayer(tr)
    for _ in range(2):
        layer.fill_grad_sentinel()
        layer.ws.fill_(0xFF)
        layer.step()
        _same(ref, layer.results())


def test_backward_on_the_forwards_tables_when_a_routed_block_gives_no_neuron():
    """A token routed to a block none of whose neurons makes its top-k: the forward's grouping holds an entry that a
    grouping rebuilt from idx does not have; its activation row is all zero and changes no result."""
    cfg = synth.small_case(T=120, d=128, n_blocks=6, block_size=64, top_e=3, top_k=20, dtype="bf16", seed=1106)
    t = synth.make_inputs(cfg)
    t.K[3 * 64:4 * 64] *= 1e-3            # block 3's scores are tiny: routed to, never selected from
    t.bias = np.array([0, 0, 0, 50, 0, 0], np.float32)
    ref = P.run_gpu(t)
    assert (ref["block_idx"] == 3).any(axis=1).all() and not ((ref["idx"] >= 192) & (ref["idx"] < 256)).any()
    tr = synth.Tensors(cfg.replace(reuse_fwd=True), t.h, t.Wg, t.K, t.V, t.dOut, t.bias, t.outlier_channels)
    _same(ref, P.run_gpu(tr))
