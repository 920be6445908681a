"""The three entry points recorded into a HIP graph (stream capture) and replayed: every replay, with eager work
of the program between the replays, gives bit for bit what the eager calls give.  Both formulations."""
import numpy as np
import pytest

from paper_2406_04984_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu

CASES = [dict(T=150, d=72, n_blocks=6, block_size=40, top_e=2, top_k=12, dtype="f32", seed=1201),
         dict(T=700, d=192, n_blocks=7, block_size=72, top_e=3, top_k=30, dtype="bf16", seed=1202),
         # unbalanced routing (blocks with a few tokens go to the per-pair kernels) and a backward on the forward's tables
         dict(T=600, d=256, n_blocks=24, block_size=64, top_e=2, top_k=16, dtype="bf16", seed=1203, zipf_s=1.5,
              reuse_fwd=True)]
NAMES = ("block_idx", "block_score", "idx", "act", "out", "dh", "dK_bits", "dV_bits", "touched")


@pytest.mark.parametrize("kw", CASES, ids=["gather_f32", "dense_bf16", "dense_bf16_skewed_reuse"])
def test_replays_of_a_captured_step_match_the_eager_step(kw):
    import torch
    t = synth.make_inputs(synth.small_case(**kw))
    ref = P.run_gpu(t)                       # eager
    layer = P.DeviceLayer(t)
    layer.fill_grad_sentinel()
    layer.step()                             # eager once more on these buffers: first-call set-up is not capturable
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):                # records on a side stream, which is the current stream inside
        layer.step()
    for rep in range(3):
        # eager work of the program between the replays: wipe every output and the workspace
        for x in (layer.block_idx, layer.idx, layer.touched, layer.n_touched):
            x.fill_(-1)
        for x in (layer.block_score, layer.act, layer.out, layer.dh):
            x.zero_()
        layer.fill_grad_sentinel()
        layer.ws.fill_(0xFF if rep % 2 == 0 else 0x00)
        torch.cuda.synchronize()
        g.replay()
        got = layer.results()
        for n in NAMES:
            assert np.array_equal(ref[n], got[n]), (rep, n)
