"""Skewed loads on the per-pair kernels (Section 3.1, last paragraph: the gradient of a neuron is the sum over the
tokens that activated it): neurons that hundreds or thousands of tokens select.  Their pairs are put in token order
by a sort in LDS and summed in chunks of 256 by several workgroups, the chunk sums added in chunk order: same
parity rules as everywhere else, and the same bits from run to run."""
import numpy as np
import pytest

from paper_2406_04984_amd import synth
from tests import parity as P

pytestmark = pytest.mark.gpu


def _hot_neurons(cfg, hot, seed):
    """Inputs in which the neurons `hot` = {id: strength} score high for every token: the hidden states share a
    common direction u, those keys are multiples of u, and a router bias sends every token to their blocks."""
    t = synth.make_inputs(cfg)
    rng = np.random.default_rng(seed)
    u = rng.standard_normal(cfg.d).astype(np.float32)
    u /= np.linalg.norm(u)
    t.h += (3.0 * u)[None, :]
    bias = np.zeros(cfg.n_blocks, np.float32)
    for j, strength in hot.items():
        t.K[j] = strength * u
        bias[j // cfg.block_size] = 100.0
    t.bias = bias
    if cfg.dtype == "bf16":
        t.h = synth.bf16_to_f32(synth.bf16_round(t.h))
        t.K = synth.bf16_to_f32(synth.bf16_round(t.K))
    return t


def _check(t):
    from oracle import oracle
    cfg = t.cfg
    g = P.run_gpu(t)
    r = oracle.route(t.h, t.Wg, cfg.top_e, t.bias)
    f = oracle.forward(t.h, t.K, t.V, r.block_idx, cfg.block_size, cfg.top_k, want_candidates=True)
    rep = P.compare(t, g, r, f, None)
    print(rep.summary(), flush=True)
    rep.assert_ok()
    again = P.run_gpu(t)
    for n in ("idx", "dK_bits", "dV_bits", "dh", "touched"):
        assert np.array_equal(g[n], again[n]), n
    return g


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_neuron_collects_every_token(dtype):
    # nearly all of 1500 tokens select neuron 70 (six chunks, sorted in LDS); neuron 200 is selected by a few hundred (two chunks)
    cfg = synth.small_case(T=1500, d=72, n_blocks=8, block_size=64, top_e=2, top_k=16, dtype=dtype, seed=1301)
    t = _hot_neurons(cfg, {70: 10.0, 200: 0.35}, seed=5)
    g = _check(t)
    counts = np.bincount(g["idx"].ravel(), minlength=cfg.N)
    assert counts[70] > 1280 and counts.argmax() == 70          # more than five chunks
    assert 256 < counts[200] < counts[70]


def test_more_tokens_than_the_lds_sort_holds():
    # nearly all of 9000 tokens select neuron 3: beyond the 8192 pairs that the sort in LDS takes
    cfg = synth.small_case(T=9000, d=8, n_blocks=2, block_size=8, top_e=1, top_k=2, dtype="f32", seed=1302)
    t = _hot_neurons(cfg, {3: 10.0}, seed=6)
    g = _check(t)
    assert np.bincount(g["idx"].ravel(), minlength=cfg.N)[3] > 8192
