"""Top-k selection over candidate sets beyond LDS capacity (more than 12288 candidates per token), the case of
the paper's ablation without key experts: one block that holds every neuron, Eq. 1-4 over all of them.
Same rules as the other parity tests (tests/parity.py)."""
import numpy as np
import pytest

from paper_2406_04984_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    from tests import parity
    return parity


def _case(P, **kw):
    cfg = synth.small_case(**kw)
    rep = P.run_and_compare(cfg)
    print(rep.summary(), flush=True)
    rep.assert_ok()
    return rep


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_block_holds_every_neuron(P, dtype):
    # 20000 candidates: five sweep tiles of 4096 with a ragged last one
    _case(P, T=40, d=64, n_blocks=1, block_size=20000, top_e=1, top_k=50, dtype=dtype, seed=901)


def test_two_large_blocks_odd_sizes(P):
    # candidate count not a multiple of 4, k larger than a wave, three blocks of which two are chosen
    _case(P, T=30, d=72, n_blocks=3, block_size=8191, top_e=2, top_k=300, dtype="f32", seed=902)


def test_k_of_thousands(P):
    _case(P, T=12, d=64, n_blocks=1, block_size=16384, top_e=1, top_k=5000, dtype="bf16", seed=903)


def test_exact_ties_across_sweep_tiles(P):
    """Every key appears four times, 4100 positions apart, so equal scores sit in different sweep tiles; the
    copies with the lower ids must win, exactly as in the oracle."""
    cfg = synth.small_case(T=16, d=64, n_blocks=1, block_size=16400, top_e=1, top_k=37, dtype="bf16", seed=904)
    t = synth.make_inputs(cfg)
    t.K[4100:8200] = t.K[0:4100]
    t.K[8200:12300] = t.K[0:4100]
    t.K[12300:16400] = t.K[0:4100]
    from oracle import oracle
    g = P.run_gpu(t)
    r = oracle.route(t.h, t.Wg, cfg.top_e, t.bias)
    f = oracle.forward(t.h, t.K, t.V, r.block_idx, cfg.block_size, cfg.top_k, want_candidates=True)
    b = oracle.backward(t.h, t.K, t.V, f.idx, f.score, t.dOut, cfg.block_size)
    rep = P.compare(t, g, r, f, b)
    print(rep.summary(), flush=True)
    rep.assert_ok()
    assert (g["idx"] == np.sort(f.idx, 1)).all()


@pytest.mark.timeout(900)
def test_no_key_experts_at_scale(P):
    # 2048 tokens over one block of 65536 neurons (the keys and values of the LLaMA-7B-shaped configuration
    # without the router): the launch configuration bench.py times for this variant; every selection, out and dh
    # are compared row by row, dK / dV on the first and last row, the rows at every 128-row boundary and 256
    # random rows
    cfg = synth.CONFIGS["noke_bf16"]
    rows = P.stratified_rows(cfg, 256)
    rep = P.run_and_compare(cfg, rows=rows)
    print(rep.summary(), flush=True)
    rep.assert_ok()
