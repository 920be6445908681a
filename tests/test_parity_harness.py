"""The comparison rules of tests/parity.py, checked on the CPU: results made from the oracle's own output must
pass, a single wrong row must fail although the whole-tensor norm barely moves, a selection that differs inside
the tie band is replayed (not dropped), one that differs outside it fails."""
import numpy as np
import pytest

from oracle import oracle
from paper_2406_04984_amd import synth
from tests import parity as P


def _as_device_result(t, r, f, b):
    """What the HIP path would hand back if it computed exactly the oracle's values."""
    c = t.cfg
    order = np.argsort(f.idx, axis=1)
    idx = np.take_along_axis(f.idx, order, axis=1)
    act = np.take_along_axis(f.act, order, axis=1).astype(np.float32)
    touched = np.unique(idx).astype(np.int32)
    untouched = np.ones(c.N, bool)
    untouched[touched] = False
    g = dict(block_idx=r.block_idx.copy(), block_score=r.block_score.astype(np.float32), out=f.out.copy(), idx=idx,
             act=act, dh=b.dh.copy(), touched=touched, n_touched=int(touched.size), dK=b.dK.copy(), dV=b.dV.copy(),
             grad_rows=None)
    for nm in ("dK", "dV"):
        g[nm + "_row_all_sentinel"] = untouched.copy()
        g[nm + "_row_any_sentinel"] = untouched.copy()
    return g


@pytest.fixture(scope="module")
def case():
    cfg = synth.small_case(T=60, d=64, n_blocks=6, block_size=32, top_e=2, top_k=12, dtype="f32", seed=31)
    t = synth.make_inputs(cfg)
    r, f, b = oracle.layer(t, want_candidates=True)
    return t, r, f, b


def test_the_oracles_own_result_passes(case):
    t, r, f, b = case
    rep = P.compare(t, _as_device_result(t, r, f, b), r, f, b)
    assert rep.ok(), rep.summary()
    assert rep.row_err["out"][0] == 0.0 and rep.block_band_tokens == 0 and rep.idx_band_tokens == 0


@pytest.mark.parametrize("name", ["out", "dh", "dK", "dV"])
def test_one_wrong_row_fails_though_the_whole_tensor_norm_passes(case, name):
    t, r, f, b = case
    g = _as_device_result(t, r, f, b)
    row = int(g["touched"][3]) if name in ("dK", "dV") else 17
    g[name][row] *= 1.01          # one row off by 1 %: far beyond 1e-4 for that row
    rep = P.compare(t, g, r, f, b)
    assert rep.err[name] <= P.TOL["f32"] * 20
    assert not rep.ok()
    assert rep.row_err[name][0] > 1.0 and rep.row_err[name][1] == row, rep.summary()


def test_a_row_that_must_be_zero(case):
    t, r, f, b = case
    t2 = synth.Tensors(t.cfg, t.h.copy(), t.Wg, t.K, t.V, t.dOut, t.bias, t.outlier_channels)
    t2.h[5] = 0.0                 # a zero token: zero scores, zero activations, zero out and dh rows
    r2, f2, b2 = oracle.layer(t2, want_candidates=True)
    g = _as_device_result(t2, r2, f2, b2)
    assert P.compare(t2, g, r2, f2, b2).ok()
    g["out"][5, 3] = 1e-30
    rep = P.compare(t2, g, r2, f2, b2)
    assert rep.zero_rows_not_zero["out"] == 1 and not rep.ok()


def test_a_selection_inside_the_tie_band_is_replayed(case):
    t, r, f, b = case
    # token 9: its last selected neuron gets an exact duplicate among the unselected candidates of the same block
    tt = 9
    last = int(f.idx[tt, -1])
    blk = last // t.cfg.block_size
    sel = set(f.idx[tt].tolist())
    twin = next(j for j in range(blk * t.cfg.block_size, (blk + 1) * t.cfg.block_size) if j not in sel and j > last)
    K2 = t.K.copy()
    K2[twin] = K2[last]
    t2 = synth.Tensors(t.cfg, t.h, t.Wg, K2, t.V, t.dOut, t.bias, t.outlier_channels)
    r2, f2, b2 = oracle.layer(t2, want_candidates=True)
    assert last in f2.idx[tt] and twin not in f2.idx[tt]      # the oracle breaks the tie to the lower id
    # a device result that took the twin instead: valid inside the band, values follow that selection
    idx_alt = f2.idx.copy()
    idx_alt[tt, idx_alt[tt] == last] = twin
    b_alt = oracle.backward(t2.h, t2.K, t2.V, idx_alt, f2.score, t2.dOut, t2.cfg.block_size)
    f_alt = oracle.Forward(f2.out.copy(), idx_alt, f2.score, f2.act, f2.next_score, None, None)
    f_alt.out[tt] = oracle.apply_selection(t2.h[tt:tt + 1], t2.K, t2.V, idx_alt[tt:tt + 1], t2.cfg.block_size)[0]
    g = _as_device_result(t2, r2, f_alt, b_alt)
    rep = P.compare(t2, g, r2, f2, b2)
    assert rep.idx_band_tokens == 1 and rep.idx_bad_tokens == 0
    assert rep.ok(), rep.summary()
    # the replayed token is judged, not dropped: a wrong out row for it fails
    g["out"][tt] *= 1.01
    rep = P.compare(t2, g, r2, f2, b2)
    assert not rep.ok() and rep.row_err["out"][1] == tt


def test_a_selection_outside_the_band_fails(case):
    t, r, f, b = case
    g = _as_device_result(t, r, f, b)
    tt = 4
    blk = int(f.idx[tt, 0]) // t.cfg.block_size
    sel = set(g["idx"][tt].tolist())
    other = next(j for j in range(blk * t.cfg.block_size, (blk + 1) * t.cfg.block_size) if j not in sel)
    row = g["idx"][tt].copy()
    row[row == f.idx[tt, 0]] = other           # the best neuron swapped for an unselected one
    g["idx"][tt] = np.sort(row)
    g["touched"] = np.unique(g["idx"]).astype(np.int32)
    g["n_touched"] = int(g["touched"].size)
    rep = P.compare(t, g, r, f, b)
    assert rep.idx_bad_tokens == 1 and not rep.ok()


def test_stratified_rows_cover_block_and_tile_edges():
    cfg = synth.CONFIGS["llama7b_bf16"]
    rows = P.stratified_rows(cfg, 384)
    s = set(rows.tolist())
    for blk in (0, 17, cfg.n_blocks - 1):
        base = blk * cfg.block_size
        for r_in in (0, 127, 128, 511, 512, 895, 896, cfg.block_size - 1):
            assert base + r_in in s
    assert rows.size >= 64 * 16 + 300 and (np.diff(rows) > 0).all()
