"""Parity harness: runs the HIP path through its C ABI and the CPU oracle on the same seeded
inputs and compares them under the benchmark's rules.

Rules
  * selected index sets (blocks per token, neurons per token) are compared as sets and must be
    identical, except that a token may differ where the oracle's own scores tie to within 1e-5
    relative at the selection boundary: every id in the symmetric difference must then have an
    oracle score within 1e-5*|s_b| of s_b, the oracle's last selected score;
  * a token whose selection differs inside that band holds a valid selection that is not the
    oracle's: its values are judged by REPLAY -- the oracle's steps after the selection
    (activation-weighted value sum, backward) are run on the selection the HIP path took, with
    the oracle's own fp64 scores for those neurons, and everything is compared against that.
    Nothing is left out of the value comparison except tokens outside the band (which fail);
  * out, dh, dK, dV agree within relative L2 2e-2 (bf16) / 1e-4 (fp32) over the whole tensor, AND
    row by row: |x_r - y_r|_2 <= tol |y_r|_2 + 1e-2 tol rms(y) sqrt(d); a row the oracle has exactly
    zero must be exactly zero;
  * rows of dK, dV outside `touched` still hold the sentinel they were filled with.
A selected pair whose oracle score is within 1e-5 (relative to the token's largest score) of the
ReLU kink may take either branch of the derivative in fp32; its token / neuron rows are left out of
the row-by-row check (and counted in the report).
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Tuple

import numpy as np

from oracle import oracle
from paper_2406_04984_amd import synth
from paper_2406_04984_amd.harness import (SENTINEL_BF16, SENTINEL_F32, DeviceLayer, to_device,  # noqa: F401
                                          to_host, to_pinned)

TIE_BAND = 1e-5
TOL = {"f32": 1e-4, "bf16": 2e-2}
ROW_FLOOR = 1e-2        # absolute slack of a row, in units of tol * (rms of the tensor) * sqrt(d)


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    den = np.linalg.norm(b)
    num = np.linalg.norm(a - b)
    return float(num / den) if den > 0 else float(num)


def row_check(x: np.ndarray, y: np.ndarray, tol: float, skip: Optional[np.ndarray] = None) -> Tuple[float, int, int]:
    """Row-by-row bound of x against the oracle's y.  Returns (largest error / bound over the rows,
    index of that row, number of rows the oracle has exactly zero that are not exactly zero in x)."""
    x = np.asarray(x, np.float64)
    y = np.asarray(y, np.float64)
    if y.size == 0:
        return 0.0, -1, 0
    d = y.shape[1]
    floor = ROW_FLOOR * tol * float(np.sqrt(np.mean(y * y))) * np.sqrt(d)
    err = np.linalg.norm(x - y, axis=1)
    bound = tol * np.linalg.norm(y, axis=1) + floor
    zero = ~y.any(axis=1)
    nonzero_where_zero = zero & x.any(axis=1)
    ratio = np.where(bound > 0, err / np.where(bound > 0, bound, 1.0), np.where(err > 0, np.inf, 0.0))
    if skip is not None:
        ratio = np.where(skip, 0.0, ratio)
        nonzero_where_zero &= ~skip
    w = int(np.argmax(ratio))
    return float(ratio[w]), w, int(nonzero_where_zero.sum())


def stratified_rows(cfg: synth.Config, n_random: int, tile: int = 128) -> np.ndarray:
    """Neuron rows for a sampled dK / dV comparison: of every block the first and the last neuron and the two
    rows on either side of every `tile`-row boundary inside it, plus `n_random` seeded random rows."""
    bs = cfg.block_size
    inside = {0, bs - 1}
    for m in range(tile, bs, tile):
        inside.update((m - 1, m))
    base = (np.arange(cfg.n_blocks)[:, None] * bs + np.array(sorted(inside))[None, :]).ravel()
    rnd = np.random.default_rng(cfg.seed).choice(cfg.N, size=min(n_random, cfg.N), replace=False)
    return np.unique(np.concatenate([base, rnd])).astype(np.int32)


@dataclasses.dataclass
class Report:
    name: str
    dtype: str
    tokens: int
    block_band_tokens: int = 0          # tokens whose block set differs inside the tie band (replayed)
    block_bad_tokens: int = 0           # ... outside the band (failure)
    idx_band_tokens: int = 0            # tokens whose neuron set differs inside the tie band (replayed)
    idx_bad_tokens: int = 0
    invariant_errors: List[str] = dataclasses.field(default_factory=list)
    err: Dict[str, float] = dataclasses.field(default_factory=dict)        # whole-tensor relative L2
    row_err: Dict[str, Tuple[float, int]] = dataclasses.field(default_factory=dict)   # worst row: (err / bound, row)
    zero_rows_not_zero: Dict[str, int] = dataclasses.field(default_factory=dict)
    kink_pairs: int = 0
    rows_compared: int = 0
    n_touched: int = 0

    def ok(self) -> bool:
        tol = TOL[self.dtype]
        return (self.block_bad_tokens == 0 and self.idx_bad_tokens == 0 and not self.invariant_errors
                and all(v <= tol for v in self.err.values())
                and all(v[0] <= 1.0 for v in self.row_err.values())
                and all(v == 0 for v in self.zero_rows_not_zero.values())
                and (self.block_band_tokens + self.idx_band_tokens) <= max(2, 0.05 * self.tokens))

    def summary(self) -> str:
        e = " ".join(f"{k}={v:.2e}" for k, v in self.err.items())
        rw = " ".join(f"{k}:{v[0]:.2f}@{v[1]}" for k, v in self.row_err.items())
        z = {k: v for k, v in self.zero_rows_not_zero.items() if v}
        return (f"{self.name}: tokens={self.tokens} blocks(band/bad)={self.block_band_tokens}/{self.block_bad_tokens} "
                f"idx(band/bad)={self.idx_band_tokens}/{self.idx_bad_tokens} touched={self.n_touched} "
                f"grad_rows={self.rows_compared} kink_pairs={self.kink_pairs} {e} "
                f"worst_row(err/bound@row) {rw} zero_rows_not_zero={z or 0} "
                f"invariants={self.invariant_errors or 'ok'}")

    def assert_ok(self):
        assert self.ok(), self.summary()


def _band_ok(diff_scores: np.ndarray, boundary: float) -> bool:
    return bool(np.all(np.abs(diff_scores - boundary) <= TIE_BAND * abs(boundary)))


def _lookup(cand_id: np.ndarray, cand_score: np.ndarray, ids: np.ndarray):
    """Oracle scores of `ids` among a token's candidates (ascending ids); second result: all found."""
    pos = np.searchsorted(cand_id, ids)
    pos_c = np.minimum(pos, cand_id.size - 1)
    found = (pos < cand_id.size) & (cand_id[pos_c] == ids)
    return cand_score[pos_c], bool(found.all())


def compare(t: synth.Tensors, g: Dict[str, np.ndarray], r: oracle.Route, f: oracle.Forward,
            b: Optional[oracle.Backward], tokens: Optional[np.ndarray] = None,
            rows: Optional[np.ndarray] = None, want_bwd: bool = True) -> Report:
    """`tokens`: the token ids the oracle results r, f (and b.dh) cover, default all.  `rows`: the
    neuron ids b.dK / b.dV cover (in that order), default all N.  `b` is the oracle's backward on its own
    selection; when some token is replayed the backward is computed here on the replayed selection instead
    (also when b is None and want_bwd)."""
    c = t.cfg
    T, k, e, N, bs = c.T, c.top_k, c.top_e, c.N, c.block_size
    tok = np.arange(T) if tokens is None else np.asarray(tokens)
    rep = Report(c.name, c.dtype, len(tok))
    tol = TOL[c.dtype]
    if f.cand_id is None:
        raise ValueError("compare needs the oracle's candidate scores (forward(..., want_candidates=True))")

    # ---- structural invariants of the GPU result, all tokens
    gi = g["idx"]
    gs = np.sort(gi, axis=1)
    if (gi != gs).any():
        rep.invariant_errors.append("idx rows are not ascending")
    if (gs[:, 1:] == gs[:, :-1]).any():
        rep.invariant_errors.append("duplicate neuron id inside a token")
    if gi.min() < 0 or gi.max() >= N:
        rep.invariant_errors.append("neuron id out of range")
    gb = g["block_idx"]
    if gb.min() < 0 or gb.max() >= c.n_blocks:
        rep.invariant_errors.append("block id out of range")
    if (np.sort(gb, 1)[:, 1:] == np.sort(gb, 1)[:, :-1]).any():
        rep.invariant_errors.append("duplicate block id inside a token")
    blk_of = gi // bs
    inside = (blk_of[:, :, None] == gb[:, None, :]).any(-1)
    if not inside.all():
        rep.invariant_errors.append("a selected neuron lies outside the token's blocks")
    if (np.diff(g["block_score"], axis=1) > 0).any():
        rep.invariant_errors.append("block scores are not descending")
    uniq = np.unique(gi)
    if g["n_touched"] != uniq.size or not np.array_equal(g["touched"], uniq):
        rep.invariant_errors.append("touched is not the sorted unique of idx")
    rep.n_touched = int(g["n_touched"])
    untouched = np.ones(N, bool)
    untouched[uniq] = False
    for nm in ("dK", "dV"):
        if not g[nm + "_row_all_sentinel"][untouched].all():
            rep.invariant_errors.append(f"{nm}: an untouched row was written")
        if g[nm + "_row_any_sentinel"][~untouched].any():
            rep.invariant_errors.append(f"{nm}: a touched row was not (fully) written")
    if (g["act"] < 0).any():
        rep.invariant_errors.append("negative activation")

    # ---- selections against the oracle, covered tokens.  idx_rep / score_rep: the selection the values are
    # judged on -- the oracle's own, except for tokens inside the tie band, which take the HIP path's.
    idx_rep = f.idx.copy()
    score_rep = f.score.copy()
    valid = np.ones(len(tok), bool)      # False: selection wrong outside the band
    replayed = np.zeros(len(tok), bool)
    for n, tt in enumerate(tok):
        cand_id, cand_score, last = f.cand_id[n], f.cand_score[n], f.score[n, k - 1]
        ob, gbt = set(r.block_idx[n].tolist()), set(gb[tt].tolist())
        if ob != gbt:
            diff = np.array(sorted(ob ^ gbt))
            if not _band_ok(r.p[n][diff], r.block_score[n, e - 1]):
                rep.block_bad_tokens += 1
                valid[n] = False
                continue
            rep.block_band_tokens += 1
            # a valid routing that is not the oracle's: the oracle's steps 3-4 on the blocks the HIP path took
            f1 = oracle.forward(t.h[tt:tt + 1], t.K, t.V, gb[tt:tt + 1], bs, k, want_candidates=True)
            cand_id, cand_score, last = f1.cand_id[0], f1.cand_score[0], f1.score[0, k - 1]
            idx_rep[n], score_rep[n] = f1.idx[0], f1.score[0]
            replayed[n] = True
        oi, git = set(idx_rep[n].tolist()), set(gi[tt].tolist())
        if oi != git:
            diff = np.array(sorted(oi ^ git))
            sc_diff, found = _lookup(cand_id, cand_score, diff)
            if not (found and _band_ok(sc_diff, last)):
                rep.idx_bad_tokens += 1
                valid[n] = False
                continue
            rep.idx_band_tokens += 1
            idx_rep[n] = gi[tt]
            score_rep[n], _ = _lookup(cand_id, cand_score, gi[tt])
            replayed[n] = True

    # ---- the oracle's values on idx_rep
    out_o = f.out.copy()
    if replayed.any():
        rp = np.nonzero(replayed)[0]
        out_o[rp] = oracle.apply_selection(t.h[tok[rp]], t.K, t.V, idx_rep[rp], bs)
    full_cover = tokens is None
    if want_bwd and full_cover and (b is None or replayed.any()) and valid.all():
        b = oracle.backward(t.h, t.K, t.V, idx_rep, score_rep, t.dOut, bs, rows=rows)

    # pairs at the ReLU kink: either branch of the derivative is right within fp32
    scale = np.abs(score_rep).max(axis=1, keepdims=True)
    kink = (np.abs(score_rep) <= TIE_BAND * scale) & t.h[tok].any(axis=1, keepdims=True)
    rep.kink_pairs = int(kink.sum())
    kink_tok = kink.any(axis=1)
    kink_neurons = np.unique(idx_rep[kink])

    # ---- values
    gt = tok[valid]
    if gt.size:
        order = np.argsort(idx_rep[valid], axis=1)       # oracle rows are ordered by score, the HIP path's by id
        o_act = np.take_along_axis(np.maximum(score_rep[valid], 0.0), order, axis=1)
        rep.err["act"] = rel_l2(g["act"][gt], o_act)
        unre = valid & ~replayed
        if unre.any():
            rep.err["block_score"] = rel_l2(g["block_score"][tok[unre]], r.block_score[unre])
        rep.err["out"] = rel_l2(g["out"][gt], out_o[valid])
        w, at, z = row_check(g["out"][gt], out_o[valid], tol)
        rep.row_err["out"], rep.zero_rows_not_zero["out"] = (w, int(gt[at]) if at >= 0 else -1), z
        if b is not None and b.dh is not None:
            rep.err["dh"] = rel_l2(g["dh"][gt], b.dh[valid])
            w, at, z = row_check(g["dh"][gt], b.dh[valid], tol, skip=kink_tok[valid])
            rep.row_err["dh"], rep.zero_rows_not_zero["dh"] = (w, int(gt[at]) if at >= 0 else -1), z
    if b is not None:
        if not full_cover:
            # gradient rows need every token's selection: only valid when the oracle covered all tokens
            raise ValueError("row comparison needs oracle results for all tokens")
        rws = np.arange(N) if rows is None else np.asarray(rows)
        o_touched = np.zeros(N, bool)
        o_touched[b.touched] = True
        if valid.all() and not np.array_equal(o_touched[rws], (~untouched)[rws]):
            rep.invariant_errors.append("touched differs from the oracle's")
        sel = (~untouched)[rws] & o_touched[rws]
        if g.get("grad_rows") is not None:
            assert np.array_equal(g["grad_rows"], rws), "GPU gradient rows were fetched for other neurons"
            gK, gV = g["dK"], g["dV"]
        else:
            gK, gV = g["dK"][rws], g["dV"][rws]
        rep.rows_compared = int(sel.sum())
        rep.err["dK"] = rel_l2(gK[sel], b.dK[sel])
        rep.err["dV"] = rel_l2(gV[sel], b.dV[sel])
        skip = np.isin(rws[sel], kink_neurons)
        for nm, gx, ox in (("dK", gK, b.dK), ("dV", gV, b.dV)):
            w, at, z = row_check(gx[sel], ox[sel], tol, skip=skip if nm == "dK" else None)
            rep.row_err[nm], rep.zero_rows_not_zero[nm] = (w, int(rws[sel][at]) if at >= 0 else -1), z
    return rep


def run_gpu(t: synth.Tensors, binding=None, rows: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    layer = DeviceLayer(t, binding)
    layer.fill_grad_sentinel()
    layer.step()
    return layer.results(rows)


def run_and_compare(cfg: synth.Config, rows: Optional[np.ndarray] = None) -> Report:
    """Full comparison; with `rows`, dK / dV are compared on those neuron ids only (large shapes)."""
    t = synth.make_inputs(cfg)
    g = run_gpu(t, rows=rows)
    r = oracle.route(t.h, t.Wg, cfg.top_e, t.bias)
    f = oracle.forward(t.h, t.K, t.V, r.block_idx, cfg.block_size, cfg.top_k, want_candidates=True)
    return compare(t, g, r, f, None, rows=rows)
