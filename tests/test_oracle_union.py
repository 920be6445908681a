"""Pins of the oracle's batch-union evaluation (Algorithm 1 as printed), no GPU."""
import numpy as np

from oracle import dense_ref as D
from oracle import oracle as O
from paper_2406_04984_amd import synth


def _case(T=24, d=16, nb=6, bs=8, e=2, k=5, seed=21):
    cfg = synth.small_case(T, d, nb, bs, e, k, dtype="f32", seed=seed)
    return synth.make_inputs(cfg)


def _selection(t):
    c = t.cfg
    r = O.route(t.h, t.Wg, c.top_e, t.bias)
    return O.forward(t.h, t.K, t.V, r.block_idx, c.block_size, c.top_k)


def test_union_is_the_dense_adapter_over_the_compacted_rows():
    # library matmuls over K[S], V[S]: pins the indexing through S and the ReLU
    t = _case()
    f = _selection(t)
    S = O.union_of(f.idx)
    assert 0 < len(S) < t.cfg.N
    out = O.union_forward(t.h, t.K, t.V, S)
    np.testing.assert_allclose(out, D.dense_adapter(t.h, t.K[S], t.V[S]), rtol=1e-12, atol=1e-14)
    dh, dK, dV = O.union_backward(t.h, t.K, t.V, S, t.dOut)
    rh, rK, rV = D.dense_adapter_grads(t.h, t.K[S], t.V[S], t.dOut)
    np.testing.assert_allclose(dh, rh, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dK, rK, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dV, rV, rtol=1e-11, atol=1e-13)


def test_everything_selected_is_the_dense_adapter():
    t = _case(T=9, d=8, nb=3, bs=4, e=3, k=12)
    f = _selection(t)
    S = O.union_of(f.idx)
    assert np.array_equal(S, np.arange(t.cfg.N))
    np.testing.assert_allclose(O.union_forward(t.h, t.K, t.V, S), D.dense_adapter(t.h, t.K, t.V), rtol=1e-12)


def test_one_token_union_equals_the_per_token_result():
    t = _case(T=1, d=16, nb=4, bs=8, e=2, k=6, seed=22)
    f = _selection(t)
    S = O.union_of(f.idx)
    assert len(S) == t.cfg.top_k
    np.testing.assert_allclose(O.union_forward(t.h, t.K, t.V, S), f.out, rtol=1e-12, atol=1e-15)


def test_union_minus_per_token_is_the_other_tokens_neurons():
    # per token, the union result exceeds the per-token result by the positive-score neurons the token did
    # not select itself (they come from other tokens' lists)
    t = _case(seed=23)
    f = _selection(t)
    S = O.union_of(f.idx)
    out = O.union_forward(t.h, t.K, t.V, S)
    sc = np.asarray(t.h, np.float64) @ np.asarray(t.K, np.float64).T
    extra = np.zeros_like(out)
    for tok in range(t.cfg.T):
        others = np.setdiff1d(S, f.idx[tok])
        a = np.maximum(sc[tok, others], 0.0)
        extra[tok] = a @ np.asarray(t.V, np.float64)[others]
    np.testing.assert_allclose(out - f.out, extra, rtol=1e-9, atol=1e-12)
    assert np.abs(extra).max() > 0


def test_union_gradients_by_central_differences():
    t = _case(T=5, d=6, nb=3, bs=4, e=2, k=3, seed=24)
    f = _selection(t)
    S = O.union_of(f.idx)
    dh, dK, dV = O.union_backward(t.h, t.K, t.V, S, t.dOut)
    g = np.asarray(t.dOut, np.float64)

    def loss(h, K, V):
        s = np.asarray(h, np.float64) @ np.asarray(K, np.float64)[S].T
        return float((np.maximum(s, 0.0) @ np.asarray(V, np.float64)[S] * g).sum())

    eps = 1e-6
    rng = np.random.default_rng(0)
    for name, grad in (("h", dh), ("K", dK), ("V", dV)):
        for _ in range(12):
            base = {"h": t.h.astype(np.float64), "K": t.K.astype(np.float64), "V": t.V.astype(np.float64)}
            if name == "h":
                r, c = rng.integers(t.cfg.T), rng.integers(t.cfg.d)
                want = grad[r, c]
            else:
                i, c = rng.integers(len(S)), rng.integers(t.cfg.d)
                r, want = S[i], grad[i, c]
            hi = {k_: v.copy() for k_, v in base.items()}
            lo = {k_: v.copy() for k_, v in base.items()}
            hi[name][r, c] += eps
            lo[name][r, c] -= eps
            num = (loss(hi["h"], hi["K"], hi["V"]) - loss(lo["h"], lo["K"], lo["V"])) / (2 * eps)
            assert abs(num - want) <= 1e-6 * max(1.0, abs(want)), (name, r, c, num, want)


def test_union_rejects_unsorted_lists():
    import pytest
    t = _case(T=2)
    with pytest.raises(ValueError):
        O.union_forward(t.h, t.K, t.V, np.array([3, 1], np.int32))
