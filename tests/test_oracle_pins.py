"""Pins of the CPU oracle to things other than itself (no GPU needed).

Each test states which part of the paper or of the mathematics fixes the expected value.
"""
import numpy as np
import pytest

from oracle import dense_ref, oracle
from paper_2406_04984_amd import synth


def _inputs(T=12, d=16, B=4, bs=8, e=2, k=5, seed=3, dtype="f32"):
    return synth.make_inputs(synth.small_case(T, d, B, bs, e, k, dtype=dtype, seed=seed))


def _rel(a, b):
    return np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), 1e-300)


# ---------------------------------------------------------------- hand-worked example
def test_worked_example(golden):
    g = golden("worked_example.txt")
    h, Wg, K, V, dOut = (np.array(g[n], np.float32) for n in ("h", "Wg", "K", "V", "dOut"))
    r = oracle.route(h, Wg, g["top_e"])
    assert r.block_idx.tolist() == g["block_idx"]
    assert r.block_score.tolist() == g["block_score"]
    f = oracle.forward(h, K, V, r.block_idx, g["block_size"], g["top_k"])
    assert f.idx.tolist() == g["idx"]
    assert f.score.tolist() == g["score"]
    assert f.out.tolist() == g["out"]
    b = oracle.backward(h, K, V, f.idx, f.score, dOut, g["block_size"])
    assert b.dh.tolist() == g["dh"]
    assert b.dK.tolist() == g["dK"]
    assert b.dV.tolist() == g["dV"]
    assert b.touched.tolist() == g["touched"]


# ---------------------------------------------------------------- dense equivalence (Section 2)
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_all_experts_all_neurons_is_the_dense_parallel_adapter(seed):
    """top_e = n_blocks and top_k = N: the layer is ReLU(h W_A) W_B, values and gradients."""
    t = _inputs(T=9, d=12, B=3, bs=5, e=3, k=15, seed=seed)
    r, f, b = oracle.layer(t)
    assert _rel(f.out, dense_ref.dense_adapter(t.h, t.K, t.V)) < 1e-13
    dh, dK, dV = dense_ref.dense_adapter_grads(t.h, t.K, t.V, t.dOut)
    assert _rel(b.dh, dh) < 1e-13
    assert _rel(b.dK, dK) < 1e-13
    assert _rel(b.dV, dV) < 1e-13
    assert b.touched.tolist() == list(range(15))


def test_all_neurons_of_the_chosen_experts(seed=5):
    """top_k = top_e*block_size: dense adapter restricted to each token's chosen experts (Eq. 6-7)."""
    t = _inputs(T=10, d=8, B=5, bs=4, e=2, k=8, seed=seed)
    r, f, b = oracle.layer(t)
    mask = np.zeros((t.cfg.T, t.cfg.N), bool)
    p = t.h.astype(np.float64) @ t.Wg.astype(np.float64).T
    for tok in range(t.cfg.T):
        for blk in np.argsort(-p[tok], kind="stable")[:2]:
            mask[tok, blk * 4:(blk + 1) * 4] = True
    assert _rel(f.out, dense_ref.masked_adapter(t.h, t.K, t.V, mask)) < 1e-13


def test_saturation_when_few_candidates_are_positive():
    """If a token has at most top_k positive candidates, extra picks add ReLU(<=0)=0 (Eq. 4)."""
    t = _inputs(T=6, d=8, B=2, bs=8, e=1, k=6, seed=11)
    K = t.K.copy()
    # make most keys point away from every token: scores of rows 2.. become negative
    K[:] = -np.abs(K) * np.sign(t.h.sum(0, keepdims=True) + 1e-3)
    hh = np.abs(t.h) * np.sign(t.h.sum(0, keepdims=True) + 1e-3)
    K[0] *= -1
    K[8] *= -1
    r = oracle.route(hh, t.Wg, 1)
    f = oracle.forward(hh, K, t.V, r.block_idx, 8, 6)
    assert (np.sum(f.score > 0, axis=1) <= 1).all()
    mask = np.zeros((6, 16), bool)
    for tok in range(6):
        b0 = r.block_idx[tok, 0]
        mask[tok, b0 * 8:(b0 + 1) * 8] = True
    assert _rel(f.out, dense_ref.masked_adapter(hh, K, t.V, mask)) < 1e-13


# ---------------------------------------------------------------- selection (Eq. 1, Eq. 5)
def test_topk_is_the_head_of_a_stable_descending_sort():
    t = _inputs(T=20, d=16, B=6, bs=16, e=3, k=10, seed=21)
    r, f, _ = oracle.layer(t, want_candidates=True)
    p = t.h.astype(np.float64) @ t.Wg.astype(np.float64).T
    np.testing.assert_allclose(r.p, p, rtol=0, atol=1e-12)
    for tok in range(t.cfg.T):
        want_b = np.argsort(-r.p[tok], kind="stable")[:3]
        assert r.block_idx[tok].tolist() == want_b.tolist()
        cand = np.sort(np.concatenate([np.arange(b * 16, (b + 1) * 16) for b in want_b]))
        assert f.cand_id[tok].tolist() == cand.tolist()
        sc = t.K[cand].astype(np.float64) @ t.h[tok].astype(np.float64)
        np.testing.assert_allclose(f.cand_score[tok], sc, rtol=0, atol=1e-12)
        order = np.argsort(-f.cand_score[tok], kind="stable")[:10]
        assert f.idx[tok].tolist() == cand[order].tolist()
        assert f.next_score[tok] == np.sort(f.cand_score[tok])[::-1][10]


def test_ties_go_to_the_lower_index_and_signed_zeros_tie():
    d = 4
    h = np.array([[1, 0, 0, 0]], np.float32)
    # router: blocks 1 and 2 tie at the top (score 2), block 0 below; top-1 must take block 1
    Wg = np.array([[1, 0, 0, 0], [2, 0, 0, 0], [2, 0, 0, 0]], np.float32)
    r = oracle.route(h, Wg, 1)
    assert r.block_idx.tolist() == [[1]]
    r2 = oracle.route(h, Wg, 2)
    assert r2.block_idx.tolist() == [[1, 2]]
    # keys of block 1 (neurons 4..7): scores 3, 5, 5, 3 -> top-3 = 5, 6, then 4 (tie 3: lower id)
    K = np.zeros((12, d), np.float32)
    K[4:8, 0] = [3, 5, 5, 3]
    V = np.eye(12, d, dtype=np.float32)
    f = oracle.forward(h, K, V, r.block_idx, 4, 3)
    assert f.idx.tolist() == [[5, 6, 4]]
    # +0 and -0 tie: scores [-0, +0, -1, -1] -> top-1 is the lower id although its zero is negative
    K2 = np.zeros((12, d), np.float32)
    K2[4:8, 0] = [-0.0, 0.0, -1, -1]
    f2 = oracle.forward(h, K2, V, r.block_idx, 4, 1)
    assert f2.idx.tolist() == [[4]]


def test_one_expert_equals_global_topk():
    """n_blocks = 1: every neuron is in the one expert (Section 5, number of key experts)."""
    t = _inputs(T=15, d=8, B=1, bs=32, e=1, k=7, seed=9)
    r, f, _ = oracle.layer(t)
    s = t.h.astype(np.float64) @ t.K.astype(np.float64).T
    for tok in range(15):
        assert f.idx[tok].tolist() == np.argsort(-s[tok], kind="stable")[:7].tolist()


def test_one_neuron_per_expert_equals_global_topk():
    """block_size = 1 with the keys as router and top_e = top_k: same as no partitioning."""
    t = _inputs(T=15, d=8, B=32, bs=1, e=7, k=7, seed=10)
    r = oracle.route(t.h, t.K, 7)
    f = oracle.forward(t.h, t.K, t.V, r.block_idx, 1, 7)
    t1 = oracle.route(t.h, np.ones((1, 8), np.float32), 1)
    f1 = oracle.forward(t.h, t.K, t.V, t1.block_idx, 32, 7)
    assert f.idx.tolist() == f1.idx.tolist()
    assert _rel(f.out, f1.out) < 1e-15


def test_index_invariants():
    t = _inputs(T=40, d=16, B=8, bs=16, e=3, k=20, seed=4)
    r, f, b = oracle.layer(t)
    for tok in range(40):
        assert len(set(r.block_idx[tok])) == 3
        assert len(set(f.idx[tok])) == 20
        assert set(f.idx[tok] // 16) <= set(r.block_idx[tok])
    assert b.touched.tolist() == np.unique(f.idx).tolist()
    untouched = np.setdiff1d(np.arange(t.cfg.N), b.touched)
    assert untouched.size > 0
    assert not b.dK[untouched].any() and not b.dV[untouched].any()


# ---------------------------------------------------------------- gradients
def test_gradients_match_central_differences():
    """L = sum(out*dOut) with the selection frozen: fp64 central differences of the oracle's own
    forward on perturbed float32 inputs would round the step away, so the loss is re-evaluated
    with the dense masked formula in numpy (an independent implementation)."""
    t = _inputs(T=5, d=6, B=3, bs=4, e=2, k=5, seed=13)
    r, f, b = oracle.layer(t)
    mask = np.zeros((5, 12), bool)
    for tok in range(5):
        mask[tok, f.idx[tok]] = True
    h, K, V, dOut = (x.astype(np.float64) for x in (t.h, t.K, t.V, t.dOut))

    def loss(h_, K_, V_):
        return float(np.sum(dense_ref.masked_adapter(h_, K_, V_, mask) * dOut))

    eps = 1e-6
    rng = np.random.default_rng(0)
    for name, arr, grad in (("h", h, b.dh), ("K", K, b.dK), ("V", V, b.dV)):
        for _ in range(25):
            i = tuple(rng.integers(0, s) for s in arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[i] += eps
            am[i] -= eps
            args_p = {"h": (ap, K, V), "K": (h, ap, V), "V": (h, K, ap)}[name]
            args_m = {"h": (am, K, V), "K": (h, am, V), "V": (h, K, am)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - grad[i]) < 1e-7 * max(1.0, abs(fd)), (name, i, fd, grad[i])


def test_relu_derivative_is_zero_for_nonpositive_scores():
    h = np.array([[1, 0]], np.float32)
    K = np.array([[0, 1], [-1, 0], [2, 0], [0, 0]], np.float32)   # scores 0, -1, 2, 0
    V = np.array([[1, 1], [1, 2], [3, 1], [5, 5]], np.float32)
    dOut = np.array([[1, 1]], np.float32)
    blk = np.array([[0]], np.int32)
    f = oracle.forward(h, K, V, blk, 4, 3)
    assert f.idx.tolist() == [[2, 0, 3]]
    b = oracle.backward(h, K, V, f.idx, f.score, dOut, 4)
    assert b.dK.tolist() == [[0, 0], [0, 0], [4, 0], [0, 0]]
    assert b.dV.tolist() == [[0, 0], [0, 0], [2, 2], [0, 0]]
    assert b.dh.tolist() == [[8, 0]]
    assert b.touched.tolist() == [0, 2, 3]


def test_row_subset_backward_matches_dense_backward():
    t = _inputs(T=30, d=8, B=4, bs=8, e=2, k=6, seed=17)
    r, f, b = oracle.layer(t)
    rows = np.array([31, 0, 7, 12, 20], np.int32)
    sub = oracle.backward(t.h, t.K, t.V, f.idx, f.score, t.dOut, 8, rows=rows)
    assert (sub.dK == b.dK[rows]).all() and (sub.dV == b.dV[rows]).all()


# ---------------------------------------------------------------- algebraic properties (Eq. 4)
def test_linearity_in_values_and_token_permutation():
    t = _inputs(T=16, d=8, B=4, bs=8, e=2, k=6, seed=19)
    r, f, _ = oracle.layer(t)
    f2 = oracle.forward(t.h, t.K, 2 * t.V, r.block_idx, 8, 6)
    assert (f2.out == 2 * f.out).all()
    perm = np.random.default_rng(1).permutation(16)
    rp = oracle.route(t.h[perm], t.Wg, 2)
    fp = oracle.forward(t.h[perm], t.K, t.V, rp.block_idx, 8, 6)
    assert (fp.out == f.out[perm]).all() and (fp.idx == f.idx[perm]).all()


def test_apply_selection_reproduces_forward():
    t = _inputs(T=16, d=8, B=4, bs=8, e=2, k=6, seed=23)
    r, f, _ = oracle.layer(t)
    assert (oracle.apply_selection(t.h, t.K, t.V, f.idx, 8) == f.out).all()


def test_router_bias_shifts_scores():
    t = _inputs(T=16, d=8, B=4, bs=8, e=2, k=6, seed=29)
    bias = np.array([0, 100, 0, -100], np.float32)
    r = oracle.route(t.h, t.Wg, 2, bias)
    assert (r.block_idx[:, 0] == 1).all() and (r.block_idx != 3).all()
    p = t.h.astype(np.float64) @ t.Wg.astype(np.float64).T + bias
    np.testing.assert_allclose(r.p, p, atol=1e-12)


def test_flop_model_of_the_efficiency_analysis():
    """Section 3.3: routing + in-expert scoring cost T*n_blocks*d + top_e*(N/n_blocks)*T*d MACs;
    the number of candidates the oracle scores per token is top_e*block_size."""
    t = _inputs(T=7, d=8, B=4, bs=8, e=2, k=6, seed=31)
    r, f, _ = oracle.layer(t, want_candidates=True)
    assert r.p.shape == (7, 4) and f.cand_score.shape == (7, 2 * 8)


def test_bad_arguments_are_rejected():
    t = _inputs()
    with pytest.raises(ValueError):
        oracle.route(t.h, t.Wg, 5)            # top_e > n_blocks
    r = oracle.route(t.h, t.Wg, 2)
    with pytest.raises(ValueError):
        oracle.forward(t.h, t.K, t.V, r.block_idx, 8, 17)   # top_k > top_e*block_size
