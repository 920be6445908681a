"""Pins of the oracle's row-sparse Adam step (no GPU): closed form, two library optimizers, invariants."""
import numpy as np
import pytest
import torch

from oracle import oracle as O


def _case(N=12, d=8, seed=0):
    rng = np.random.default_rng(seed)
    return rng.normal(size=(N, d)), rng.normal(size=(N, d)) * 0.1


def test_first_step_closed_form():
    # from zero moments the first step moves every touched weight by lr * g / (|g| + eps)  (Adam, bias-corrected)
    w, g = _case()
    touched = np.arange(w.shape[0], dtype=np.int32)
    lr, eps = 1e-2, 1e-8
    w1, m1, v1 = O.adam_rows(w, g, np.zeros_like(w), np.zeros_like(w), touched, 1, lr, 0.9, 0.999, eps)
    np.testing.assert_allclose(w1, w - lr * g / (np.abs(g) + eps), rtol=1e-13, atol=0)
    np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-13)
    np.testing.assert_allclose(v1, 0.001 * g * g, rtol=1e-12)


def test_all_rows_equals_torch_adam():
    # with every row touched in every step the method is plain Adam: torch.optim.Adam in float64
    w, _ = _case(seed=1)
    N, d = w.shape
    rng = np.random.default_rng(2)
    p = torch.nn.Parameter(torch.tensor(w, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=3e-3, betas=(0.9, 0.999), eps=1e-8)
    m, v = np.zeros_like(w), np.zeros_like(w)
    touched = np.arange(N, dtype=np.int32)
    for step in range(1, 7):
        g = rng.normal(size=(N, d)) * (0.1 if step % 2 else 1e-6)   # tiny gradients make eps matter
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = O.adam_rows(w, g, m, v, touched, step, 3e-3, 0.9, 0.999, 1e-8)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-11, atol=1e-14)


def test_row_subsets_equal_torch_sparse_adam():
    # rows without a gradient keep their state; the step count is global: torch.optim.SparseAdam.
    # (eps is made negligible: that optimizer adds it before the bias correction of the second moment.)
    w, _ = _case(N=16, d=4, seed=3)
    N, d = w.shape
    rng = np.random.default_rng(4)
    p = torch.nn.Parameter(torch.tensor(w, dtype=torch.float64))
    opt = torch.optim.SparseAdam([p], lr=1e-2, betas=(0.8, 0.95), eps=1e-30)
    m, v = np.zeros_like(w), np.zeros_like(w)
    for step in range(1, 8):
        rows = np.sort(rng.choice(N, size=rng.integers(1, N), replace=False)).astype(np.int32)
        g = np.zeros((N, d))
        g[rows] = rng.normal(size=(len(rows), d))
        p.grad = torch.sparse_coo_tensor(torch.tensor(rows[None, :].astype(np.int64)),
                                         torch.tensor(g[rows], dtype=torch.float64), size=(N, d))
        opt.step()
        w, m, v = O.adam_rows(w, g, m, v, rows, step, 1e-2, 0.8, 0.95, 1e-30)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-11, atol=1e-14)


def test_untouched_rows_are_bit_identical():
    w, g = _case(seed=5)
    m = np.abs(g) * 0.3
    v = g * g * 0.2
    touched = np.array([1, 4, 5, 10], dtype=np.int32)
    w1, m1, v1 = O.adam_rows(w, g, m, v, touched, 3, 1e-2)
    rest = np.setdiff1d(np.arange(w.shape[0]), touched)
    assert np.array_equal(w1[rest], w[rest]) and np.array_equal(m1[rest], m[rest]) and np.array_equal(v1[rest], v[rest])
    assert not np.any(w1[touched] == w[touched])


def test_rejects_bad_lists_and_steps():
    w, g = _case()
    z = np.zeros_like(w)
    with pytest.raises(ValueError):
        O.adam_rows(w, g, z, z, np.array([3, 2], dtype=np.int32), 1, 1e-3)      # not ascending
    with pytest.raises(ValueError):
        O.adam_rows(w, g, z, z, np.array([0, 99], dtype=np.int32), 1, 1e-3)     # out of range
    with pytest.raises(ValueError):
        O.adam_rows(w, g, z, z, np.array([0], dtype=np.int32), 0, 1e-3)         # steps count from 1
