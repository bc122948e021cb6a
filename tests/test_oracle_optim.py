"""Pins of the optimiser oracle: PyTorch's CPU optimisers (library routines) in fp64, and closed forms."""
import numpy as np
import torch

from oracle import optim_oracle as P


def test_dense_adam_against_torch():
    rng = np.random.default_rng(0)
    th0 = rng.normal(size=(7, 5))
    p = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=3e-3, betas=(0.8, 0.95), eps=1e-6)
    th, m, v = th0, np.zeros_like(th0), np.zeros_like(th0)
    for step in range(1, 8):
        g = rng.normal(size=th0.shape) * 10.0 ** rng.integers(-4, 2)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, m, v = P.adam_step(th, g, m, v, step, 3e-3, 0.8, 0.95, 1e-6)
        assert np.allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_rows_adam_against_torch_sparse_adam():
    rng = np.random.default_rng(1)
    V, F = 30, 4
    th0 = rng.normal(size=(V, F))
    p = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    # torch's sparse variant adds eps before the bias correction of the second moment; with eps -> 0 (and non-zero
    # gradients) the two forms coincide, so this pins what is specific to rows: untouched rows keep their moments,
    # the bias correction counts global steps.  Where eps goes is pinned by the dense comparison above.
    opt = torch.optim.SparseAdam([p], lr=2e-2, betas=(0.9, 0.99), eps=1e-300)   # (it refuses an exact zero)
    th, m, v = th0, np.zeros_like(th0), np.zeros_like(th0)
    for step in range(1, 7):
        ids = rng.choice(V, size=rng.integers(1, 12), replace=False)
        g = rng.normal(size=(len(ids), F))
        p.grad = torch.sparse_coo_tensor(torch.tensor(ids[None, :]), torch.tensor(g), size=(V, F))
        opt.step()
        th, m, v = P.adam_rows_step(th, ids, g, m, v, step, 2e-2, 0.9, 0.99, 0.0)
        assert np.allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_closed_forms():
    g = np.array([3.0, -0.5, 0.0, 1e-3])
    th = np.array([1.0, 1.0, 1.0, 1.0])
    # first step: m^ = g, v^ = g^2, so the step is lr * g / (|g| + eps)
    t1, m, v = P.adam_step(th, g, 0 * g, 0 * g, 1, lr=0.1, eps=1e-8)
    assert np.allclose(t1, th - 0.1 * g / (np.abs(g) + 1e-8), rtol=1e-13)
    # a constant gradient keeps m^ = g and v^ = g^2 at every step: n equal steps
    t, m, v = th, 0 * g, 0 * g
    for step in range(1, 6):
        t, m, v = P.adam_step(t, g, m, v, step, lr=0.1, eps=1e-8)
    assert np.allclose(t, th - 5 * 0.1 * g / (np.abs(g) + 1e-8), rtol=1e-12)
    assert t[2] == 1.0                                           # zero gradient, zero moments: no move
    # rows that are not listed keep parameters and moments
    tab = np.arange(12.0).reshape(4, 3)
    mm, vv = np.full((4, 3), 0.5), np.full((4, 3), 0.25)
    t2, m2, v2 = P.adam_rows_step(tab, [2], np.ones((1, 3)), mm, vv, 3)
    assert np.array_equal(t2[[0, 1, 3]], tab[[0, 1, 3]]) and np.array_equal(m2[[0, 1, 3]], mm[[0, 1, 3]])
    assert np.array_equal(v2[[0, 1, 3]], vv[[0, 1, 3]]) and not np.array_equal(t2[2], tab[2])
