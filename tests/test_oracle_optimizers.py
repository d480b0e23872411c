"""Pins for the oracle's other optimizers (Experiment settings: the paper trains with Adam and
counts its two moment rows as training state; row-wise Adagrad is the one-scalar-per-row variant
of the benchmark's Adagrad)."""
import numpy as np
import pytest
import torch

import sfc_inputs as si
from oracle import Oracle
from helpers import close


def _tables(V, D, S, seed=5, state0=0.0):
    w = si.table_rows(seed, 0, V, D).numpy().copy()
    return w, np.full((V, S), state0, np.float32)


def _dense_grad(V, D, ids, grad):
    G = np.zeros((V, D), np.float64)
    np.add.at(G, ids, grad.astype(np.float64))
    return G.astype(np.float32)


def test_adam_first_step_closed_form():
    # from zero moments the bias corrections cancel the (1 - beta) factors exactly:
    # m_hat = g, v_hat = g^2, so the first step moves every touched weight by lr * g / (|g| + eps)
    V, D, lr, eps = 40, 8, 0.05, 1e-8
    w, st = _tables(V, D, 2 * D)
    w0 = w.copy()
    ids = np.arange(0, V, 2)
    grad = si.grads(len(ids), D, 3, 0).numpy()
    o = Oracle(V, D, w, st, lr=lr, eps=eps, optimizer="adam", betas=(0.9, 0.999))
    o.step(ids, grad); o.flush()
    g = grad.astype(np.float64)
    assert close(w[ids], w0[ids] - lr * g / (np.abs(g) + eps), rtol=2e-6, atol=1e-7)
    assert np.array_equal(w[1::2], w0[1::2])                 # untouched rows: no decay, no move
    assert not st[1::2].any()
    assert close(st[ids, :D], 0.1 * g, rtol=2e-6) and close(st[ids, D:], 0.001 * g * g, rtol=1e-4, atol=1e-12)


def test_adam_equals_dense_library_adam_when_every_row_is_in_every_batch():
    # with all rows touched on every step the lazy update is the ordinary dense one
    V, D, lr, eps, betas = 30, 4, 0.01, 1e-8, (0.9, 0.999)
    w, st = _tables(V, D, 2 * D)
    p = torch.nn.Parameter(torch.from_numpy(w.copy()))
    opt = torch.optim.Adam([p], lr=lr, betas=betas, eps=eps)
    o = Oracle(7, D, w, st, lr=lr, eps=eps, optimizer="adam", betas=betas)   # small cache: rows travel
    rng = np.random.default_rng(1)
    for t in range(12):
        ids = np.concatenate([rng.permutation(V), rng.integers(0, V, 50)])
        grad = si.grads(len(ids), D, 8, t).numpy()
        o.step(ids, grad)
        p.grad = torch.from_numpy(_dense_grad(V, D, ids, grad))
        opt.step()
    o.flush()
    assert close(w, p.detach().numpy())
    assert close(st[:, :D], opt.state[p]["exp_avg"].numpy())
    assert close(st[:, D:], opt.state[p]["exp_avg_sq"].numpy(), atol=1e-9)


def test_adam_lazy_rows_match_library_sparse_adam():
    # torch's SparseAdam is the lazy variant: only rows present in the (coalesced) sparse gradient
    # move, with the global step in the bias correction.  It places eps slightly differently
    # (eps vs eps*sqrt(1-b2^t) beside sqrt(v)), invisible for gradients bounded away from zero:
    # every id once per batch, |g| >= 0.5.
    V, D, lr, eps, betas = 200, 4, 0.02, 1e-8, (0.9, 0.999)
    w, st = _tables(V, D, 2 * D)
    p = torch.nn.Parameter(torch.from_numpy(w.copy()))
    opt = torch.optim.SparseAdam([p], lr=lr, betas=betas, eps=eps)
    o = Oracle(64, D, w, st, lr=lr, eps=eps, optimizer="adam", betas=betas)
    for t in range(15):
        ids = np.random.default_rng(t).choice(V, 80, replace=False)
        grad = si.grads(len(ids), D, 21, t).numpy()
        grad = (np.sign(grad) * (np.abs(grad) + 0.5)).astype(np.float32)
        o.step(ids, grad)
        u = np.unique(ids)
        G = _dense_grad(V, D, ids, grad)[u]
        p.grad = torch.sparse_coo_tensor(torch.from_numpy(u)[None, :], torch.from_numpy(G), (V, D)).coalesce()
        opt.step()
    o.flush()
    assert close(w, p.detach().numpy(), rtol=1e-5, atol=1e-6)
    assert close(st[:, :D], opt.state[p]["exp_avg"].numpy(), rtol=1e-5, atol=1e-7)
    assert close(st[:, D:], opt.state[p]["exp_avg_sq"].numpy(), rtol=1e-5, atol=1e-9)


@pytest.mark.parametrize("optimizer,S", [("adam", 16), ("rowwise_adagrad", 1)])
def test_cache_is_invisible_for_every_optimizer(optimizer, S):
    # the cache only moves bytes: any capacity gives bit-identical tables
    V, D = 300, 8
    res = []
    for C in (0, 17, 300):
        w, st = _tables(V, D, S, state0=0.0 if optimizer == "adam" else 0.1)
        o = Oracle(C, D, w, st, lr=0.01, optimizer=optimizer)
        for t in range(10):
            ids = si.zipf_ids(150, 1.1, V, 4, t).numpy()
            o.step(ids, si.grads(len(ids), D, 4, t).numpy())
        o.flush()
        res.append((w, st))
    for w, st in res[1:]:
        assert np.array_equal(w, res[0][0]) and np.array_equal(st, res[0][1])


def test_rowwise_adagrad_equals_library_adagrad_on_rows_with_one_gradient_value():
    # if all D entries of a row's gradient are equal, mean_j g_j^2 = g^2: the row-wise rule and the
    # element-wise rule coincide, and the element-wise one is torch.optim.Adagrad
    V, D, lr, eps, acc0 = 60, 8, 0.01, 1e-8, 0.1
    w, st = _tables(V, D, 1, state0=acc0)
    p = torch.nn.Parameter(torch.from_numpy(w.copy()))
    opt = torch.optim.Adagrad([p], lr=lr, initial_accumulator_value=acc0, eps=eps)
    o = Oracle(16, D, w, st, lr=lr, eps=eps, optimizer="rowwise_adagrad")
    for t in range(10):
        ids = si.zipf_ids(80, 1.1, V, 6, t).numpy()
        g1 = si.grads(len(ids), 1, 6, t).numpy()
        grad = np.repeat(g1, D, axis=1)
        o.step(ids, grad)
        p.grad = torch.from_numpy(_dense_grad(V, D, ids, grad))
        opt.step()
    o.flush()
    assert close(w, p.detach().numpy())
    assert close(st[:, 0], opt.state[p]["sum"].numpy()[:, 0])


def test_rowwise_adagrad_accumulates_the_mean_square_of_the_row():
    # one step, one row: acc1 = acc0 + |g|^2 / D; the weights move along -g by lr / (sqrt(acc1) + eps),
    # so (w0 - w1) / g is the same number in every column; a sum instead of a mean, or a missing
    # square, changes it
    D, lr, eps, acc0 = 16, 0.1, 1e-8, 0.1
    w, st = _tables(4, D, 1, state0=acc0)
    w0 = w.copy()
    g = si.grads(1, D, 2, 0).numpy()
    o = Oracle(4, D, w, st, lr=lr, eps=eps, optimizer="rowwise_adagrad")
    o.step(np.array([2]), g); o.flush()
    acc1 = acc0 + float(np.linalg.norm(g.astype(np.float64)) ** 2) / D
    assert close(st[2, 0], acc1, rtol=1e-6)
    assert close((w0[2] - w[2]) / g[0], np.full(D, lr / (np.sqrt(acc1) + eps)), rtol=1e-4)
    assert np.array_equal(st[[0, 1, 3]], np.full((3, 1), acc0, np.float32))
