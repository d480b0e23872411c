"""Shared test helpers: tiny host tables and an uncached dense trainer built on
library routines (numpy scatter-add in float64, torch.optim.Adagrad)."""
import numpy as np
import torch

import sfc_inputs as si


def make_table(V, D, seed=5, init_acc=0.1):
    w = si.table_rows(seed, 0, V, D).numpy().copy()
    a = np.full((V, D), init_acc, np.float32)
    return w, a


class DenseTrainer:
    """Plain table, no cache, no dedup: what the cached path must be invisible against.

    Gradient rows are scatter-added per raw id with numpy in float64 (one add
    per occurrence), rounded to fp32, and the table is stepped by torch's dense
    Adagrad.  Rows whose gradient is zero are left unchanged by that optimizer.
    """

    def __init__(self, w, acc0, lr=0.01, eps=1e-8):
        self.p = torch.nn.Parameter(torch.from_numpy(w.copy()))
        self.opt = torch.optim.Adagrad([self.p], lr=lr, lr_decay=0, weight_decay=0,
                                       initial_accumulator_value=float(acc0), eps=eps)

    def lookup(self, ids, offsets=None):
        w = self.p.detach().numpy().astype(np.float64)
        if offsets is None:
            return w[ids].astype(np.float32)
        out = np.zeros((len(offsets) - 1, w.shape[1]))
        bag = np.repeat(np.arange(len(offsets) - 1), np.diff(offsets))
        np.add.at(out, bag, w[ids])
        return out.astype(np.float32)

    def step(self, ids, grad, offsets=None):
        V, D = self.p.shape
        G = np.zeros((V, D), np.float64)
        if offsets is None:
            rows = grad.astype(np.float64)
        else:
            rows = grad.astype(np.float64)[np.repeat(np.arange(len(offsets) - 1), np.diff(offsets))]
        np.add.at(G, ids, rows)
        self.p.grad = torch.from_numpy(G.astype(np.float32))
        self.opt.step()

    @property
    def w(self):
        return self.p.detach().numpy()

    @property
    def acc(self):
        return self.opt.state[self.p]["sum"].numpy()


def close(a, b, rtol=1e-5, atol=1e-6):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return bool(np.all(np.abs(a - b) <= atol + rtol * np.abs(b)))
