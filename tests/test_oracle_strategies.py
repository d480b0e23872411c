"""Pins for the oracle's Host and Prefetch strategies (RQ3, the MixCache ablation: Host keeps
every row in host memory and fetches nothing ahead; Prefetch copies the next batch's rows before
the current batch is trained, without consistency)."""
import numpy as np
import torch

import sfc_inputs as si
from oracle import Oracle
from helpers import DenseTrainer, close, make_table

LR, EPS, ACC0 = 0.05, 1e-8, 0.1


def _adagrad_rows(w, a, g):
    """One step of torch's Adagrad on a gathered block of rows (library routine)."""
    p = torch.nn.Parameter(torch.from_numpy(w.copy()))
    opt = torch.optim.Adagrad([p], lr=LR, initial_accumulator_value=0.0, eps=EPS)
    opt.state[p]["sum"].copy_(torch.from_numpy(a))
    p.grad = torch.from_numpy(g)
    opt.step()
    return p.detach().numpy().copy(), opt.state[p]["sum"].numpy().copy()


def _batches(V, D, T, disjoint):
    out = []
    for t in range(T):
        if disjoint:        # consecutive batches share no id
            ids = np.random.default_rng(t).permutation(V // 2)[:40] * 2 + (t % 2)
            ids = np.concatenate([ids, ids[:7]])
        else:
            ids = si.zipf_ids(90, 1.1, V, 12, t).numpy()
        out.append((ids, si.grads(len(ids), D, 12, t).numpy()))
    return out


def test_host_strategy_is_the_uncached_dense_trainer():
    V, D = 120, 4
    w, a = make_table(V, D, init_acc=ACC0)
    ref = DenseTrainer(w, ACC0, lr=LR, eps=EPS)
    o = Oracle(0, D, w, a, lr=LR, eps=EPS)
    for ids, g in _batches(V, D, 8, False):
        pr, _ = o.step(ids, g)
        assert pr.stats["n_bypass"] == pr.stats["n_unique"] and pr.stats["n_hit"] == 0
        ref.step(ids, g)
    o.flush()
    assert close(w, ref.w) and close(a, ref.acc)


def test_prefetch_equals_host_when_consecutive_batches_share_no_row():
    # staleness is invisible if no row of batch t is in batch t+1
    V, D = 200, 4
    w, a = make_table(V, D, init_acc=ACC0)
    ref = DenseTrainer(w, ACC0, lr=LR, eps=EPS)
    o = Oracle(0, D, w, a, lr=LR, eps=EPS, strategy="prefetch")
    for ids, g in _batches(V, D, 9, True):
        o.step(ids, g)
        ref.step(ids, g)
    o.flush()
    assert close(w, ref.w) and close(a, ref.acc)


def test_prefetch_is_stale_by_exactly_one_step():
    # brute force with explicit snapshots of the Host table: batch t trains from snapshot t-2 and
    # overwrites its rows in snapshot t-1 to give snapshot t
    V, D, T = 60, 4, 10
    w, a = make_table(V, D, init_acc=ACC0)
    snaps = [(w.copy(), a.copy())]                     # snaps[k] = table after the write-back of batch k-1
    o = Oracle(0, D, w, a, lr=LR, eps=EPS, strategy="prefetch")
    overlap = 0
    prev = set()
    for t, (ids, g) in enumerate(_batches(V, D, T, False)):
        _, out = o.step(ids, g)
        u = np.unique(ids)
        overlap += len(prev & set(u.tolist())); prev = set(u.tolist())
        G = np.zeros((V, D)); np.add.at(G, ids, g.astype(np.float64))
        sw, sa = snaps[max(t - 1, 0)]                  # what the copy for batch t saw
        assert close(out, sw[ids])
        nw, na = _adagrad_rows(sw[u], sa[u], G[u].astype(np.float32))
        hw, ha = snaps[t][0].copy(), snaps[t][1].copy()
        hw[u], ha[u] = nw, na
        snaps.append((hw, ha))
    assert overlap > 50                                # the batches do share rows
    o.flush()
    assert close(w, snaps[-1][0]) and close(a, snaps[-1][1])
    ref = DenseTrainer(snaps[0][0], ACC0, lr=LR, eps=EPS)   # and so the result is not the consistent one
    for ids, g in _batches(V, D, T, False):
        ref.step(ids, g)
    assert not close(w, ref.w, rtol=1e-3, atol=1e-4)
