"""Pins for the oracle's forward gather, gradient segment-sum, Adagrad update and
for the transparency of the cache (GPU-Worker section; MixCache consistency)."""
import numpy as np
import pytest
import torch

import sfc_inputs as si
from oracle import Oracle
from conftest import golden_ints
from helpers import DenseTrainer, close, make_table


def test_paper_forward_backward_example():
    g = golden_ints("forward_backward_example.txt")
    D = 4
    w, a = make_table(8, D)
    e = w.copy()
    o = Oracle(8, D, w, a)
    batch = np.asarray(g["batch"])
    pr = o.prepare(batch)
    o.fetch_misses()
    out = o.lookup()
    # recovered per-position embeddings [e1,e3,e2],[e2,e3,e1]
    assert np.array_equal(out, e[np.asarray(g["recovered_ids"])])
    grad = np.random.default_rng(0).standard_normal((6, D)).astype(np.float32)
    cg = o.backward_update(grad, want_common_grad=True)
    assert pr.unique_ids.tolist() == g["common_order"]
    for row, seg in zip(cg, g["segments"]):
        pos = [int(x) for x in seg.split(",")]
        assert close(row, grad[pos].astype(np.float64).sum(0))


def test_lookup_is_plain_table_indexing():
    wl = si.WORKLOADS["tiny"]
    ids = wl.batch_ids(0)[0].numpy()
    w, a = make_table(wl.vocab, wl.dim)
    table = w.copy()
    o = Oracle(wl.cache_rows, wl.dim, w, a)
    o.prepare(ids); o.fetch_misses()
    assert np.array_equal(o.lookup(), table[ids])


def test_multihot_lookup_is_embedding_bag_sum():
    V, D, nb = 300, 8, 200
    off = si.bag_offsets(nb, 1, 20, 9, 0).numpy()
    ids = si.zipf_ids(int(off[-1]), 1.1, V, 9, 0).numpy()
    w, a = make_table(V, D)
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(ids), torch.from_numpy(w).double(),
                                            torch.from_numpy(off[:-1]), mode="sum").numpy()
    o = Oracle(64, D, w, a)
    o.prepare(ids, off); o.fetch_misses()
    assert close(o.lookup(), ref, rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("multihot", [False, True])
def test_segment_sum_is_unsorted_segment_sum(multihot):
    V, D = 500, 8
    if multihot:
        off = si.bag_offsets(300, 1, 20, 3, 1).numpy()
        n, nb = int(off[-1]), 300
    else:
        off, n, nb = None, 2000, 2000
    ids = si.zipf_ids(n, 1.2, V, 3, 1).numpy()
    grad = si.grads(nb, D, 3, 1).numpy()
    w, a = make_table(V, D)
    o = Oracle(V, D, w, a)
    pr = o.prepare(ids, off); o.fetch_misses(); o.lookup()
    cg = o.backward_update(grad, want_common_grad=True)
    per_pos = grad if off is None else grad[np.repeat(np.arange(nb), np.diff(off))]
    ref = torch.zeros(len(pr.unique_ids), D, dtype=torch.float64).index_add_(
        0, torch.from_numpy(pr.inverse.astype(np.int64)), torch.from_numpy(per_pos).double()).numpy()
    assert close(cg, ref, rtol=1e-6, atol=1e-9)
    # column sums are preserved
    assert np.allclose(cg.astype(np.float64).sum(0), per_pos.astype(np.float64).sum(0), atol=1e-3)
    # with duplicates a per-occurrence (un-summed) update would differ: G of a repeated id
    # is the sum, not the last term
    v = np.bincount(pr.inverse).argmax()
    pos = np.nonzero(pr.inverse == v)[0]
    assert len(pos) > 1 and not close(cg[v], per_pos[pos[-1]])


def test_adagrad_one_step_closed_form():
    # from acc0 = 0.1 : acc1 = 0.1 + g^2 ; w1 = w0 - lr*g/(sqrt(acc1)+eps)
    D = 4
    w, a = make_table(4, D)
    w0 = w.copy()
    o = Oracle(4, D, w, a, lr=0.01, eps=1e-8)
    ids = np.array([2, 2, 0])
    grad = np.array([[1, -2, 0.5, 0], [3, 1, 0.5, 0], [0.25, 0, -1, 2]], np.float32)
    o.prepare(ids); o.fetch_misses(); o.lookup(); o.backward_update(grad); o.flush()
    G = {2: grad[0].astype(np.float64) + grad[1], 0: grad[2].astype(np.float64)}
    for i, g in G.items():
        acc1 = 0.1 + g * g
        assert close(a[i], acc1, rtol=1e-6, atol=0)
        assert close(w[i], w0[i] - 0.01 * g / (np.sqrt(acc1) + 1e-8), rtol=1e-6, atol=1e-9)
    # hand-computed scalar: g=4 -> acc=16.1, step = 0.01*4/sqrt(16.1) = 0.00996889...
    assert abs((w0[2, 0] - w[2, 0]) - 0.009968895) < 1e-7
    # eps sits outside the square root: with acc ~ 0 and g = 0 nothing moves
    assert np.array_equal(w[1], w0[1]) and np.array_equal(w[3], w0[3])
    assert np.array_equal(w[0, 1], w0[0, 1]) and a[0, 1] == np.float32(0.1)   # g == 0 column


@pytest.mark.parametrize("C,lookahead,multihot", [(0, 0, False), (7, 0, False), (64, 0, False),
                                                  (64, 1, False), (64, 2, False), (64, 3, False), (1000, 0, False),
                                                  (40, 0, True), (1000, 0, True)])
def test_cache_is_transparent(C, lookahead, multihot):
    """Training through the cache equals training a plain table (consistency of Host and
    Cache strategies), for any capacity including none at all."""
    V, D, steps = 400, 8, 12
    w, a = make_table(V, D)
    dense = DenseTrainer(w, 0.1)
    o = Oracle(C, D, w, a, lookahead=lookahead)
    for t in range(steps):
        if multihot:
            off = si.bag_offsets(60, 1, 20, 11, t).numpy()
            nb = 60
        else:
            off, nb = None, 256
        n = nb if off is None else int(off[-1])
        ids = si.zipf_ids(n, 1.1, V, 11, t).numpy()
        grad = si.grads(nb, D, 11, t).numpy()
        pr, out = o.step(ids, grad, off)
        assert close(out, dense.lookup(ids, off))        # sees every earlier update: no staleness
        dense.step(ids, grad, off)
    o.flush()
    assert close(w, dense.w) and close(a, dense.acc)


def test_results_do_not_depend_on_capacity():
    """The cache only moves bytes: final tables are bit-identical for every capacity."""
    V, D, steps = 300, 4, 10
    finals = []
    for C, la in [(0, 0), (5, 0), (50, 1), (50, 2), (300, 0)]:
        w, a = make_table(V, D)
        o = Oracle(C, D, w, a, lookahead=la)
        for t in range(steps):
            o.step(si.zipf_ids(128, 1.05, V, 2, t).numpy(), si.grads(128, D, 2, t).numpy())
        o.flush()
        finals.append((w, a))
    for w, a in finals[1:]:
        assert np.array_equal(w, finals[0][0]) and np.array_equal(a, finals[0][1])


def test_null_ids_read_zero_and_drop_gradient():
    D = 4
    w, a = make_table(10, D)
    w0 = w.copy()
    o = Oracle(4, D, w, a)
    ids = np.array([3, -1, 99, 3])
    pr = o.prepare(ids); o.fetch_misses()
    out = o.lookup()
    assert not out[1].any() and not out[2].any() and np.array_equal(out[0], w0[3])
    o.backward_update(np.ones((4, D), np.float32)); o.flush()
    touched = np.zeros(10, bool); touched[3] = True
    assert np.array_equal(w[~touched], w0[~touched]) and not np.array_equal(w[3], w0[3])
