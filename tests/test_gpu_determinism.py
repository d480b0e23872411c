"""What two runs of the same seeded sequence have in common.

The library promises: every integer result (unique ids, inverse, slots, miss lists, cache state)
and the lookup output are the same bit for bit in every run; so are the updated rows of ids with
at most two positions in a batch (their two gradient rows are added in a fixed order).  The
gradient sum of a more frequent id is an fp64 sum whose order follows the order in which the
grouping pass ranked the id's positions, which atomics decide: the fp64 sums of two runs differ in
their last bits, and once in a great while that moves the fp32 value they are rounded to by one
unit in the last place.  (The paper's backward pass is an unsorted segment sum: it fixes the
value, not the order.)  So two runs agree far inside the parity tolerance, and nearly everywhere
exactly; this test measures both."""
import numpy as np
import pytest
import torch

import sfc_inputs as si

pytestmark = pytest.mark.gpu


def _run(V, D, C, n, steps, seed, lookahead):
    import paper_2104_08542_amd as sfc
    dev = torch.device("cuda:0")
    table = sfc.HostTable(V, D)
    chunk = 1 << 22
    for r0 in range(0, V, chunk):
        r1 = min(V, r0 + chunk)
        table.w_t[r0:r1] = si.table_rows(seed, r0, r1, D, dev).cpu()
    table.acc[:] = 0.1
    cache = sfc.Cache(table, C, n, n, lookahead=lookahead)
    ints, outs = [], []
    ids = [si.zipf_ids(n, 1.2, V, seed, t, dev) for t in range(steps)]
    grads = [si.grads(n, D, seed, t, dev) for t in range(steps)]
    L = lookahead
    for t in range(min(L, steps)):
        cache.prepare(ids[t]); cache.fetch_misses()
    for t in range(steps):
        outs.append(cache.lookup().clone())
        if t + L < steps:
            b = cache.prepare(ids[t + L]); cache.fetch_misses()
            torch.cuda.synchronize()
            st = cache.stats()
            U, M = st["n_unique"], st["n_miss"]
            ints.append((st, b.unique_ids[:U].cpu().numpy().copy(), b.inverse[:n].cpu().numpy().copy(),
                         b.slot[:U].cpu().numpy().copy(), b.miss_vids[:M].cpu().numpy().copy()))
        cache.backward_update(grads[t])
    torch.cuda.synchronize()
    cache.check()
    assert cache.verify() == [0, 0, 0, 0]
    sid, stamp = cache.state()
    cache.flush()
    w, a = table.w.copy(), table.acc.copy()
    outs = [o.cpu().numpy() for o in outs]
    cache.close(); table.free()
    return ints, outs, (sid, stamp), w, a


def test_two_runs_of_one_seeded_sequence():
    V, D, C, n, steps = 20_000_000, 32, 1_600_000, 65536 * 39, 10     # the target batch shape
    r1 = _run(V, D, C, n, steps, 1002, 2)
    r2 = _run(V, D, C, n, steps, 1002, 2)
    # integer results: identical
    for (s1, u1, i1, l1, m1), (s2, u2, i2, l2, m2) in zip(r1[0], r2[0]):
        assert s1 == s2
        assert np.array_equal(u1, u2) and np.array_equal(i1, i2)
        assert np.array_equal(l1, l2) and np.array_equal(m1, m2)
    assert np.array_equal(r1[2][0], r2[2][0]) and np.array_equal(r1[2][1], r2[2][1])
    # the first lookup reads untouched rows: identical; later ones read updated rows
    assert np.array_equal(r1[1][0], r2[1][0])
    # flushed tables: within the parity tolerance everywhere, and identical nearly everywhere
    touched = 0
    for x, y, what in ((r1[3], r2[3], "weights"), (r1[4], r2[4], "accumulators")):
        d = x != y
        nd = int(d.sum())
        if nd:
            err = np.abs(x[d].astype(np.float64) - y[d])
            assert np.all(err <= 1e-6 + 1e-5 * np.abs(y[d])), what
            # one unit in the last place of the summed gradient moves a weight by far less than this
            rel = err / np.maximum(np.abs(y[d]), 1e-30)
            assert rel.max() < 1e-5, (what, rel.max())
        rows = np.unique(np.concatenate([s[1] for s in r1[0]])).size
        touched = rows * D
        print("%s: %d of %d updated elements differ between the two runs" % (what, nd, touched))
        assert nd <= max(10, touched // 1000), (what, nd, touched)
