"""Parity at the full size of the target configuration (batch 65536 x 39 positions, dim 32,
1e8-row Host table, 8e6-slot cache), in the launch configuration bench.py times.

The oracle runs in lock step on its own copy of the Host table, so every output of every call is
compared element by element, as in the small tests.  Four batches of uniform ids fill the 8e6
slots (a Zipf batch brings only ~2.4e5 new ids), then Zipf batches run against the full cache, so
eviction, tombstones in the index and long hot groups are all exercised at full size.
The last five steps run pipelined at lookahead 2, the order and streams bench.py times.
Needs about 60 GB of host memory; skipped when the box has less.
"""
import sys
import time

import numpy as np
import psutil
import pytest

import sfc_inputs as si
from gpu_common import Pair

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[fullsize] " + msg, file=sys.__stderr__, flush=True)


def test_target_configuration_full_size():
    w = si.WORKLOADS["c2"]
    need = 2 * 2 * w.vocab * w.dim * 4 + 12e9
    if psutil.virtual_memory().available < need:
        pytest.skip("needs %.0f GB of free host memory" % (need / 1e9))
    t0 = time.time()
    p = Pair(w.vocab, w.dim, w.cache_rows, w.max_ids, seed=w.seed, lookahead=2)
    _say("tables ready after %.0fs" % (time.time() - t0))
    n = w.max_ids
    evicted = bypassed = 0
    # calls in order first: every output of every call compared
    for t in range(5):
        if t < 4:
            ids = si.uniform_ids(n, w.vocab, w.seed, t).numpy()       # ~2.5e6 new ids per step
        else:
            ids = w.batch_ids(t)[0].numpy()
        grad = w.batch_grads(t).numpy()
        pr = p.step(ids, grad, check_state=(t in (3, 4)), check_rows=False)
        evicted += pr.stats["n_evict"]
        bypassed += pr.stats["n_bypass"]
        _say("step %d: U=%d hit=%d miss=%d evict=%d, %.0fs" % (
            t, pr.stats["n_unique"], pr.stats["n_hit"], pr.stats["n_miss"], pr.stats["n_evict"],
            time.time() - t0))
    # then as bench.py issues them: prepare / copies two steps ahead on their own streams, nothing
    # waits; lookup outputs, final cache state and flushed tables are compared
    bs = [(w.batch_ids(t)[0].numpy(), w.batch_grads(t).numpy(), None) for t in range(5, 10)]
    expect = p.run_pipelined(bs, False)
    for pr, _ in expect:
        evicted += pr.stats["n_evict"]
        bypassed += pr.stats["n_bypass"]
    _say("5 pipelined steps and flushed tables compared after %.0fs" % (time.time() - t0))
    assert evicted > 1_000_000 and bypassed == 0
    # properties that hold at any size, on the last step's outputs
    c = p.cache
    ids = bs[-1][0]
    U = c.stats()["n_unique"]
    uniq = c.unique_ids[:U].cpu().numpy()
    inv = c.inverse[:n].cpu().numpy()
    assert np.array_equal(uniq[inv], ids)
    assert np.array_equal(np.sort(uniq), np.unique(ids))
    sid, _ = c.state()
    slot = c.slot[:U].cpu().numpy()
    assert np.array_equal(sid[slot], uniq)                 # every id of the batch is resident
    res = sid[sid >= 0]
    assert res.size == np.unique(res).size == w.cache_rows  # full cache, no id twice
    p.close()


def test_multihot_configuration_shape():
    """Batch shape of the multi-hot configuration (32768 x 26 bags of 1-20 ids, dim 64) with the
    vocabulary cut to 4e6 rows so that the oracle's table stays small; the cache holds the whole
    table, as in that configuration (compulsory misses only)."""
    w = si.WORKLOADS["c3"]
    V = 4_000_000
    t0 = time.time()
    p = Pair(V, w.dim, V, w.max_ids, max_bags=w.n_bags, seed=w.seed)
    for t in range(2):
        off = si.bag_offsets(w.n_bags, w.bag_lo, w.bag_hi, w.seed, t).numpy()
        ids = si.zipf_ids(int(off[-1]), w.zipf_s, V, w.seed, t).numpy()
        pr = p.step(ids, w.batch_grads(t).numpy(), offsets=off, check_state=False)
        _say("multi-hot step %d: N=%d U=%d, %.0fs" % (t, ids.size, pr.stats["n_unique"], time.time() - t0))
        assert pr.stats["n_evict"] == 0 and pr.stats["n_bypass"] == 0
    p.finish()
    p.close()


def test_low_locality_configuration_shape():
    """Batch shape of the low-locality stress configuration (131072 x 39 uniform ids, dim 16):
    nearly every position is its own virtual id and nearly every id misses; vocabulary and cache
    cut 25x (4e7 rows, 8e5 slots) at the same cache/vocabulary ratio."""
    w = si.WORKLOADS["c4"]
    V, C = 40_000_000, 800_000
    t0 = time.time()
    p = Pair(V, w.dim, C, w.max_ids, seed=w.seed)
    for t in range(3):
        ids = si.uniform_ids(w.max_ids, V, w.seed, t).numpy()
        pr = p.step(ids, w.batch_grads(t).numpy(), check_state=(t == 2), check_rows=False)
        _say("low-locality step %d: U=%d miss=%d evict=%d bypass=%d, %.0fs" % (
            t, pr.stats["n_unique"], pr.stats["n_miss"], pr.stats["n_evict"], pr.stats["n_bypass"],
            time.time() - t0))
    assert pr.stats["n_bypass"] > 0          # 5e6 new ids per step against 8e5 slots
    p.finish()
    p.close()


@pytest.mark.parametrize("lookahead,index_kind", [(0, 1), (2, 1), (2, 2)])
def test_long_run_keeps_every_resident_id_findable(lookahead, index_kind):
    """640 steps at the target batch size against a 2e6-row cache (about 1e5 victims per step; with
    the hashed index (index_kind 1) an index rebuild every few dozen steps), no oracle beside it:
    the device-side consistency checks must stay silent, the recount of the manager state must
    agree, and afterwards a batch made of resident ids must resolve to hits only."""
    import torch
    import paper_2104_08542_amd as sfc
    w = si.WORKLOADS["c2"]
    C = 2_000_000
    if psutil.virtual_memory().available < 2 * w.vocab * w.dim * 4 + 8e9:
        pytest.skip("needs the 1e8-row Host table")
    dev = torch.device("cuda:0")
    table = sfc.HostTable(w.vocab, w.dim)
    table.acc[:] = 0.1
    cache = sfc.Cache(table, C, w.max_ids, w.n_bags, lookahead=lookahead, max_steps=2000,
                      index_kind=index_kind)
    out = torch.empty(w.n_bags, w.dim, device=dev)
    g = w.batch_grads(0, dev)
    t0 = time.time()
    step = 0
    for _ in range(lookahead):
        cache.prepare(w.batch_ids(step, dev)[0]); cache.fetch_misses(); step += 1
    for t in range(640):
        ids = w.batch_ids(step, dev)[0]; step += 1
        if lookahead:
            cache.lookup(out); cache.prepare(ids); cache.fetch_misses(); cache.backward_update(g)
        else:
            cache.prepare(ids); cache.fetch_misses(); cache.lookup(out); cache.backward_update(g)
        if t % 80 == 79:
            st = cache.stats()                       # raises if a device check has fired
            assert st["n_evict"] > 50_000
    for _ in range(lookahead):
        cache.lookup(out); cache.backward_update(g)
    _say("640 steps at lookahead %d in %.0fs" % (lookahead, time.time() - t0))
    cache.check()
    assert cache.verify() == [0, 0, 0, 0]
    sid, _ = cache.state()
    res = sid[sid >= 0]
    assert res.size == C and np.unique(res).size == C
    probe = torch.from_numpy(np.random.default_rng(0).choice(res, 1_000_000, replace=False)).to(dev)
    for _ in range(lookahead + 1):                   # fills every step context
        cache.prepare(probe); cache.fetch_misses()
        st = cache.stats()
        assert st["n_miss"] == 0 and st["n_hit"] == st["n_unique"] == 1_000_000
    cache.close(); table.free()


def test_host_row_offsets_beyond_32_bits():
    """A 1e8-row Host table of dim 64 (51 GB pinned, the largest this box pins in one piece): Host
    row offsets beyond 2^31 sixteen-byte chunks and 2^32 bytes.  No oracle beside it (it would need
    a second table): the rows of the batch are planted on the host, and every output is checked
    against numpy and the planted values.  (Ids beyond 2^31 would need a table of more than 2^31
    rows, which cannot be pinned here.)"""
    import torch
    import paper_2104_08542_amd as sfc
    V, D, n, C = 100_000_000, 64, 20_000, 6_000
    need = V * 2 * D * 4 + 8e9
    if psutil.virtual_memory().available < need:
        pytest.skip("needs %.0f GB of free host memory" % (need / 1e9))
    t0 = time.time()
    dev = torch.device("cuda:0")
    try:
        table = sfc.HostTable(V, D)
    except sfc.SfcError as e:
        pytest.skip("cannot pin the table on this box: %s" % e)
    _say("1e8 x 64 table pinned after %.0fs" % (time.time() - t0))
    cache = sfc.Cache(table, C, n)
    rng = np.random.default_rng(3)
    planted = {}
    for t in range(3):
        ids = rng.integers(V // 2, V, size=n, dtype=np.int64)  # upper half: offsets beyond 2^31 chunks
        ids[:50] = V - 1 - np.arange(50)                      # the very end of the table
        ids[50:60] = [-7, V, V + 123, 2**40, -1, V, V, -2, 2**62, V + 1]   # outside [0, V): null entry
        ok = (ids >= 0) & (ids < V)
        for i in np.unique(ids[ok]):                          # plant weights / accumulators of new rows
            if int(i) not in planted:
                w = (np.arange(D) + (int(i) % 1000) * 1e-3).astype(np.float32)
                table.w[i] = w; table.acc[i] = 0.1
                planted[int(i)] = (w.copy(), np.full(D, 0.1, np.float32))
        d_ids = torch.from_numpy(ids).to(dev)
        g = np.full((n, D), 0.5, np.float32)
        cache.prepare(d_ids); cache.fetch_misses()
        out = cache.lookup().cpu().numpy()
        st = cache.stats()
        U = st["n_unique"]
        uniq = cache.unique_ids[:U].cpu().numpy()
        inv = cache.inverse[:n].cpu().numpy()
        canon = np.where(ok, ids, -1)
        assert np.array_equal(uniq[inv], canon)
        first = np.unique(canon, return_index=True)[1]
        assert np.array_equal(uniq, canon[np.sort(first)])    # first-appearance order
        assert st["n_invalid"] == int((~ok).sum())
        exp = np.stack([planted[int(i)][0] if 0 <= i < V else np.zeros(D, np.float32) for i in ids])
        assert np.array_equal(out, exp), "lookup rows"
        cache.backward_update(torch.from_numpy(g).to(dev))
        # host-side Adagrad on the planted copies: one update per id from the summed gradient
        cnt = dict(zip(*np.unique(ids[ok], return_counts=True)))
        for i, c in cnt.items():
            w, a = planted[int(i)]
            gs = np.float32(0.5 * c)
            a += gs * gs
            w -= np.float32(0.01) * gs / (np.sqrt(a) + np.float32(1e-8))
        _say("step %d with ids up to %d: U=%d miss=%d evict=%d bypass=%d" % (
            t, ids[ok].max(), U, st["n_miss"], st["n_evict"], st["n_bypass"]))
    cache.flush()
    for i, (w, a) in planted.items():
        assert np.allclose(table.w[i], w, rtol=1e-5, atol=1e-6) and np.allclose(table.acc[i], a, rtol=1e-5, atol=1e-6)
    cache.close(); table.free()
