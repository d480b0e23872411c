"""HIP path vs CPU oracle, element by element (run with -m gpu on an MI355X)."""
import numpy as np
import pytest
import torch

import sfc_inputs as si
from gpu_common import Pair

pytestmark = pytest.mark.gpu

HASHED, DENSE = 1, 2        # sfc_config.index_kind (0 = automatic: dense for every table of these tests)


def _zipf_steps(p, V, n, s, seed, steps, **kw):
    for t in range(steps):
        ids = si.zipf_ids(n, s, V, seed, t).numpy()
        p.step(ids, si.grads(n, p.D, seed, t).numpy(), **kw)


def test_paper_examples_on_gpu():
    # VSI example + MixCache example (12 slots; 7 replaces 1, 8 takes the free slot)
    p = Pair(V=32, D=4, C=12, max_ids=64)
    z = lambda n: np.zeros((n, 4), np.float32)
    pr = p.step([1, 3, 2, 5, 4, 6, 12, 13, 14, 15, 9], z(11))
    pr = p.step([3, 2, 5, 4], z(4))
    pr = p.step([6, 7, 8], z(3))
    assert p.cache.state()[0].tolist() == [7, 3, 2, 5, 4, 6, 12, 13, 14, 15, 9, 8]
    p.finish(); p.close()
    p = Pair(V=8, D=4, C=8, max_ids=16)
    pr = p.step([1, 3, 2, 2, 3, 1], np.ones((6, 4), np.float32))
    assert p.cache.unique_ids[:3].tolist() == [1, 3, 2]
    assert p.cache.inverse[:6].tolist() == [0, 1, 2, 2, 1, 0]
    p.finish(); p.close()


@pytest.mark.parametrize("index_kind", [HASHED, DENSE])
def test_tiny_config_bypass_every_step(index_kind):
    w = si.WORKLOADS["tiny"]                  # U ~ 10.7k > C = 10k: bypass rows on every step
    p = Pair(w.vocab, w.dim, w.cache_rows, w.max_ids, seed=w.seed, index_kind=index_kind)
    saw_bypass = saw_evict = False
    for t in range(6):
        ids, _ = w.batch_ids(t)
        pr = p.step(ids.numpy(), w.batch_grads(t).numpy())
        saw_bypass |= pr.stats["n_bypass"] > 0
        saw_evict |= pr.stats["n_evict"] > 0
    assert saw_bypass and saw_evict
    p.finish(); p.close()


@pytest.mark.parametrize("index_kind", [HASHED, DENSE])
@pytest.mark.parametrize("lookahead", [0, 1])
def test_eviction_heavy_small_cache(lookahead, index_kind):
    V, D, n = 5000, 8, 3000                    # several scan tiles, ragged tails (3000 % 256, % 2048)
    p = Pair(V, D, C=1500, max_ids=4096, lookahead=lookahead, index_kind=index_kind)
    _zipf_steps(p, V, n, 1.05, 21, 10)
    p.finish(); p.close()


def test_ties_in_stamp_break_by_slot():
    # fill 100 slots in one step (all stamp 1), then need 7 victims among equal stamps
    p = Pair(V=1000, D=4, C=100, max_ids=256)
    p.step(np.arange(100), np.zeros((100, 4), np.float32))
    pr = p.step(np.arange(500, 507), np.ones((7, 4), np.float32))
    assert pr.evict_slots.tolist() == list(range(7))
    pr = p.step(np.array([99, 98, 600, 601, 602]), np.ones((5, 4), np.float32))
    assert pr.evict_slots.tolist() == [7, 8, 9]
    p.finish(); p.close()


@pytest.mark.parametrize("index_kind", [HASHED, DENSE])
def test_multihot_bags(index_kind):
    V, D, nb = 20000, 16, 1500
    p = Pair(V, D, C=4000, max_ids=nb * 20, max_bags=nb, index_kind=index_kind)
    for t in range(6):
        off = si.bag_offsets(nb, 1, 20, 31, t).numpy()
        ids = si.zipf_ids(int(off[-1]), 1.1, V, 31, t).numpy()
        p.step(ids, si.grads(nb, D, 31, t).numpy(), offsets=off)
    p.finish(); p.close()


def test_multihot_with_empty_bags_and_repeats_inside_a_bag():
    p = Pair(V=50, D=4, C=8, max_ids=64, max_bags=8)
    off = np.array([0, 0, 3, 3, 7, 8])
    ids = np.array([4, 4, 9, 1, 4, 30, 30, 2])
    p.step(ids, si.grads(5, 4, 1, 0).numpy(), offsets=off)
    p.finish(); p.close()


def test_capacity_zero_is_the_host_strategy():
    V, D, n = 3000, 8, 1000
    p = Pair(V, D, C=0, max_ids=1024)
    _zipf_steps(p, V, n, 1.1, 41, 4)
    p.finish(); p.close()


@pytest.mark.parametrize("index_kind", [HASHED, DENSE])
def test_degenerate_batches(index_kind):
    p = Pair(V=100, D=4, C=16, max_ids=512, index_kind=index_kind)
    g = lambda n, t: si.grads(n, 4, 77, t).numpy()
    p.step(np.zeros(0, np.int64), np.zeros((0, 4), np.float32))     # empty batch
    p.step(np.full(300, 42), g(300, 1))                              # one id, many times
    p.step(np.array([-5, 100, 10 ** 12, -1]), g(4, 2))               # only out-of-range ids
    p.step(np.array([3, -1, 3, 200, 7]), g(5, 3))                    # mixed
    p.step(np.arange(100)[::-1].copy(), g(100, 4))                   # all distinct, > C
    p.step(np.arange(512) % 100, g(512, 5))                          # n_ids == max_ids
    p.finish(); p.close()


@pytest.mark.parametrize("index_kind", [HASHED, DENSE])
def test_medium_zipf_many_tiles(index_kind):
    # 16384 x 39 positions like the second configuration, vocabulary shrunk so that the oracle
    # and its table stay small; cache small enough to evict from the third step on
    V, D, n = 10 ** 6, 16, 16384 * 39
    p = Pair(V, D, C=200_000, max_ids=n, index_kind=index_kind)
    for t in range(5):
        ids = si.zipf_ids(n, 1.1, V, 1001, t).numpy()
        p.step(ids, si.grads(n, D, 1001, t).numpy(), check_state=(t in (0, 4)))
    p.finish(); p.close()


@pytest.mark.parametrize("D", [4, 8, 16, 64, 80, 128, 256])
def test_row_widths(D):
    # every lane-group geometry of the row kernels (D/4 lanes per row, also a D that does not
    # divide the wavefront), with a hot id, mid-frequency ids and singletons in one batch
    V, n = 6000, 5000
    p = Pair(V, D, C=1200, max_ids=n + 37)
    for t in range(3):
        ids = si.zipf_ids(n + 37 * (t % 2), 1.3, V, 60 + D, t).numpy()
        p.step(ids, si.grads(ids.size, D, 60 + D, t).numpy())
    p.finish(); p.close()


def test_long_groups_cross_many_spans():
    # three ids own almost all of 300k positions: their groups span hundreds of wavefronts
    V, D, n = 500, 32, 300_000
    p = Pair(V, D, C=500, max_ids=n)
    rng = np.random.default_rng(11)
    r = rng.random(n)
    ids = np.where(r < 0.5, 3, np.where(r < 0.8, 5, np.where(r < 0.97, 8, rng.integers(0, V, n))))
    p.step(ids, si.grads(n, D, 12, 0).numpy())
    p.step(ids[::-1].copy(), si.grads(n, D, 12, 1).numpy())
    p.finish(); p.close()


@pytest.mark.parametrize("D,C,optimizer", [(4, 400, "adagrad"), (16, 0, "adagrad"), (80, 400, "adagrad"),
                                           (256, 7, "adagrad"), (16, 400, "adam"), (32, 0, "adam")])
def test_groups_cut_by_block_edges_are_updated_once(D, C, optimizer):
    # Adagrad and Adam path: the optimizer kernel itself adds up the partial sums of groups that the gradient
    # stream's blocks cut (a lane group per short run, the whole block for a run of many slots) and
    # updates those rows; here one id has a run of hundreds of slots, a dozen ids have runs of a few
    # slots, the rest close inside a block.  Row widths of one lane and of a whole wavefront, a width
    # that does not divide the wavefront, rows that bypass the cache (C = 0: every one; C = 7: most).
    V, n = 400, 150_000
    rng = np.random.default_rng(100 + D)
    r = rng.random(n)
    mid = 20 + (rng.integers(0, 12, n))
    ids = np.where(r < 0.45, 3, np.where(r < 0.85, mid, rng.integers(0, V, n)))
    p = Pair(V, D, C=C, max_ids=n, optimizer=optimizer, init_acc=0.0 if optimizer == "adam" else 0.1)
    p.step(ids, si.grads(n, D, 70 + D, 0).numpy())
    p.step(ids[::-1].copy(), si.grads(n, D, 70 + D, 1).numpy())
    p.finish(); p.close()


def test_frequent_ids_that_first_appear_late():
    # the grouping passes treat the lowest virtual ids (the early, usually frequent ones) in LDS and
    # rank the others with atomics: here the batch opens with 9000 distinct ids, so the frequent ids
    # that follow get virtual ids beyond that range and their long groups take the other path;
    # multi-hot as well, where the payload of a grouped entry is the bag, not the position
    V, D, n = 40_000, 16, 120_000
    rng = np.random.default_rng(21)
    head = rng.permutation(V)[:9000]
    r = rng.random(n - 9000)
    tail = np.where(r < 0.4, 39_000, np.where(r < 0.7, 39_001, np.where(r < 0.8, head[17],
                                                                        rng.integers(0, V, n - 9000))))
    ids = np.concatenate([head, tail])
    p = Pair(V, D, C=30_000, max_ids=n)
    p.step(ids, si.grads(n, D, 22, 0).numpy())
    p.step(np.concatenate([head[::-1], tail[::-1]]), si.grads(n, D, 22, 1).numpy())
    p.finish(); p.close()
    lens = rng.integers(0, 7, 30_000)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    m = int(offsets[-1])
    ids = np.concatenate([head, tail])[:m] if m <= n else None
    assert ids is not None
    p = Pair(V, D, C=30_000, max_ids=n, max_bags=lens.size)
    p.step(ids, si.grads(lens.size, D, 23, 0).numpy(), offsets)
    p.finish(); p.close()


def test_same_stream_and_separate_host_arrays():
    # copies on the main stream; Host weights and accumulators as two separate arrays
    V, D, n = 4000, 32, 2000
    p = Pair(V, D, C=1000, max_ids=2048, side_stream=False, interleaved=False)
    _zipf_steps(p, V, n, 1.2, 5, 4)
    p.finish(); p.close()


def test_hot_id_accumulation_stays_in_tolerance():
    # one id owns ~half of 400k positions: the segment sum has ~2e5 N(0,1) terms per element
    V, D, n = 1000, 32, 400_000
    p = Pair(V, D, C=1000, max_ids=n)
    rng = np.random.default_rng(3)
    ids = np.where(rng.random(n) < 0.5, 7, rng.integers(0, V, n))
    p.step(ids, si.grads(n, D, 9, 0).numpy())
    p.finish(); p.close()


def test_index_rebuild_after_many_evictions():
    # tiny cache, every step evicts almost everything: deleted index entries pile up and the
    # rebuild path runs many times; state must stay identical to the oracle throughout
    V, D = 100_000, 4
    p = Pair(V, D, C=64, max_ids=64, index_kind=HASHED)
    for t in range(60):
        ids = si.uniform_ids(64, V, 3, t).numpy()
        p.step(ids, si.grads(64, D, 3, t).numpy(), check_common=False)
    p.finish(); p.close()


def test_call_order_and_argument_errors():
    import paper_2104_08542_amd as sfc
    p = Pair(V=100, D=4, C=16, max_ids=32)
    c = p.cache
    ids = torch.arange(8, dtype=torch.int64, device="cuda:0")
    out = torch.empty(8, 4, device="cuda:0")
    for fn in (lambda: c.lookup(out), lambda: c.backward_update(out), c.fetch_misses):
        with pytest.raises(sfc.SfcError) as e:
            fn()
        assert e.value.code == sfc.SFC_ESTATE
    with pytest.raises(sfc.SfcError) as e:
        c.prepare(torch.zeros(33, dtype=torch.int64, device="cuda:0"))
    assert e.value.code == sfc.SFC_EINVAL
    c.prepare(ids)
    with pytest.raises(sfc.SfcError) as e:
        c.prepare(ids)
    assert e.value.code == sfc.SFC_ESTATE
    c.fetch_misses(); c.lookup(out); c.backward_update(out)
    p.close()


def test_step_limit():
    import paper_2104_08542_amd as sfc
    p = Pair(V=100, D=4, C=16, max_ids=32, max_steps=3)
    for t in range(3):
        p.step(np.arange(5) + t, np.zeros((5, 4), np.float32))
    with pytest.raises(sfc.SfcError) as e:
        p.cache.prepare(torch.arange(5, dtype=torch.int64, device="cuda:0"))
    assert e.value.code == sfc.SFC_ELIMIT
    p.close()


def _batches(V, D, n, s, seed, steps):
    return [(si.zipf_ids(n, s, V, seed, t).numpy(), si.grads(n, D, seed, t).numpy(), None)
            for t in range(steps)]


@pytest.mark.parametrize("index_kind", [HASHED, DENSE])
@pytest.mark.parametrize("lookahead", [1, 2, 3])
@pytest.mark.parametrize("sync_every_call", [True, False])
def test_pipelined_steps_match_sequential_oracle(sync_every_call, lookahead, index_kind):
    # prepare / fetch of later steps overlap lookup / update of the current one; the cache is
    # small enough to evict on every step and large enough never to bypass
    V, D, n = 20000, 32, 6000
    p = Pair(V, D, C=12000, max_ids=8192, lookahead=lookahead, index_kind=index_kind)
    p.run_pipelined(_batches(V, D, n, 1.05, 77, 12), sync_every_call)
    p.close()


@pytest.mark.parametrize("lookahead", [1, 2, 3])
@pytest.mark.parametrize("sync_every_call", [True, False])
def test_pipelined_steps_with_bypass_rows(sync_every_call, lookahead):
    # the working set of two consecutive batches exceeds the cache: rows bypass it, and a row that
    # bypassed in step t is missed again in step t+1 and must arrive with the update of step t
    V, D, n = 3000, 16, 2500
    p = Pair(V, D, C=500, max_ids=4096, lookahead=lookahead)
    expect = p.run_pipelined(_batches(V, D, n, 1.05, 78, 10), sync_every_call)
    assert min(pr.stats["n_bypass"] for pr, _ in expect[1:]) > 0
    p.close()


@pytest.mark.parametrize("lookahead", [2, 3])
def test_pipelined_mixed_bypass_and_none(lookahead):
    # steps with and without bypass rows alternate, so the Host copies switch between the two
    # streams from step to step
    V, D = 6000, 8
    p = Pair(V, D, C=1000, max_ids=4096, lookahead=lookahead)
    bs = []
    for t in range(16):
        n = 3500 if t % 5 == 0 else 300
        bs.append((si.zipf_ids(n, 1.02, V, 80, t).numpy(), si.grads(n, D, 80, t).numpy(), None))
    expect = p.run_pipelined(bs, False)
    nb = [pr.stats["n_bypass"] for pr, _ in expect]
    assert max(nb) > 0 and min(nb) == 0
    p.close()


@pytest.mark.parametrize("lookahead", [1, 2, 3])
def test_pipelined_degenerate_batches(lookahead):
    # empty batches, a single id, only out-of-range ids and full-size batches in flight together
    V, D = 300, 4
    p = Pair(V, D, C=64, max_ids=512, lookahead=lookahead)
    g = lambda n, t: si.grads(n, D, 81, t).numpy()
    ids = [np.zeros(0, np.int64), np.full(300, 42), np.zeros(0, np.int64), np.array([-5, V, 10 ** 12, -1]),
           np.arange(512) % V, np.array([3, -1, 3, 200, 7]), np.zeros(0, np.int64), np.zeros(0, np.int64),
           np.arange(200)[::-1].copy(), np.arange(512) % 100]
    p.run_pipelined([(a, g(a.size, t), None) for t, a in enumerate(ids)], False)
    p.close()
    p = Pair(V, D, C=64, max_ids=512, lookahead=lookahead)
    p.run_pipelined([(a, g(a.size, t), None) for t, a in enumerate(ids)], True)
    p.close()


@pytest.mark.parametrize("lookahead", [1, 2, 3])
def test_pipelined_multihot(lookahead):
    V, D, nb = 8000, 8, 700
    p = Pair(V, D, C=5000, max_ids=nb * 20, max_bags=nb, lookahead=lookahead)
    bs = []
    for t in range(6):
        off = si.bag_offsets(nb, 1, 20, 79, t).numpy()
        bs.append((si.zipf_ids(int(off[-1]), 1.1, V, 79, t).numpy(), si.grads(nb, D, 79, t).numpy(), off))
    p.run_pipelined(bs, False)
    p.close()


@pytest.mark.parametrize("index_kind", [HASHED, DENSE])
@pytest.mark.parametrize("lookahead", [0, 2, 3])
def test_many_rebuilds_with_many_victims(lookahead, index_kind):
    # a cache much smaller than the id range with thousands of victims per step: the hashed index
    # fills with deleted entries and is rebuilt every few steps, also while other steps are in
    # flight; the dense one just follows
    V, D, n, C = 400_000, 4, 30_000, 40_000
    p = Pair(V, D, C=C, max_ids=n, lookahead=lookahead, index_kind=index_kind)
    bs = [(si.zipf_ids(n, 1.05, V, 77, t).numpy(), si.grads(n, D, 77, t).numpy(), None) for t in range(60)]
    if lookahead:
        expect = p.run_pipelined(bs, False)
        assert sum(pr.stats["n_evict"] for pr, _ in expect) > 5 * C
    else:
        ev = 0
        for ids, g, _ in bs:
            ev += p.step(ids, g, check_common=False, check_rows=False).stats["n_evict"]
        assert ev > 5 * C
        p.finish()
    p.close()


@pytest.mark.parametrize("max_ids", [1, 5, 16, 31])
def test_tiny_max_ids_with_id_zero(max_ids):
    # batch tables smaller than the 64 entries the unique pass always probes; id 0 is the value
    # that zero-filled memory would pass for
    V, D = 50, 4
    p = Pair(V, D, C=8, max_ids=max_ids)
    rng = np.random.default_rng(max_ids)
    for t in range(6):
        n = max_ids if t % 2 == 0 else max(1, max_ids // 2)
        ids = rng.integers(0, V, n)
        ids[rng.integers(0, n)] = 0
        if n > 2:
            ids[-1] = 0                      # id 0 again, later: its first appearance must win
        p.step(ids, si.grads(n, D, 90 + max_ids, t).numpy())
    p.finish(); p.close()


def test_malformed_offsets_are_reported_not_followed():
    # the oracle refuses such a batch; the device cannot be refused on the host (the offsets live
    # in device memory), so the kernels count the violations, stay inside their buffers and the
    # step is reported by sfc_check and in the stats
    import paper_2104_08542_amd as sfc
    from oracle import Oracle
    V, D = 200, 8
    ids = np.arange(40) % 23
    good = np.array([0, 5, 5, 17, 30, 40])
    cases = [np.array([1, 5, 5, 17, 30, 40]),          # does not start at 0
             np.array([0, 5, 5, 17, 30, 39]),          # does not end at n_ids
             np.array([0, 5, 5, 17, 30, 4000]),        # ends far outside
             np.array([0, 17, 5, 30, 30, 40]),         # decreasing
             np.array([0, -7, 5, 30, 30, 40])]         # negative
    for k, off in enumerate(cases):
        p = Pair(V, D, C=64, max_ids=64, max_bags=8)
        p.step(ids, si.grads(5, D, 3, 0).numpy(), offsets=good)       # a good step first
        tab = np.zeros((V, D), np.float32)
        with pytest.raises(ValueError):                 # the oracle's -1
            Oracle(64, D, tab.copy(), tab.copy()).prepare(ids.astype(np.int64), off.astype(np.int64))
        c = p.cache
        c.prepare(torch.from_numpy(ids).to(p.dev), torch.from_numpy(off.astype(np.int64)).to(p.dev))
        st = c.stats()
        assert st["n_bad_offsets"] >= 1, (k, st)
        c.fetch_misses()
        out = c.lookup()
        c.backward_update(torch.zeros(5, D, device=p.dev))
        torch.cuda.synchronize()
        assert out.shape == (5, D)
        with pytest.raises(sfc.SfcError) as e:
            c.check()
        assert e.value.code == sfc.SFC_EINVAL and "step 2" in str(e.value)
        c.check()                                       # reported once
        assert c.verify() == [0, 0, 0, 0]               # the manager state depends on the ids alone
        pk, step = c.peek_stats()
        assert step == 2 and pk["n_bad_offsets"] == st["n_bad_offsets"]
        p.close()


def test_status_block_needs_no_waiting():
    # counters and health of the latest planned step, read from pinned memory
    V, D, n = 5000, 8, 3000
    p = Pair(V, D, C=1500, max_ids=4096, lookahead=2)
    c = p.cache
    assert c.peek_stats()[1] == 0
    want = []
    for t in range(5):
        ids = si.zipf_ids(n, 1.05, V, 21, t).numpy()
        pr = p.orc.prepare(ids, None); p.orc.fetch_misses(); p.orc.lookup()
        p.orc.backward_update(si.grads(n, D, 21, t).numpy())
        want.append(pr.stats)
        c.prepare(torch.from_numpy(ids).to(p.dev)); c.fetch_misses()
        if t >= 2:
            c.lookup(); c.backward_update(si.grads(n, D, 21, t - 2).to(p.dev))
        c.check()
        torch.cuda.synchronize()
        pk, step = c.peek_stats()
        assert step == t + 1 and {k: pk[k] for k in want[t]} == want[t]
    p.close()


def test_discard_frees_a_step_that_was_only_read():
    import paper_2104_08542_amd as sfc
    V, D, n = 3000, 8, 800
    p = Pair(V, D, C=1000, max_ids=1024, lookahead=1)
    c = p.cache
    ids = [torch.from_numpy(si.zipf_ids(n, 1.1, V, 44, t).numpy()).to(p.dev) for t in range(4)]
    c.prepare(ids[0]); c.fetch_misses()
    c.prepare(ids[1]); c.fetch_misses()
    with pytest.raises(sfc.SfcError) as e:              # both contexts hold steps that were not updated
        c.prepare(ids[2])
    assert e.value.code == sfc.SFC_ESTATE
    a = c.lookup().clone()
    c.discard()                                          # step 1 given up, rows stay as they are
    c.prepare(ids[2]); c.fetch_misses()
    b = c.lookup().clone()                               # step 2
    c.discard()
    c.prepare(ids[0]); c.fetch_misses()                  # the ids of step 1 again: all hits now
    c.lookup(); c.discard()
    again = c.lookup()                                   # step 4 = ids[0]: same rows as the first lookup
    assert torch.equal(again, a)
    assert c.stats()["n_miss"] == 0
    c.discard()
    with pytest.raises(sfc.SfcError) as e:
        c.discard()
    assert e.value.code == sfc.SFC_ESTATE
    assert c.verify() == [0, 0, 0, 0]
    p.close()
