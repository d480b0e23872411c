"""Pins for the oracle's MixCache resolution and eviction policy (Host-Manager section)."""
import numpy as np
import pytest

from oracle import Oracle
from conftest import golden_ints
from helpers import make_table


def _run(o, ids, D):
    pr = o.prepare(np.asarray(ids))
    o.fetch_misses()
    o.lookup()
    o.backward_update(np.zeros((len(ids), D), np.float32))
    return pr


@pytest.mark.parametrize("lookahead", [0, 1])
def test_paper_mixcache_example(lookahead):
    g = golden_ints("mixcache_example.txt")
    D = 4
    w, a = make_table(32, D)
    o = Oracle(g["capacity"][0], D, w, a, lookahead=lookahead)
    pr1 = _run(o, g["batch1"], D)
    assert pr1.stats["n_hit"] == 0 and pr1.stats["n_miss"] == len(g["batch1"])  # cold start
    assert o.state()[0].tolist() == g["before"]
    pr2 = _run(o, g["batch2"], D)
    assert pr2.stats["n_hit"] == len(g["batch2"]) and pr2.stats["n_miss"] == 0
    pr3 = o.prepare(np.asarray(g["batch3"]))
    hits = [int(pr3.unique_ids[v]) for v in range(len(pr3.unique_ids)) if v not in pr3.miss_vids]
    assert hits == g["hit3"]
    assert pr3.unique_ids[pr3.miss_vids].tolist() == g["miss3"]
    assert pr3.evict_ids.tolist() == g["evicted3"]
    o.fetch_misses()
    assert o.state()[0].tolist() == g["after"]


class BruteCache:
    """Policy P1 re-derived from its statement with python lists: sort all slots."""

    def __init__(self, C, lookahead=0):
        self.C, self.la, self.t = C, lookahead, 0
        self.ids = [-1] * C
        self.stamp = [0] * C

    def step(self, uniq):
        self.t += 1
        t = self.t
        slot = {}
        miss = []
        for u in uniq:
            if u in self.ids:
                s = self.ids.index(u)
                self.stamp[s] = t
                slot[u] = s
            else:
                miss.append(u)
        free = [s for s in range(self.C) if self.ids[s] < 0]
        need = len(miss) - len(free)
        victims = []
        if need > 0:
            cand = sorted((self.stamp[s], s) for s in range(self.C)
                          if self.ids[s] >= 0 and self.stamp[s] < t - self.la)
            victims = [s for _, s in cand[:need]]
        evicted = sorted((s, self.ids[s]) for s in victims)
        avail = sorted(free + victims)
        for s in victims:
            self.ids[s] = -1
        nb = 0
        for i, u in enumerate(miss):
            if i < len(avail):
                s = avail[i]
                self.ids[s], self.stamp[s], slot[u] = u, t, s
            else:
                slot[u] = self.C + nb
                nb += 1
        return slot, miss, evicted, nb


@pytest.mark.parametrize("C,lookahead,vocab", [(8, 0, 20), (8, 1, 20), (5, 0, 40), (1, 0, 6),
                                               (0, 0, 10), (16, 1, 18), (12, 0, 13),
                                               (8, 2, 20), (16, 2, 18), (24, 2, 40),
                                               (8, 3, 20), (30, 3, 40)])
def test_p1_against_brute_force(C, lookahead, vocab):
    rng = np.random.default_rng(100 + C + lookahead)
    D = 2
    w, a = make_table(vocab, D)
    o = Oracle(C, D, w, a, lookahead=lookahead)
    bc = BruteCache(C, lookahead)
    prev_slot = {}
    for step in range(40):
        n = int(rng.integers(1, 14))
        ids = rng.integers(0, vocab, size=n)
        pr = o.prepare(ids)
        stamp_before = o.state()[1].copy()
        o.fetch_misses()
        o.lookup()
        o.backward_update(np.zeros((n, D), np.float32))
        slot, miss, evicted, nb = bc.step(pr.unique_ids.tolist())
        assert pr.unique_ids[pr.miss_vids].tolist() == miss
        assert [(int(s), int(i)) for s, i in zip(pr.evict_slots, pr.evict_ids)] == evicted
        assert pr.stats["n_bypass"] == nb
        assert {int(u): int(s) for u, s in zip(pr.unique_ids, pr.slot)} == slot
        sid, stamp = o.state()
        assert sid.tolist() == bc.ids and stamp.tolist() == bc.stamp
        # invariants the paper states
        t = step + 1
        resident = set(sid[sid >= 0].tolist())
        assert not (resident & set(pr.evict_ids.tolist()))          # evicted rows are gone
        assert len(resident) <= C
        assert not (set(pr.evict_ids.tolist()) & set(pr.unique_ids.tolist()))  # never a needed row
        assert all(stamp_before[s] < t - lookahead for s in pr.evict_slots)
        assert len(set(pr.miss_vids.tolist())) == len(pr.miss_vids)  # fetched at most once
        # a row shared by consecutive batches keeps its slot
        for u, s in slot.items():
            if u in prev_slot and prev_slot[u] < C and s < C and u in prev_resident:
                assert prev_slot[u] == s
        prev_slot, prev_resident = slot, resident
        # LRU: no survivor that was evictable is older than a victim
        if len(pr.evict_slots):
            newest_victim = max(stamp_before[s] for s in pr.evict_slots)
            surv = [stamp_before[s] for s in range(C)
                    if sid[s] >= 0 and stamp_before[s] < t - lookahead and s not in pr.evict_slots
                    and stamp[s] == stamp_before[s]]
            assert all(x >= newest_victim for x in surv)


def test_bypass_when_working_set_exceeds_cache():
    D = 2
    w, a = make_table(50, D)
    o = Oracle(4, D, w, a)
    pr = o.prepare(np.arange(10))
    assert pr.slot.tolist() == [0, 1, 2, 3, 4, 5, 6, 7, 8, 9]   # 4..9 are bypass rows C+j
    assert pr.stats["n_bypass"] == 6 and pr.stats["n_evict"] == 0
    o.fetch_misses()
    assert o.state()[0].tolist() == [0, 1, 2, 3]
    # nothing of the current batch may be evicted: all four slots are stamped t
    o.lookup(); o.backward_update(np.zeros((10, D), np.float32))
    pr = o.prepare(np.array([0, 1, 2, 3, 20, 21]))
    assert pr.stats["n_evict"] == 0 and pr.stats["n_bypass"] == 2
