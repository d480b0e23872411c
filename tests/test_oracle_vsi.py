"""Pins for the oracle's Virtual Sparse Id step (Data-Loader section)."""
import numpy as np
import pytest

import sfc_inputs as si
from oracle import Oracle
from conftest import golden_ints
from helpers import make_table


def _oracle(V=64, D=4, C=16):
    w, a = make_table(V, D)
    return Oracle(C, D, w, a)


def test_paper_vsi_example():
    g = golden_ints("vsi_example.txt")
    pr = _oracle().prepare(np.array(g["batch"]))
    assert pr.unique_ids.tolist() == g["global_id"]
    assert pr.inverse.tolist() == g["virtual_id"]
    # the batch can be recovered from the two outputs: global_id indexed by virtual_id is the batch
    assert pr.unique_ids[pr.inverse].tolist() == g["batch"]


def _brute_force_vsi(ids):
    """O(N^2): an id's vid is the number of distinct ids whose first position is earlier."""
    n = len(ids)
    first = [min(q for q in range(n) if ids[q] == ids[p]) for p in range(n)]
    firsts = sorted(set(first))
    return [ids[f] for f in firsts], [firsts.index(f) for f in first]


@pytest.mark.parametrize("seed", range(6))
def test_vsi_brute_force_tiny(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 60))
    ids = rng.integers(0, 12, size=n)
    pr = _oracle().prepare(ids)
    u, inv = _brute_force_vsi(ids.tolist())
    assert pr.unique_ids.tolist() == u
    assert pr.inverse.tolist() == inv


def test_vsi_invariants_zipf_batch():
    w = si.WORKLOADS["tiny"]
    ids = w.batch_ids(0)[0].numpy()
    tw, ta = make_table(w.vocab, 4)
    pr = Oracle(100, 4, tw, ta).prepare(ids)
    U = len(pr.unique_ids)
    # every raw id maps to exactly one vid, vids are dense in [0, U)
    assert np.array_equal(np.unique(pr.inverse), np.arange(U))
    assert len(set(pr.unique_ids.tolist())) == U
    assert np.array_equal(pr.unique_ids[pr.inverse], ids)
    # the unique set is the library sort-unique; the order is first appearance
    su, first_idx = np.unique(ids, return_index=True)
    assert np.array_equal(np.sort(pr.unique_ids), su)
    assert np.array_equal(pr.unique_ids, ids[np.sort(first_idx)])
    assert pr.stats["n_unique"] == U and pr.stats["n_invalid"] == 0


def test_vsi_all_equal_and_all_distinct_and_empty():
    pr = _oracle().prepare(np.full(50, 7))
    assert pr.unique_ids.tolist() == [7] and not pr.inverse.any()
    pr = _oracle().prepare(np.arange(40)[::-1].copy())
    assert pr.unique_ids.tolist() == list(range(39, -1, -1))
    assert pr.inverse.tolist() == list(range(40))
    pr = _oracle().prepare(np.zeros(0, np.int64))
    assert pr.unique_ids.size == 0 and pr.inverse.size == 0 and pr.stats["n_unique"] == 0


def test_vsi_out_of_range_ids_collapse_to_null():
    o = _oracle(V=64)
    pr = o.prepare(np.array([5, -3, 64, 5, 1000, 2]))
    assert pr.unique_ids.tolist() == [5, -1, 2]
    assert pr.inverse.tolist() == [0, 1, 1, 0, 1, 2]
    assert pr.stats["n_invalid"] == 3
    assert pr.slot[1] == -1 and 1 not in pr.miss_vids.tolist()
