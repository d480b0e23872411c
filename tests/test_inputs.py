"""The seeded input generators: reproducible, in range, and distributed as stated."""
import numpy as np
import torch

import sfc_inputs as si


def test_reproducible_and_step_dependent():
    a = si.zipf_ids(5000, 1.1, 10 ** 6, 7, 3)
    assert torch.equal(a, si.zipf_ids(5000, 1.1, 10 ** 6, 7, 3))
    assert not torch.equal(a, si.zipf_ids(5000, 1.1, 10 ** 6, 7, 4))
    assert not torch.equal(a, si.zipf_ids(5000, 1.1, 10 ** 6, 8, 3))
    assert a.min() >= 0 and a.max() < 10 ** 6


def test_zipf_pmf_matches_power_law():
    V, s, n = 40, 1.2, 1_000_000
    r = si.zipf_ranks(n, s, V, 1, 0)
    assert r.min() == 1 and r.max() == V
    cnt = torch.bincount(r, minlength=V + 1)[1:].double().numpy()
    p = np.arange(1, V + 1, dtype=np.float64) ** -s
    p /= p.sum()
    chi2 = ((cnt - n * p) ** 2 / (n * p)).sum()
    assert chi2 < 90.0          # 39 dof: mean 39, 99.999th percentile ~ 86


def test_scatter_is_a_bijection():
    V = 10 ** 5
    ids = si.scatter_rank(torch.arange(1, V + 1), V)
    assert torch.unique(ids).numel() == V


def test_table_values_std_and_determinism():
    t = si.table_rows(5, 0, 20000, 16)
    assert abs(float(t.std()) - 0.01) < 2e-4 and abs(float(t.mean())) < 1e-4
    sub = si.table_rows_for_ids(5, torch.tensor([3, 19999, 0]), 16)
    assert torch.equal(sub, t[[3, 19999, 0]])
    assert torch.equal(si.table_rows(5, 100, 200, 16), t[100:200])


def test_workload_shapes():
    w = si.WORKLOADS["tiny"]
    ids, off = w.batch_ids(0)
    assert off is None and ids.numel() == 1024 * 39
    w3 = si.WORKLOADS["c3"]
    off = si.bag_offsets(1000, w3.bag_lo, w3.bag_hi, w3.seed, 0)
    lens = (off[1:] - off[:-1])
    assert lens.min() >= 1 and lens.max() <= 20 and abs(float(lens.double().mean()) - 10.5) < 0.6
    assert w3.cache_rows == w3.vocab     # a 100 GB cache holds the whole table: never evicts
