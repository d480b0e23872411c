"""HIP path vs oracle for the optimizers other than element-wise Adagrad: Adam (the paper's
optimizer, Experiment settings) and row-wise Adagrad.  Same comparisons as the Adagrad parity
tests: every output of every call, cache state after each step, flushed Host tables."""
import numpy as np
import pytest

import sfc_inputs as si
from gpu_common import Pair, assert_close

pytestmark = pytest.mark.gpu

STATE0 = {"adam": 0.0, "rowwise_adagrad": 0.1}


@pytest.mark.parametrize("interleaved", [True, False])
@pytest.mark.parametrize("D", [4, 32, 80, 256])
@pytest.mark.parametrize("optimizer", ["adam", "rowwise_adagrad"])
def test_optimizer_steps_with_evictions_and_bypass(optimizer, D, interleaved):
    # cache smaller than some batches: rows and their state travel both ways on most steps, and
    # the larger batches leave bypass rows; D = 80 is a row width that does not divide a wavefront
    V = 5000
    p = Pair(V, D, C=600, max_ids=4096, optimizer=optimizer, init_acc=STATE0[optimizer],
             interleaved=interleaved, lr=0.02)
    saw_bypass = saw_evict = False
    for t in range(8):
        n = 3000 if t % 3 == 2 else 1200 + 37 * t
        ids = si.zipf_ids(n, 1.1, V, 90 + D, t).numpy()
        pr = p.step(ids, si.grads(n, D, 90 + D, t).numpy())
        saw_bypass |= pr.stats["n_bypass"] > 0
        saw_evict |= pr.stats["n_evict"] > 0
    assert saw_bypass and saw_evict
    p.finish(); p.close()


@pytest.mark.parametrize("optimizer", ["adam", "rowwise_adagrad"])
def test_optimizer_multihot_and_invalid_ids(optimizer):
    V, D, nb = 3000, 16, 900
    p = Pair(V, D, C=1000, max_ids=nb * 20, max_bags=nb, optimizer=optimizer,
             init_acc=STATE0[optimizer])
    for t in range(5):
        off = si.bag_offsets(nb, 0, 20, 33, t).numpy()
        ids = si.zipf_ids(int(off[-1]), 1.15, V, 33, t).numpy()
        ids[::97] = V + 5                       # out-of-range ids: the null entry
        p.step(ids, si.grads(nb, D, 33, t).numpy(), off)
    p.finish(); p.close()


@pytest.mark.parametrize("lookahead", [1, 2])
@pytest.mark.parametrize("optimizer", ["adam", "rowwise_adagrad"])
def test_optimizer_pipelined(optimizer, lookahead):
    # steps in flight together: Adam's bias correction must use each step's own batch number
    V, D = 6000, 8
    p = Pair(V, D, C=1000, max_ids=4096, lookahead=lookahead, optimizer=optimizer,
             init_acc=STATE0[optimizer])
    bs = []
    for t in range(12):
        n = 3500 if t % 5 == 0 else 300
        bs.append((si.zipf_ids(n, 1.02, V, 81, t).numpy(), si.grads(n, D, 81, t).numpy(), None))
    p.run_pipelined(bs, False)
    p.close()


def test_adam_capacity_zero_and_full_residency():
    # the Host strategy (every row bypasses) and a cache that never evicts give the same table
    V, D = 800, 16
    tabs = []
    for C in (0, V):
        p = Pair(V, D, C=C, max_ids=2048, optimizer="adam", init_acc=0.0)
        for t in range(5):
            ids = si.zipf_ids(1500, 1.1, V, 14, t).numpy()
            p.step(ids, si.grads(1500, D, 14, t).numpy())
        p.finish()
        tabs.append((p.table.w.copy(), p.table.acc.copy()))
        p.close()
    assert_close(tabs[0][0], tabs[1][0], "weights, C = 0 vs C = V")
    assert_close(tabs[0][1], tabs[1][1], "moments, C = 0 vs C = V")

