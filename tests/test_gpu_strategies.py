"""HIP path vs oracle for the comparison strategies of the MixCache ablation (RQ3): Host is
capacity 0 (covered with the Adagrad parity tests as well), Prefetch copies the next batch's rows
before the current update and so trains rows that are stale by one step."""
import numpy as np
import pytest

import sfc_inputs as si
from gpu_common import Pair

pytestmark = pytest.mark.gpu

STATE0 = {"adam": 0.0}


@pytest.mark.parametrize("sync_every_call", [True, False])
@pytest.mark.parametrize("optimizer", ["adagrad", "adam"])
def test_prefetch_strategy_is_stale_by_one_step(optimizer, sync_every_call):
    # the ablation's Prefetch strategy: no cache, the next batch's rows copied before the current
    # update; Zipf batches share their hot rows, so every step trains stale rows
    V, D = 3000, 16
    p = Pair(V, D, C=0, max_ids=2048, lookahead=1, optimizer=optimizer, init_acc=STATE0.get(optimizer, 0.1),
             strategy="prefetch")
    bs = [(si.zipf_ids(1500 + 11 * t, 1.1, V, 71, t).numpy(), si.grads(1500 + 11 * t, D, 71, t).numpy(), None)
          for t in range(9)]
    p.run_pipelined(bs, sync_every_call)
    p.close()


def test_prefetch_strategy_argument_errors():
    import paper_2104_08542_amd as sfc
    t = sfc.HostTable(100, 4)
    for C, L in ((10, 1), (0, 0), (0, 2)):
        with pytest.raises(sfc.SfcError):
            sfc.Cache(t, C, 64, lookahead=L, policy=sfc.SFC_POLICY_PREFETCH)
    t.free()
