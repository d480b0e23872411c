"""The allocation-free variant of the segment sum (scratch in a fixed device array of the library)
against the ordinary entry point and the oracle, through the C ABI: two calls in a row, the second
on a smaller batch, then a size beyond the fixed array."""
import numpy as np
import pytest
import torch

import sfc_inputs as si
from gpu_common import Pair, assert_close

pytestmark = pytest.mark.gpu


def test_static_scratch_segment_sum_matches_the_allocating_one():
    import paper_2104_08542_amd as sfc
    V, D = 30_000, 32
    p = Pair(V, D, C=8000, max_ids=200_000)
    c, o = p.cache, p.orc
    for t, n in enumerate((200_000, 37_001, 5)):     # the second and third smaller than the first
        ids = si.zipf_ids(n, 1.2, V, 91, t).numpy()
        grad = si.grads(n, D, 91, t).numpy()
        d_grad = torch.from_numpy(grad).to(p.dev)
        pr = o.prepare(ids, None); o.fetch_misses(); o.lookup()
        c.prepare(torch.from_numpy(ids).to(p.dev)); c.fetch_misses(); c.lookup()
        U = pr.stats["n_unique"]
        ref = torch.full((n, D), 7.0, device=p.dev)
        got = torch.full((n, D), -7.0, device=p.dev)
        sfc.sfc_segment_sum(c.h, d_grad, ref)
        sfc.sfc_segment_sum_static(c.h, d_grad, got)
        torch.cuda.synchronize()
        assert torch.equal(got[:U], ref[:U]), "step %d: static and allocating variants differ" % t
        assert torch.all(got[U:] == -7.0)             # rows beyond the unique ids are not touched
        ocg = o.backward_update(grad, want_common_grad=True)
        assert_close(got[:U].cpu().numpy(), ocg, "common gradient (static scratch), step %d" % t)
        c.backward_update(d_grad)
    p.finish(); p.close()


def test_static_scratch_refuses_what_does_not_fit():
    import paper_2104_08542_amd as sfc
    # dim 256 at 2e6 positions needs 2 * 3049 blocks * (8 * 256 + 4) bytes = 12.5 MB > 8 MiB
    V, D, n = 1000, 256, 2_000_000
    p = Pair(V, D, C=1000, max_ids=n)
    ids = torch.from_numpy(si.zipf_ids(n, 1.2, V, 92, 0).numpy()).to(p.dev)
    c = p.cache
    c.prepare(ids); c.fetch_misses(); c.lookup()
    g = torch.zeros(n, D, device=p.dev)
    out = torch.empty(n, D, device=p.dev)
    with pytest.raises(sfc.SfcError) as e:
        sfc.sfc_segment_sum_static(c.h, g, out)
    assert e.value.code == sfc.SFC_ELIMIT and "scratch" in str(e.value)
    sfc.sfc_segment_sum(c.h, g, out)                  # the allocating entry point still takes it
    c.backward_update(g)
    p.close()
