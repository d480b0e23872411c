"""Drives the HIP path and the CPU oracle side by side on the same seeded inputs and compares
every output of every call: bit-exact for ids / indices / counts / cache state, and within
1e-5 relative + 1e-6 absolute for fp32 values."""
import numpy as np
import torch

import sfc_inputs as si
from oracle import Oracle, state_floats as oracle_state_floats

RTOL, ATOL = 1e-5, 1e-6


def assert_close(a, b, what):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    assert a.shape == b.shape, (what, a.shape, b.shape)
    bad = np.abs(a - b) > ATOL + RTOL * np.abs(b)
    assert not bad.any(), "%s: %d of %d outside tolerance, worst abs err %.3e" % (
        what, int(bad.sum()), bad.size, float(np.abs(a - b).max()))


def same_stats(st, ost, table):
    """Counts are compared as they are; the byte counts after the library's padding of the
    row-wise accumulator to one 16-byte chunk is taken out."""
    if table.optimizer == "rowwise_adagrad":
        st = dict(st)
        scale = lambda b: b // (table.dim + 4) * (table.dim + 1)
        st["h2d_bytes"], st["d2h_bytes"] = scale(st["h2d_bytes"]), scale(st["d2h_bytes"])
    return {k: st[k] for k in ost} == ost and st["n_bad_offsets"] == 0


class Pair:
    """One HIP cache and one oracle over identical copies of a host table."""

    def __init__(self, V, D, C, max_ids, max_bags=None, lookahead=0, seed=5, lr=0.01, eps=1e-8,
                 init_acc=0.1, max_steps=0, side_stream=True, interleaved=True, device="cuda:0",
                 optimizer="adagrad", betas=(0.9, 0.999), strategy="cache", index_kind=0):
        import paper_2104_08542_amd as sfc
        self.sfc = sfc
        self.V, self.D, self.C = V, D, C
        self.dev = torch.device(device)
        self.table = sfc.HostTable(V, D, interleaved=interleaved, optimizer=optimizer)
        self.optimizer = optimizer
        chunk = max(1, (1 << 24) // D)
        for r0 in range(0, V, chunk):
            r1 = min(V, r0 + chunk)
            self.table.w_t[r0:r1] = si.table_rows(seed, r0, r1, D, self.dev).cpu()
        self.table.acc[:] = init_acc
        # the oracle's state has S floats per row; the library pads the row-wise accumulator to four
        self.ns = oracle_state_floats(optimizer, D)
        self.ow, self.oa = self.table.w.copy(), self.table.acc[:, :self.ns].copy()
        self.cache = sfc.Cache(self.table, C, max_ids, max_bags, lr=lr, eps=eps, lookahead=lookahead,
                               max_steps=max_steps, device=device, side_stream=side_stream, betas=betas,
                               policy=sfc.SFC_POLICY_PREFETCH if strategy == "prefetch" else None,
                               index_kind=index_kind)
        self.orc = Oracle(C, D, self.ow, self.oa, lr=lr, eps=eps, lookahead=lookahead,
                          optimizer=optimizer, betas=betas, strategy=strategy)

    def close(self):
        self.cache.close()
        self.table.free()

    def step(self, ids, grad, offsets=None, check_common=True, check_state=True, update=True,
             check_rows=True):
        """ids/offsets: int64 CPU tensors or numpy; grad: [bags, D] fp32.  Returns oracle's Prepared."""
        c, o = self.cache, self.orc
        ids_np = np.asarray(ids, np.int64)
        off_np = None if offsets is None else np.asarray(offsets, np.int64)
        grad_np = np.asarray(grad, np.float32)
        d_ids = torch.from_numpy(ids_np).to(self.dev)
        d_off = None if off_np is None else torch.from_numpy(off_np).to(self.dev)
        d_grad = torch.from_numpy(grad_np).to(self.dev)
        n = ids_np.size

        pr = o.prepare(ids_np, off_np)
        c.prepare(d_ids, d_off)
        st = c.stats()
        assert same_stats(st, pr.stats, self.table), (st, pr.stats)
        U, M = st["n_unique"], st["n_miss"]
        assert np.array_equal(c.unique_ids[:U].cpu().numpy(), pr.unique_ids), "unique_ids"
        assert np.array_equal(c.inverse[:n].cpu().numpy(), pr.inverse), "inverse"
        assert np.array_equal(c.slot[:U].cpu().numpy(), pr.slot), "slot"
        assert np.array_equal(c.miss_vids[:M].cpu().numpy(), pr.miss_vids), "miss_vids"

        o.fetch_misses()
        c.fetch_misses()
        if check_state and self.C:
            sid, stamp = c.state()
            osid, ostamp = o.state()
            assert np.array_equal(sid, osid), "slot_id after fetch"
            assert np.array_equal(stamp, ostamp), "stamp after fetch"

        out = c.lookup()
        assert_close(out.cpu().numpy(), o.lookup(), "lookup")
        if not update:
            c.discard()
            return pr
        if check_common:
            cg = c.segment_sum(d_grad)
            ocg = o.backward_update(grad_np, want_common_grad=True)
            assert_close(cg[:U].cpu().numpy(), ocg, "common gradient")
        else:
            o.backward_update(grad_np)
        c.backward_update(d_grad)
        if check_state and check_rows and self.C:
            _, _, w, a = c.state(rows=True)
            _, _, ow, oa = o.state(rows=True)
            res = o.state()[0] >= 0
            assert_close(w[res], ow[res], "cached rows after update")
            assert_close(a[res][:, :self.ns], oa[res], "cached optimizer state after update")
        return pr

    def finish(self, chunk_rows=1 << 20):
        self.cache.check()                    # nothing reported by the device on the way
        assert self.cache.verify() == [0, 0, 0, 0]   # index, slots and recency histogram recounted
        self.cache.flush()
        self.orc.flush()
        # chunked: identical chunks (rows never touched) are skipped by a plain memory compare
        for name, a, b in (("host weights", self.table.w, self.ow),
                           ("host optimizer state", self.table.acc, self.oa)):
            for r0 in range(0, self.V, chunk_rows):
                x, y = a[r0:r0 + chunk_rows, :b.shape[1]], b[r0:r0 + chunk_rows]
                if not np.array_equal(x, y):
                    assert_close(x, y, "%s after flush, rows %d.." % (name, r0))


    def run_pipelined(self, batches, sync_every_call):
        """Steps issued in pipelined order (lookahead L >= 1): prepare / fetch of step t+L go
        out between lookup and backward_update of step t.  The oracle runs the same steps one
        after the other.  With sync_every_call the device is drained after each call and every
        output of every step is compared; without it nothing waits until the end, so the side
        stream really overlaps the main one, and lookup outputs, final cache state and flushed
        tables are compared."""
        c, o = self.cache, self.orc
        dev = self.dev
        sync = torch.cuda.synchronize if sync_every_call else (lambda: None)
        T = len(batches)
        d_in = []
        for ids, grad, off in batches:
            d_in.append((torch.from_numpy(np.asarray(ids, np.int64)).to(dev),
                         torch.from_numpy(np.asarray(grad, np.float32)).to(dev),
                         None if off is None else torch.from_numpy(np.asarray(off, np.int64)).to(dev)))
        torch.cuda.synchronize()
        expect = []
        for ids, grad, off in batches:
            pr = o.prepare(np.asarray(ids, np.int64), None if off is None else np.asarray(off, np.int64))
            o.fetch_misses()
            out = o.lookup()
            o.backward_update(np.asarray(grad, np.float32))
            expect.append((pr, out))
        outs = []

        def check_prepared(t, b):
            if not sync_every_call:
                return
            pr = expect[t][0]
            st = c.stats()
            assert same_stats(st, pr.stats, self.table), (t, st, pr.stats)
            U, M, n = st["n_unique"], st["n_miss"], b.n_ids
            assert np.array_equal(b.unique_ids[:U].cpu().numpy(), pr.unique_ids), "unique_ids step %d" % t
            assert np.array_equal(b.inverse[:n].cpu().numpy(), pr.inverse), "inverse step %d" % t
            assert np.array_equal(b.slot[:U].cpu().numpy(), pr.slot), "slot step %d" % t
            assert np.array_equal(b.miss_vids[:M].cpu().numpy(), pr.miss_vids), "miss_vids step %d" % t

        L = max(1, c.lookahead)
        for t in range(min(L, T)):                  # fill the pipeline
            b = c.prepare(d_in[t][0], d_in[t][2]); sync(); check_prepared(t, b)
            c.fetch_misses(); sync()
        for t in range(T):
            outs.append(c.lookup()); sync()
            if t + L < T:
                b = c.prepare(d_in[t + L][0], d_in[t + L][2]); sync(); check_prepared(t + L, b)
                c.fetch_misses(); sync()
            c.backward_update(d_in[t][1]); sync()
        torch.cuda.synchronize()
        for t in range(T):
            assert_close(outs[t].cpu().numpy(), expect[t][1], "lookup of step %d" % t)
        if self.C:
            sid, stamp = c.state()
            osid, ostamp = o.state()
            assert np.array_equal(sid, osid) and np.array_equal(stamp, ostamp), "final cache state"
        self.finish()
        return expect
