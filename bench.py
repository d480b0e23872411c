#!/usr/bin/env python3
"""Benchmark of the sparse-embedding hot path on one MI355X.

One step = sfc_prepare + sfc_fetch_misses + sfc_lookup + sfc_backward_update over one seeded
synthetic batch whose ids already sit in HBM.  Prints ONE JSON line: whole-job raw ids/s, the
roofline of the dominant kernel (hipEvent-timed in this run on the batches that follow the timed
region, see roofline.timing_source) and the CPU oracle timed on a bounded sample of the same
workload.  An untimed fill phase first steps the seeded batch sequence until the cache is full
and evicting at a steady rate, whatever --warmup says.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(workload, kernel):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE counters, calibrated against a plain copy)
    as recorded in profiles/hbm_traffic.txt by an earlier rocprofv3 --pmc run; None if absent."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.txt")) as f:
            for line in f:
                p = line.split()
                if len(p) >= 4 and p[0] == workload and p[1] == kernel:
                    return float(p[2]) + float(p[3])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--max-fill-steps", type=int, default=400,
                    help="cap on the untimed fill phase that precedes the warm-up: batches of the seeded "
                         "sequence are stepped until the cache is full and evicting at a steady rate")
    ap.add_argument("--workload", default="c2", help="tiny | c1 | c2 | c3 | c4 (see sfc_inputs.WORKLOADS)")
    ap.add_argument("--lookahead", type=int, default=2, choices=[0, 1, 2, 3],
                    help="L > 0: prepare/fetch of step t+L overlap lookup/update of step t; with 2 "
                         "(default) the copies of step t+1 also overlap the prepare of step t+2; 3 adds a step "
                         "context")
    ap.add_argument("--optimizer", default="adagrad", choices=["adagrad", "adam", "rowwise_adagrad"],
                    help="adagrad is the benchmark's; adam is the paper's (state 2x the row)")
    ap.add_argument("--strategy", default="cache", choices=["cache", "host", "prefetch"],
                    help="the MixCache ablation's strategies: cache (MixCache, default), host (no cache, "
                         "nothing fetched ahead: capacity 0, lookahead 0), prefetch (no cache, next "
                         "batch's rows copied before the current update, stale by one step)")
    ap.add_argument("--align-floats", type=int, default=32,
                    help="pad each Host row block [weights | state] to a multiple of this many floats")
    ap.add_argument("--cache-rows", type=int, default=None, help="override the workload's cache size")
    ap.add_argument("--host-rows", type=int, default=None,
                    help="override the rows of the Host table (the ids are drawn over that range): for "
                         "workloads whose table the box cannot pin, e.g. c4 needs 128 GB")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-in-order", action="store_true",
                    help="skip the extra pass that times the calls of a step in order at lookahead 0")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="end with three plain 1 GiB device copies (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build is the one-GPU hot path; there is no multi-GPU exchange to run. "
            "Use --gpus 1.")
        sys.exit(2)

    import numpy as np
    import torch
    import sfc_inputs as si
    import __graft_entry__
    __graft_entry__.build_if_missing()          # loads what is built; compiles only if nothing is
    import paper_2104_08542_amd as sfc

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = si.WORKLOADS[args.workload]
    if args.host_rows is not None:
        import dataclasses
        w = dataclasses.replace(w, vocab=args.host_rows)
    K, W = args.steps, args.warmup
    D, V, C = w.dim, w.vocab, w.cache_rows
    if args.cache_rows is not None:
        C = args.cache_rows
    policy = None
    if args.strategy != "cache":
        C = 0
        args.lookahead = 0 if args.strategy == "host" else 1
        policy = sfc.SFC_POLICY_PREFETCH if args.strategy == "prefetch" else None
    R = 4 * D

    t0 = time.time()
    S = sfc.state_floats(args.optimizer, D)
    table = sfc.HostTable(V, D, optimizer=args.optimizer, align_floats=args.align_floats)
    chunk = max(1, (1 << 26) // D)
    for r0 in range(0, V, chunk):
        r1 = min(V, r0 + chunk)
        table.w_t[r0:r1].copy_(si.table_rows(w.seed, r0, r1, D, dev))
    table.acc_t.fill_(0.0 if args.optimizer == "adam" else w.init_acc)
    log("host table [%d, %d + %d] pinned and filled in %.1fs" % (V, D, S, time.time() - t0))

    cache = sfc.Cache(table, C, w.max_ids, w.n_bags, lr=w.lr, eps=w.eps, lookahead=args.lookahead,
                      device="cuda:0", policy=policy)
    out = torch.empty(w.n_bags, D, dtype=torch.float32, device=dev)
    grads = [w.batch_grads(i, dev) for i in range(4)]
    step_no = [0]          # next batch of the seeded sequence

    def next_batch():
        b = w.batch_ids(step_no[0], dev)
        step_no[0] += 1
        return b

    # One step = prepare + fetch_misses + lookup + backward_update.  With lookahead 1 the prepare
    # and fetch issued in an iteration belong to the next step and overlap this step's lookup and
    # update; every iteration still issues exactly one of each call.
    for _ in range(args.lookahead):          # fill the pipeline
        b0 = next_batch()
        cache.prepare(b0[0], b0[1])
        cache.fetch_misses()

    def run_steps(batches, k0=0, overlap=True):
        for i, b in enumerate(batches):
            g = grads[(k0 + i) % 4]
            if args.lookahead and overlap:
                # prepare first: it waits for what the main stream has been given so far, and
                # issued here that is the previous update (whose context it reuses), not this
                # step's lookup
                cache.prepare(b[0], b[1])
                cache.fetch_misses()
                cache.lookup(out)
                cache.backward_update(g)
            elif args.lookahead:
                # same calls, same kernels, but the next step's prepare is issued after this
                # step's update, so the two streams never run at the same time
                cache.lookup(out)
                cache.backward_update(g)
                cache.prepare(b[0], b[1])
                cache.fetch_misses()
                if args.lookahead > 1:
                    cache.stream.wait_stream(cache.side)   # lookup(t+1) would not wait for fetch(t+2)
            else:
                cache.prepare(b[0], b[1])
                cache.fetch_misses()
                cache.lookup(out)
                cache.backward_update(g)

    # Fill phase (untimed, independent of --warmup): the timed region must show the regime the
    # workload is defined for, a full cache that evicts on every step.  Batches of the seeded
    # sequence are stepped until the device reports evictions and their number has levelled off
    # (mean of the last 8 steps within 5 % of the 8 before), or until nothing can change any more
    # (a cache that holds the whole table never evicts: there the misses must level off instead).
    # The counters come from the pinned status block, so the loop never waits for the device
    # except where it reads them.
    t0 = time.time()
    hit_curve, ev_hist, miss_hist = {}, [], []
    fill_steps = 0
    never_evicts = C >= V or C == 0
    while fill_steps < args.max_fill_steps:
        run_steps([next_batch()], fill_steps)
        fill_steps += 1
        torch.cuda.synchronize()
        st, _ = cache.peek_stats()                     # of the most recently planned batch
        ev_hist.append(st["n_evict"]); miss_hist.append(st["n_miss"])
        if fill_steps % 10 == 1:
            hit_curve[step_no[0]] = round(st["n_hit"] / max(1, st["n_hit"] + st["n_miss"]), 4)
        if fill_steps >= 16:
            h = miss_hist if never_evicts else ev_hist
            a, b = sum(h[-8:]) / 8.0, sum(h[-16:-8]) / 8.0
            if (never_evicts or a > 0) and abs(a - b) <= 0.05 * max(a, b, 1.0):
                break
    cache.check()
    log("fill phase: %d steps in %.1fs, evictions per step now %d" % (fill_steps, time.time() - t0,
                                                                    ev_hist[-1] if ev_hist else 0))
    # warm-up proper: W untimed steps in the timed region's order
    for t in range(W):
        run_steps([next_batch()], t)
    torch.cuda.synchronize()

    batches = [next_batch() for _ in range(K)]
    n_ids_total = sum(b[0].numel() for b in batches)
    torch.cuda.synchronize()

    # pass 1: whole-job throughput, no instrumentation inside the timed region
    t_start = time.perf_counter()
    run_steps(batches)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start

    # pass 2: K more steps with hipEvents around every step call (the next batches of the same
    # sequence, so the cache keeps evolving as in training); device counters sampled on the way.
    # Kernel and call durations are taken with the two streams not overlapping, i.e. each kernel
    # has the GPU to itself as in the lookahead-0 order; pass 4 below times the calls again in the
    # overlapped order of the timed region.
    batches2 = [next_batch() for _ in range(K)]
    torch.cuda.synchronize()
    sfc.sfc_profile_enable(cache.h, 1)
    agg = dict(n_unique=0, n_hit=0, n_miss=0, n_evict=0, n_bypass=0, h2d_bytes=0, d2h_bytes=0)
    ns = 0
    for t in range(K):
        run_steps([batches2[t]], t, overlap=False)
        if t % max(1, K // 10) == 0:          # sample the device counters (each read synchronises)
            st = cache.stats()
            for k in agg:
                agg[k] += st[k]
            ns += 1
    prof = sfc.sfc_profile_read(cache.h)
    # pass 3: K more steps with events around the kernels inside backward_update as well
    batches3 = [next_batch() for _ in range(K)]
    torch.cuda.synchronize()
    sfc.sfc_profile_enable(cache.h, 2)
    run_steps(batches3, overlap=False)
    prof3 = sfc.sfc_profile_read(cache.h)
    for k in ("k_seg_stream", "k_seg_finish", "k_adagrad_rows"):
        prof[k] = prof3[k]
    overlapped_ms = None
    if args.lookahead:
        # pass 4: call durations in the overlapped order of the timed region
        batches4 = [next_batch() for _ in range(K)]
        torch.cuda.synchronize()
        sfc.sfc_profile_enable(cache.h, 1)
        run_steps(batches4)
        p4 = sfc.sfc_profile_read(cache.h)
        overlapped_ms = {k: (p4[k][0] / p4[k][1] if p4[k][1] else 0.0)
                         for k in ("prepare", "fetch_misses", "lookup", "backward_update")}
    sfc.sfc_profile_enable(cache.h, 0)
    ms = {k: (v[0] / v[1] if v[1] else 0.0) for k, v in prof.items()}
    avg = {k: v / ns for k, v in agg.items()}
    N = n_ids_total / K
    U = avg["n_unique"]
    bags = w.n_bags

    # algorithmic bytes per launch (rows counted once per unique id)
    extra = 0 if w.one_hot else 8 * bags
    b_lookup = 4 * N + 4 * U + U * R + bags * R + extra
    RS = R + 4 * S                                                    # a row and its optimizer state
    b_update = bags * R + 4 * N + 4 * U + 2 * U * RS + extra         # sfc_backward_update as a whole
    # With Adagrad and Adam the ids with at most two positions (outside the 8192 lowest virtual ids) are summed
    # by the optimizer kernel from their own gradient rows: that share of the gradient bytes is the
    # optimizer kernel's, not the stream's, and those rows make no trip through the common matrix.
    # Counted here on one batch of the timed passes (torch, outside every timed region).
    Pc = Uc = 0
    if args.optimizer in ("adagrad", "adam"):
        ids1 = batches2[0][0].reshape(-1)
        uq, inv, cnt = torch.unique(ids1, return_inverse=True, return_counts=True)
        first = torch.full((uq.numel(),), ids1.numel(), dtype=torch.int64, device=dev)
        first.scatter_reduce_(0, inv, torch.arange(ids1.numel(), device=dev), "amin")
        rank = torch.empty_like(first)
        rank[first.argsort()] = torch.arange(uq.numel(), device=dev)
        cold = (cnt <= 2) & (rank >= 8192)
        Uc, Pc = float(cold.sum().item()), float(cnt[cold].sum().item())
        del uq, inv, cnt, first, rank, cold
    g_stream = bags * R * (N - Pc) / N        # one-hot: a gradient row per position; bags: in proportion
    kernels = {
        # the lookup call is two kernels: the batch's rows are warmed into the memory-side cache, then gathered
        ("k_warm_rows+k_lookup_onehot" if w.one_hot else "k_warm_rows+k_lookup_bags"): (b_lookup, ms["lookup"]),
        # gradient rows of the other ids + grouping in, their common rows out
        "k_seg_stream": (g_stream + 4 * N + (U - Uc) * R + extra, ms["k_seg_stream"]),
        # slot per row, the cold ids' gradient rows, the other ids' common rows, row + state in and out
        "k_%s_rows" % args.optimizer: (4 * U + (bags * R - g_stream) + (U - Uc) * R + 2 * U * RS,
                                      ms["k_adagrad_rows"]),
    }
    dom = max(kernels, key=lambda k: kernels[k][1])
    ach = kernels[dom][0] / (kernels[dom][1] * 1e-3) / 1e9
    traffic = measured_traffic(w.name, dom)
    pair_bytes = b_lookup + b_update
    pair_ms = ms["lookup"] + ms["backward_update"]
    pair_kernel_ms = ms["lookup"] + ms["k_seg_stream"] + ms["k_seg_finish"] + ms["k_adagrad_rows"]
    link_ms = ms["fetch_misses"]

    # what plain copies reach over the same link, one direction at a time (pinned buffer, 256 MiB)
    hb = torch.empty(1 << 28, dtype=torch.uint8, pin_memory=True)
    db = torch.empty(1 << 28, dtype=torch.uint8, device=dev)
    copy_gbs = {}
    for name, src, dst in (("h2d", hb, db), ("d2h", db, hb)):
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(4):
            dst.copy_(src, non_blocking=True)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs[name] = 4 * (1 << 28) / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del hb, db

    result = {
        "metric": "raw ids/sec through prepare+fetch_misses+lookup+backward_update",
        "value": n_ids_total / wall,
        "unit": "ids/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": "%s: batch %d x %d fields%s, ids %s over %.3g rows, dim %d fp32, cache %d rows LRU, %s"
                        % (w.name, w.batch, w.fields,
                           "" if w.one_hot else " (bags of %d-%d ids)" % (w.bag_lo, w.bag_hi),
                           "uniform" if w.zipf_s is None else "Zipf(s=%.2f)" % w.zipf_s, V, D, C,
                           {"adagrad": "Adagrad", "adam": "Adam", "rowwise_adagrad": "row-wise Adagrad"}[args.optimizer]),
            "ids_per_step": N, "unique_per_step": U,
            "cold_ids_per_step": Uc, "cold_positions_per_step": Pc,
            "hit_rate": avg["n_hit"] / max(1.0, avg["n_hit"] + avg["n_miss"]),
            "miss_per_step": avg["n_miss"], "evict_per_step": avg["n_evict"],
            "bypass_per_step": avg["n_bypass"], "lookahead": args.lookahead,
            "strategy": args.strategy,
            "fill_steps": fill_steps,
            "hit_rate_by_batch": hit_curve,
            "host_to_gpu_rows_per_unique": avg["n_miss"] / max(1.0, U),
            "gpu_to_host_rows_per_unique": (avg["n_evict"] + avg["n_bypass"]) / max(1.0, U),
        },
        "roofline": {
            "bound": "hbm", "kernel": dom, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": ach / HBM_PEAK_GBS, "traffic": traffic,
            "algorithmic_bytes_per_launch": kernels[dom][0], "avg_ms": kernels[dom][1],
            "timing_source": "hipEvents that the kernel's dispatch records at its start and end, on its "
                             "own stream, in this run, pass 2: the same calls on the batches that "
                             "follow the timed region, issued so that the streams do not overlap "
                             "(each kernel has the GPU to itself)",
            "traffic_source": "profiles/hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an "
                              "earlier run of this command, calibrated against a copy kernel); not "
                              "measured in this run",
        },
        "kernels": {k: {"algorithmic_bytes": v[0], "avg_ms": v[1],
                        "GB/s": (v[0] / (v[1] * 1e-3) / 1e9 if v[1] else None)} for k, v in kernels.items()},
        "lookup_plus_update": {"algorithmic_bytes": pair_bytes, "avg_ms": pair_ms,
                               "GB/s": pair_bytes / (pair_ms * 1e-3) / 1e9,
                               "frac_of_hbm_peak": pair_bytes / (pair_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                               "what": "the durations of the lookup call's two kernels + the backward_update call "
                                       "between two events on its stream (its kernels and their launch gaps; with Adagrad and Adam two: "
                                       "the stream and the optimizer kernel, which also chains the stream's block-edge "
                                       "partials, so k_seg_finish reads 0)",
                               "kernel_ms_sum": pair_kernel_ms,
                               "frac_of_hbm_peak_kernel_time": (pair_bytes / (pair_kernel_ms * 1e-3) / 1e9
                                                                / HBM_PEAK_GBS) if pair_kernel_ms else None},
        "call_ms": {k: ms[k] for k in ("prepare", "fetch_misses", "lookup", "backward_update")},
        "kernel_ms": {"k_seg_stream": ms["k_seg_stream"], "k_seg_finish": ms["k_seg_finish"],
                      "k_%s_rows" % args.optimizer: ms["k_adagrad_rows"]},
        "call_ms_overlapped": overlapped_ms,
        "host_link": {"h2d_bytes_per_step": avg["h2d_bytes"], "d2h_bytes_per_step": avg["d2h_bytes"],
                      "GB/s": ((avg["h2d_bytes"] + avg["d2h_bytes"]) / (link_ms * 1e-3) / 1e9
                               if link_ms else None),
                      "copy_GB/s": copy_gbs,
                      # the time plain copies would need (the two directions side by side, each at
                      # its own measured rate) over the time the copies of a step take
                      "frac_of_measured_copy": (max(avg["h2d_bytes"] / copy_gbs["h2d"], avg["d2h_bytes"] / copy_gbs["d2h"])
                                                / 1e9 / (link_ms * 1e-3) if link_ms else None)},
    }

    if args.lookahead and args.strategy == "cache" and not args.no_in_order:
        # The same pair with the calls of a step in order and nothing else in flight: a second cache
        # with lookahead 0 on the same Host table and batch sequence, filled the same way.  In the
        # pipelined configuration above, lookup and update of step t run two steps after its prepare
        # and copies, when everything those wrote has left the caches; here they follow at once.
        for _ in range(args.lookahead):       # retire the steps that are still in flight
            cache.lookup(out)
            cache.backward_update(grads[0])
        cache.flush()
        cache.close()
        c0 = sfc.Cache(table, C, w.max_ids, w.n_bags, lr=w.lr, eps=w.eps, lookahead=0, device="cuda:0",
                       policy=policy)
        seq = [0]

        def step0(k):
            b = w.batch_ids(seq[0], dev); seq[0] += 1
            c0.prepare(b[0], b[1]); c0.fetch_misses(); c0.lookup(out); c0.backward_update(grads[k % 4])

        for k in range(fill_steps + W):
            step0(k)
        torch.cuda.synchronize()
        sfc.sfc_profile_enable(c0.h, 1)       # K steps with events around the calls only ...
        for k in range(K):
            step0(k)
        q = sfc.sfc_profile_read(c0.h)
        torch.cuda.synchronize()
        sfc.sfc_profile_enable(c0.h, 2)       # ... and K more with the update's kernels timed as well
        for k in range(K):
            step0(k)
        q2 = sfc.sfc_profile_read(c0.h)
        for k in ("k_seg_stream", "k_seg_finish", "k_adagrad_rows"):
            q[k] = q2[k]
        sfc.sfc_profile_enable(c0.h, 0)
        c0.check()
        m0 = {k: (v[0] / v[1] if v[1] else 0.0) for k, v in q.items()}
        calls0 = m0["lookup"] + m0["backward_update"]
        kern0 = m0["lookup"] + m0["k_seg_stream"] + m0["k_seg_finish"] + m0["k_adagrad_rows"]
        result["lookup_plus_update_calls_in_order"] = {
            "what": "lookahead 0: prepare, copies, lookup, update of one step in order on one cache, "
                    "nothing overlapped; the pipelined default above measures the same kernels two steps "
                    "after their inputs were written",
            "algorithmic_bytes": pair_bytes, "avg_ms": calls0,
            "frac_of_hbm_peak": pair_bytes / (calls0 * 1e-3) / 1e9 / HBM_PEAK_GBS if calls0 else None,
            "kernel_ms_sum": kern0,
            "frac_of_hbm_peak_kernel_time": pair_bytes / (kern0 * 1e-3) / 1e9 / HBM_PEAK_GBS if kern0 else None,
            "call_ms": {k: m0[k] for k in ("prepare", "fetch_misses", "lookup", "backward_update")},
            "kernel_ms": {k: m0[k] for k in ("k_seg_stream", "k_seg_finish", "k_adagrad_rows")},
        }
        cache = c0

    if not args.no_cpu_baseline:
        # The oracle as it stands, single-threaded, on the same workload: first steps of the same
        # seeded batch sequence from a cold oracle cache, on a dense copy of the host table taken
        # after the GPU run has been flushed into it (values differ from step 0, the work does not).
        from oracle import Oracle, state_floats as oracle_state_floats
        for _ in range(cache.lookahead):      # retire the steps that are still in flight
            cache.lookup(out)
            cache.backward_update(grads[0])
        cache.flush()
        t1 = time.time()
        ow = np.ascontiguousarray(table.w)
        oa = np.ascontiguousarray(table.acc[:, :oracle_state_floats(args.optimizer, D)])
        log("dense copy of the host table for the oracle in %.1fs" % (time.time() - t1))
        orc = Oracle(C, D, ow, oa, lr=w.lr, eps=w.eps, optimizer=args.optimizer,
                     strategy="prefetch" if args.strategy == "prefetch" else "cache")
        done_ids, steps_done, cpu_t = 0, 0, 0.0
        while cpu_t < args.cpu_seconds and steps_done < 50:
            ids, off = w.batch_ids(steps_done, dev)
            g = grads[steps_done % 4].cpu().numpy()
            ids_np = ids.cpu().numpy()
            off_np = None if off is None else off.cpu().numpy()
            t1 = time.perf_counter()
            orc.step(ids_np, g, off_np)
            cpu_t += time.perf_counter() - t1
            done_ids += ids_np.size
            steps_done += 1
            log("oracle step %d: %.2fs so far" % (steps_done, cpu_t))
        cpu_model = "unknown CPU"
        try:
            with open("/proc/cpuinfo") as f:
                for line in f:
                    if line.startswith("model name"):
                        cpu_model = line.split(":", 1)[1].strip()
                        break
        except OSError:
            pass
        result["cpu_baseline"] = {
            "value": done_ids / cpu_t, "unit": "ids/s", "cores": 1, "kind": "oracle",
            "sample": "first %d steps of the same seeded batch sequence from a cold cache, "
                      "%.1f s of single-thread oracle time (%s, %d logical CPUs)"
                      % (steps_done, cpu_t, cpu_model, os.cpu_count()),
        }
    if args.calibrate_copy:
        # a plain copy-like kernel of known size, with an instantiation nothing else in this
        # process uses (uint8 xor): 2^30 bytes read + 2^30 bytes written per launch, 3 launches
        a = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            torch.bitwise_xor(a, 3, out=b)
        torch.cuda.synchronize()
        del a, b
    cache.close()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
