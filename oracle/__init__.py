"""ctypes binding of the CPU oracle (oracle/sfc_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this.
Arrays are numpy; the oracle updates host_w / host_acc in place.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sfc_oracle.cpp")
_LIB = os.path.join(_HERE, "libsfc_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no fused multiply-add contraction, -O2)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared",
                               _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


class _Stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in
                ("n_unique", "n_hit", "n_miss", "n_evict", "n_bypass", "n_invalid",
                 "h2d_bytes", "d2h_bytes")]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float
        lib.orc_create.restype = vp
        lib.orc_create.argtypes = [i64, i32, i64, vp, vp, f32, f32, i32, i32, ctypes.c_double, ctypes.c_double, i32]
        lib.orc_destroy.argtypes = [vp]
        lib.orc_prepare.restype = ctypes.c_int
        lib.orc_prepare.argtypes = [vp, vp, i64, vp, i64, vp, vp, vp, vp, vp, vp, ctypes.POINTER(_Stats)]
        lib.orc_fetch_misses.argtypes = [vp]
        lib.orc_lookup.argtypes = [vp, vp]
        lib.orc_backward_update.argtypes = [vp, vp, vp]
        lib.orc_flush.argtypes = [vp]
        lib.orc_get_state.argtypes = [vp, vp, vp, vp, vp]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


OPTIMIZERS = ("adagrad", "adam", "rowwise_adagrad")
STRATEGIES = ("cache", "prefetch")     # capacity 0 with "cache" is the ablation's Host strategy


def state_floats(optimizer, dim):
    """Floats of optimizer state that travel with one row."""
    return {"adagrad": dim, "adam": 2 * dim, "rowwise_adagrad": 1}[optimizer]


@dataclass
class Prepared:
    unique_ids: np.ndarray    # [U] int64, first-appearance order (global_id); -1 = null entry
    inverse: np.ndarray       # [N] int32 virtual id per position
    slot: np.ndarray          # [U] int32 cache slot per virtual id (>= C: bypass row, -1: null)
    miss_vids: np.ndarray     # [M] int32 virtual ids to fetch, ascending
    evict_ids: np.ndarray     # [K] int64 ids written back, ascending slot order
    evict_slots: np.ndarray   # [K] int32
    stats: dict


class Oracle:
    """One cache + host table pair, stepped with prepare/fetch/lookup/backward_update."""

    def __init__(self, capacity_rows, dim, host_w, host_acc, lr=0.01, eps=1e-8, lookahead=0,
                 optimizer="adagrad", betas=(0.9, 0.999), strategy="cache"):
        """host_acc is the optimizer state [V, S]: S = dim (adagrad: accumulators), 2*dim (adam:
        first moments then second moments) or 1 (rowwise_adagrad)."""
        self.S = state_floats(optimizer, dim)
        assert host_w.dtype == np.float32 and host_acc.dtype == np.float32
        assert host_w.flags.c_contiguous and host_acc.flags.c_contiguous
        assert host_w.shape[1] == dim and host_acc.shape == (host_w.shape[0], self.S)
        self.lib = _load()
        self.C, self.D, self.V = int(capacity_rows), int(dim), int(host_w.shape[0])
        self.host_w, self.host_acc = host_w, host_acc
        self.h = self.lib.orc_create(self.C, self.D, self.V, _ptr(host_w), _ptr(host_acc),
                                     lr, eps, lookahead, OPTIMIZERS.index(optimizer),
                                     betas[0], betas[1], STRATEGIES.index(strategy))
        assert self.h, "oracle: bad optimizer / strategy (prefetch needs capacity 0)"
        self.n_bags = 0
        self.n_unique = 0

    def __del__(self):
        if getattr(self, "h", None):
            self.lib.orc_destroy(self.h)
            self.h = None

    def prepare(self, ids, offsets=None) -> Prepared:
        ids = np.ascontiguousarray(ids, dtype=np.int64).reshape(-1)
        n = ids.size
        if offsets is not None:
            offsets = np.ascontiguousarray(offsets, dtype=np.int64)
            n_bags = offsets.size - 1
        else:
            n_bags = n
        uniq = np.empty(max(n, 1), np.int64)
        inv = np.empty(max(n, 1), np.int32)
        slot = np.empty(max(n, 1), np.int32)
        miss = np.empty(max(n, 1), np.int32)
        ev_ids = np.empty(max(n, 1), np.int64)
        ev_slots = np.empty(max(n, 1), np.int32)
        st = _Stats()
        rc = self.lib.orc_prepare(self.h, _ptr(ids), n, _ptr(offsets), n_bags, _ptr(uniq), _ptr(inv),
                                  _ptr(slot), _ptr(miss), _ptr(ev_ids), _ptr(ev_slots),
                                  ctypes.byref(st))
        if rc != 0:
            raise ValueError("oracle: malformed bag offsets")
        s = {k: int(getattr(st, k)) for k, _ in _Stats._fields_}
        self.n_bags, self.n_unique = n_bags, s["n_unique"]
        U, M, K = s["n_unique"], s["n_miss"], s["n_evict"]
        return Prepared(uniq[:U].copy(), inv[:n].copy(), slot[:U].copy(), miss[:M].copy(),
                        ev_ids[:K].copy(), ev_slots[:K].copy(), s)

    def fetch_misses(self):
        self.lib.orc_fetch_misses(self.h)

    def lookup(self) -> np.ndarray:
        out = np.empty((self.n_bags, self.D), np.float32)
        self.lib.orc_lookup(self.h, _ptr(out))
        return out

    def backward_update(self, grad, want_common_grad=False):
        grad = np.ascontiguousarray(grad, dtype=np.float32)
        assert grad.shape == (self.n_bags, self.D)
        cg = np.empty((self.n_unique, self.D), np.float32) if want_common_grad else None
        self.lib.orc_backward_update(self.h, _ptr(grad), _ptr(cg))
        return cg

    def flush(self):
        self.lib.orc_flush(self.h)

    def state(self, rows=False):
        slot_id = np.empty(self.C, np.int64)
        stamp = np.empty(self.C, np.int32)
        w = np.empty((self.C, self.D), np.float32) if rows else None
        a = np.empty((self.C, self.S), np.float32) if rows else None
        self.lib.orc_get_state(self.h, _ptr(slot_id), _ptr(stamp), _ptr(w), _ptr(a))
        return (slot_id, stamp, w, a) if rows else (slot_id, stamp)

    def step(self, ids, grad, offsets=None):
        """One whole step; returns (Prepared, lookup output)."""
        pr = self.prepare(ids, offsets)
        self.fetch_misses()
        out = self.lookup()
        self.backward_update(grad)
        return pr, out
