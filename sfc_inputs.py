"""Seeded synthetic inputs for the sparse-embedding hot path.

This module only *generates data*: raw feature-id batches, multi-hot bag
offsets, upstream gradients and the initial contents of the host-resident
embedding table.  It contains none of the method's arithmetic (no unique, no
cache, no gather, no optimizer), so both the CPU oracle's tests and the GPU
path's tests/bench may draw their inputs from it.

Everything is a pure function of (seed, counters): a splitmix64-style integer
mixer turns a 64-bit counter into 64 random bits, using only wrapping int64
tensor arithmetic, so the same call gives the same integers on a CPU tensor and
on a GPU tensor.  The workloads stand in for the paper's Criteo-TB batches
(Experiment / Dataset: 26 categorical + 13 bucketised numerical fields = 39
one-hot fields per instance; feature frequencies follow a power law,
Introduction): ids are drawn from a bounded Zipf law over the vocabulary and
scattered over the row space by an affine bijection.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import torch

# --------------------------------------------------------------------------
# counter-based random bits
# --------------------------------------------------------------------------

_GOLDEN = -7046029254386353131        # 0x9E3779B97F4A7C15 as a signed int64
_M1 = -4658895280553007687            # 0xBF58476D1CE4E5B9
_M2 = -7723592293110705685            # 0x94D049BB133111EB


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical shift right of an int64 tensor (torch's >> is arithmetic)."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function on an int64 tensor (wrapping arithmetic)."""
    z = x + _GOLDEN
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def _stream_key(seed: int, stream: int, step: int) -> int:
    """A 64-bit base counter for (seed, stream, step), as a signed python int."""
    k = (seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03
         + step * 0x2545F4914F6CDD1D + 0x1234567) & 0xFFFFFFFFFFFFFFFF
    # one scalar mix round so that nearby (seed, step) pairs do not overlap
    k ^= k >> 31
    k = (k * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    k ^= k >> 29
    return k - (1 << 64) if k >= (1 << 63) else k


def random_bits(seed: int, stream: int, step: int, n: int, device="cpu",
                offset: int = 0) -> torch.Tensor:
    """n int64 tensors of 64 random bits for counters offset..offset+n-1."""
    ctr = torch.arange(offset, offset + n, dtype=torch.int64, device=device)
    return mix64(ctr * _GOLDEN + _stream_key(seed, stream, step))


def uniform01(bits: torch.Tensor) -> torch.Tensor:
    """53-bit uniform doubles in [0, 1) from 64 random bits."""
    return _lsr(bits, 11).to(torch.float64) * (2.0 ** -53)


# --------------------------------------------------------------------------
# bounded Zipf ranks by rejection-inversion (Hörmann & Derflinger 1996)
# --------------------------------------------------------------------------

def _h_integral(x, s):
    # integral of t^-s from 1 to x
    lx = torch.log(x) if isinstance(x, torch.Tensor) else math.log(x)
    t = (1.0 - s) * lx
    if isinstance(t, torch.Tensor):
        return torch.expm1(t) / (1.0 - s)
    return math.expm1(t) / (1.0 - s)


def _h_integral_inv(y, s):
    t = y * (1.0 - s)
    if isinstance(t, torch.Tensor):
        t = torch.clamp(t, min=-1.0 + 1e-16)
        return torch.exp(torch.log1p(t) / (1.0 - s))
    t = max(t, -1.0 + 1e-16)
    return math.exp(math.log1p(t) / (1.0 - s))


def zipf_ranks(n: int, s: float, vocab: int, seed: int, step: int,
               device="cpu", stream: int = 1) -> torch.Tensor:
    """n iid ranks k in [1, vocab] with P(k) proportional to k^-s (s != 1).

    Exact sampling: a candidate is drawn by inverting the integral of the
    continuous envelope x^-s over [0.5, vocab+0.5] and accepted by the
    rejection-inversion test; rejected lanes redraw with fresh counters.
    """
    assert s > 0 and abs(s - 1.0) > 1e-9 and vocab >= 1
    hx1 = _h_integral(1.5, s) - 1.0
    hn = _h_integral(vocab + 0.5, s)
    sc = 2.0 - _h_integral_inv(_h_integral(2.5, s) - 2.0 ** (-s), s)
    out = torch.zeros(n, dtype=torch.int64, device=device)
    todo = torch.arange(n, dtype=torch.int64, device=device)
    key = _stream_key(seed, stream, step)
    for rnd in range(64):
        if todo.numel() == 0:
            break
        bits = mix64((todo + rnd * n) * _GOLDEN + key)
        u = hn + uniform01(bits) * (hx1 - hn)
        x = _h_integral_inv(u, s)
        k = torch.clamp(torch.floor(x + 0.5), 1.0, float(vocab))
        acc = (k - x <= sc) | (u >= _h_integral(k + 0.5, s) - torch.exp(-s * torch.log(k)))
        out[todo[acc]] = k[acc].to(torch.int64)
        todo = todo[~acc]
    if todo.numel():
        raise RuntimeError("zipf_ranks: rejection loop did not terminate")
    return out


_SCATTER_A = 2654435761   # prime, coprime to every vocab 2^a 5^b used here
_SCATTER_B = 1013904223


def scatter_rank(rank: torch.Tensor, vocab: int) -> torch.Tensor:
    """Affine bijection rank -> row id on [0, vocab), so hot rows are not adjacent."""
    assert math.gcd(_SCATTER_A, vocab) == 1 and vocab < (1 << 31)
    return ((rank - 1) * _SCATTER_A + _SCATTER_B) % vocab


def zipf_ids(n: int, s: float, vocab: int, seed: int, step: int, device="cpu") -> torch.Tensor:
    return scatter_rank(zipf_ranks(n, s, vocab, seed, step, device), vocab)


def uniform_ids(n: int, vocab: int, seed: int, step: int, device="cpu") -> torch.Tensor:
    u = uniform01(random_bits(seed, 2, step, n, device))
    return torch.clamp((u * vocab).to(torch.int64), max=vocab - 1)


def bag_offsets(n_bags: int, lo: int, hi: int, seed: int, step: int, device="cpu") -> torch.Tensor:
    """CSR offsets [n_bags+1] with iid bag lengths uniform on {lo..hi}."""
    u = uniform01(random_bits(seed, 3, step, n_bags, device))
    lens = lo + torch.clamp((u * (hi - lo + 1)).to(torch.int64), max=hi - lo)
    off = torch.zeros(n_bags + 1, dtype=torch.int64, device=device)
    off[1:] = torch.cumsum(lens, 0)
    return off


# --------------------------------------------------------------------------
# host table initial values and gradients
# --------------------------------------------------------------------------

TABLE_STD = 0.01
# four 16-bit uniforms summed (Irwin-Hall, n=4), centred: integer in [-131070, 131070]
_IH_SCALE = TABLE_STD / math.sqrt(4.0 * (65536.0 ** 2 - 1.0) / 12.0)


def table_values(seed: int, flat_index: torch.Tensor) -> torch.Tensor:
    """fp32 initial value of table element flat_index (= row*dim + col).

    Approximately N(0, 0.01^2): a centred sum of four 16-bit uniforms scaled to
    std 0.01.  Integer arithmetic followed by one fp32 multiply, so the value is
    bit-identical wherever it is computed.
    """
    b = mix64(flat_index * _GOLDEN + _stream_key(seed, 4, 0))
    s4 = (b & 0xFFFF) + (_lsr(b, 16) & 0xFFFF) + (_lsr(b, 32) & 0xFFFF) + _lsr(b, 48)
    return (s4 - 131070).to(torch.float32) * torch.tensor(_IH_SCALE, dtype=torch.float32,
                                                            device=flat_index.device)


def table_rows(seed: int, row_start: int, row_end: int, dim: int, device="cpu") -> torch.Tensor:
    idx = torch.arange(row_start * dim, row_end * dim, dtype=torch.int64, device=device)
    return table_values(seed, idx).view(row_end - row_start, dim)


def table_rows_for_ids(seed: int, ids: torch.Tensor, dim: int) -> torch.Tensor:
    idx = ids.view(-1, 1) * dim + torch.arange(dim, dtype=torch.int64, device=ids.device)
    return table_values(seed, idx.reshape(-1)).view(-1, dim)


def grads(n_bags: int, dim: int, seed: int, step: int, device="cpu") -> torch.Tensor:
    """Upstream gradient w.r.t. the [bags, dim] lookup output, iid N(0,1) fp32."""
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + step * 7919 + 17) & 0x7FFFFFFFFFFFFFFF)
    return torch.randn(n_bags, dim, dtype=torch.float32, device=device, generator=g)


# --------------------------------------------------------------------------
# named workloads
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    fields: int
    vocab: int            # V, rows of the host table
    dim: int              # D
    cache_rows: int       # C
    zipf_s: Optional[float]   # None = uniform ids
    steps: int
    seed: int
    bag_lo: int = 1       # multi-hot: bag length range; 1..1 = one-hot
    bag_hi: int = 1
    lr: float = 0.01
    eps: float = 1e-8
    init_acc: float = 0.1

    @property
    def n_bags(self) -> int:
        return self.batch * self.fields

    @property
    def one_hot(self) -> bool:
        return self.bag_hi == 1

    @property
    def max_ids(self) -> int:
        return self.n_bags * self.bag_hi

    def batch_ids(self, step: int, device="cpu"):
        """(ids[N] int64, offsets[n_bags+1] int64 or None) for one step."""
        if self.one_hot:
            n, off = self.n_bags, None
        else:
            off = bag_offsets(self.n_bags, self.bag_lo, self.bag_hi, self.seed, step, device)
            n = int(off[-1].item())
        if self.zipf_s is None:
            ids = uniform_ids(n, self.vocab, self.seed, step, device)
        else:
            ids = zipf_ids(n, self.zipf_s, self.vocab, self.seed, step, device)
        return ids, off

    def batch_grads(self, step: int, device="cpu"):
        return grads(self.n_bags, self.dim, self.seed, step, device)


def _hbm_cache_rows(budget_bytes: float, dim: int) -> int:
    # weights + accumulator rows plus 12 B of slot metadata (id, stamp)
    return int(budget_bytes // (2 * 4 * dim + 12))


WORKLOADS = {
    # the five configurations of the benchmark definition, in order
    "tiny": Workload("tiny", 1024, 39, 10 ** 5, 16, 10 ** 4, 1.05, 20, 1000),
    "c1": Workload("c1", 16384, 39, 10 ** 7, 16, 10 ** 6, 1.1, 100, 1001),
    "c2": Workload("c2", 65536, 39, 10 ** 8, 32, 8 * 10 ** 6, 1.2, 200, 1002),
    "c3": Workload("c3", 32768, 26, 10 ** 8, 64, min(10 ** 8, _hbm_cache_rows(100e9, 64)),
                   1.1, 50, 1003, bag_lo=1, bag_hi=20),
    "c4": Workload("c4", 131072, 39, 10 ** 9, 16, 2 * 10 ** 7, None, 50, 1004),
}
