"""Synthetic click-through-rate mini-batches.

The paper trains on proprietary ads click logs (Section 7, Table 3: 100 to 500
non-zero features per example, thousands of examples per mini-batch, 30 to 60
bytes per sparse parameter).  Those logs cannot be had, so every input here is
drawn from a seeded generator with that shape: bags of uint64 feature keys whose
ids follow a bounded Zipf law over a pre-filled ("resident") id range, plus a
stated fraction of never-seen ids, and Gaussian upstream gradients.

Recipe (all draws from ``numpy.random.default_rng([seed, step])``):

* bag sizes: uniform on {lo..hi}, or max(1, Poisson(lam)) with lam chosen so that
  the mean bag size is the configured one;
* per key occurrence: with probability ``fresh_frac`` a fresh id, else a rank
  k ~ Zipf-Mandelbrot(s, q) on 1..n_prefill and id = k - 1;
* fresh ids: uniform on [n_prefill, universe) ("universe" mode) or a running
  counter starting at ``universe`` ("counter" mode: never reused);
* key = mix64(id), the SplitMix64 output function, a bijection on 64-bit words;
* the resident set is {mix64(i) : i < n_prefill};
* gradients ~ N(0, grad_std) as float32, one row per bag.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Iterator, Optional, Tuple

import numpy as np

_U64 = np.uint64


def mix64(x) -> np.ndarray:
    """SplitMix64 output function applied to the 64-bit state(s) ``x``.

    (Steele, Lea, Flood 2014; state 0 gives 0xE220A8397B1DCDAF.)
    """
    z = np.asarray(x).astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        z += _U64(0x9E3779B97F4A7C15)
        z ^= z >> _U64(30)
        z *= _U64(0xBF58476D1CE4E5B9)
        z ^= z >> _U64(27)
        z *= _U64(0x94D049BB133111EB)
        z ^= z >> _U64(31)
    return z


def prefill_keys(lo: int, hi: int) -> np.ndarray:
    """Keys of the resident ids lo..hi-1."""
    return mix64(np.arange(lo, hi, dtype=np.uint64))


class _Zipf:
    """Inverse-CDF sampler for p(k) ~ (k + q)^-s on k = 1..n_ranks.

    Ranks up to 2^20 use exact cumulative sums; the rest of the support uses the
    midpoint-rule integral of the density, inverted in closed form.
    """

    HEAD = 1 << 20

    def __init__(self, s: float, n_ranks: int, q: float = 0.0):
        assert n_ranks >= 1 and s > 0 and s != 1.0
        self.s, self.q, self.n = float(s), float(q), int(n_ranks)
        self.k0 = min(self.n, self.HEAD)
        w = (np.arange(1, self.k0 + 1, dtype=np.float64) + self.q) ** (-self.s)
        self.cum = np.cumsum(w)
        self.head_mass = float(self.cum[-1])
        if self.n > self.k0:
            a = self.k0 + 0.5 + self.q
            b = self.n + 0.5 + self.q
            e = 1.0 - self.s
            self.tail_mass = (b**e - a**e) / e
        else:
            self.tail_mass = 0.0

    def top_mass(self, k: int) -> float:
        """Probability of the k most frequent ranks (k <= HEAD)."""
        k = min(k, self.k0)
        return float(self.cum[k - 1]) / (self.head_mass + self.tail_mass)

    def sample(self, rng: np.random.Generator, size: int) -> np.ndarray:
        u = rng.random(size) * (self.head_mass + self.tail_mass)
        out = np.empty(size, dtype=np.int64)
        head = u < self.head_mass
        idx = np.searchsorted(self.cum, u[head], side="right")
        out[head] = np.minimum(idx, self.k0 - 1) + 1
        if self.tail_mass > 0.0:
            v = u[~head] - self.head_mass
            e = 1.0 - self.s
            a = self.k0 + 0.5 + self.q
            x = (a**e + v * e) ** (1.0 / e) - self.q
            k = np.floor(x + 0.5).astype(np.int64)
            out[~head] = np.clip(k, self.k0 + 1, self.n)
        else:
            out[~head] = self.k0
        return out


def zipf_ranks(rng: np.random.Generator, size: int, s: float, n_ranks: int,
               q: float = 0.0) -> np.ndarray:
    return _Zipf(s, n_ranks, q).sample(rng, size)


def _poisson_lambda_for_mean(mean: float) -> float:
    """lam with E[max(1, Poisson(lam))] = lam + exp(-lam) = mean."""
    lam = mean
    for _ in range(60):
        lam = mean - math.exp(-lam)
    return lam


@dataclass(frozen=True)
class Config:
    name: str
    n_prefill: int            # resident ids 0..n_prefill-1 inserted before step 0
    capacity: int             # maximum number of keys the table may ever hold
    dim: int
    n_examples: int           # B
    n_slots: int              # S
    bag_kind: str             # "uniform" or "poisson"
    bag_lo: int = 1
    bag_hi: int = 4           # uniform: sizes in {bag_lo..bag_hi}
    bag_mean: float = 5.0     # poisson: mean of max(1, Poisson)
    zipf_s: float = 1.05
    zipf_q: float = 0.0
    fresh_frac: float = 0.0
    fresh_mode: str = "universe"   # or "counter"
    universe: int = 1 << 40
    grad_std: float = 1e-3
    lr: float = 0.05
    eps: float = 1e-8
    init_acc: float = 0.1
    init_range: float = 0.01
    init_seed: int = 0
    seed: int = 0
    steps: int = 20

    @property
    def n_bags(self) -> int:
        return self.n_examples * self.n_slots


# The five workloads.  Resident counts leave head-room under ``capacity`` for
# the fresh keys of the stated number of steps, so that the table ends at most
# exactly full (capacity is a key count; the library sizes its slot array from it).
CONFIGS = {
    "tiny": Config("tiny", n_prefill=1 << 20, capacity=1 << 20, dim=8,
                   n_examples=512, n_slots=16, bag_kind="uniform", bag_lo=1, bag_hi=4,
                   zipf_s=1.1, lr=0.05, seed=0),
    "mid": Config("mid", n_prefill=(1 << 26) - (1 << 22), capacity=1 << 26, dim=16,
                  n_examples=4096, n_slots=100, bag_kind="poisson", bag_mean=5.0,
                  zipf_s=1.05, fresh_frac=0.05, fresh_mode="universe", lr=0.05, seed=2),
    "insert_heavy": Config("insert_heavy", n_prefill=(1 << 26) - 44_000_000, capacity=1 << 26,
                           dim=16, n_examples=8192, n_slots=100, bag_kind="poisson",
                           bag_mean=5.0, zipf_s=1.05, fresh_frac=0.20, fresh_mode="counter",
                           lr=0.05, seed=3, steps=50),
    "large": Config("large", n_prefill=1_000_000_000 - 40_000_000, capacity=1_000_000_000,
                    dim=16, n_examples=16384, n_slots=200, bag_kind="poisson", bag_mean=3.0,
                    zipf_s=1.05, fresh_frac=0.05, fresh_mode="counter", lr=0.05, seed=4),
    "skewed": Config("skewed", n_prefill=1 << 28, capacity=1 << 28, dim=64,
                     n_examples=16384, n_slots=64, bag_kind="poisson", bag_mean=8.0,
                     zipf_s=1.3, lr=0.02, seed=5),
    # The "top 1000 keys ~ 40 % of lookups" reading of the skewed workload:
    # Zipf-Mandelbrot with shift q = 222.
    "skewed_shifted": Config("skewed_shifted", n_prefill=1 << 28, capacity=1 << 28, dim=64,
                             n_examples=16384, n_slots=64, bag_kind="poisson", bag_mean=8.0,
                             zipf_s=1.3, zipf_q=222.0, lr=0.02, seed=5),
}


def scaled(cfg: Config, n_prefill: int, n_examples: int, n_slots: Optional[int] = None,
           capacity: Optional[int] = None, steps: Optional[int] = None) -> Config:
    """A smaller instance of ``cfg`` with the same distributions."""
    n_slots = cfg.n_slots if n_slots is None else n_slots
    steps = cfg.steps if steps is None else steps
    if capacity is None:
        per_step = n_examples * n_slots * (cfg.bag_mean if cfg.bag_kind == "poisson"
                                           else 0.5 * (cfg.bag_lo + cfg.bag_hi))
        capacity = n_prefill + int(math.ceil(1.25 * cfg.fresh_frac * per_step * steps)) + 64
    return dataclasses.replace(cfg, name=cfg.name + "_scaled", n_prefill=n_prefill,
                               capacity=capacity, n_examples=n_examples, n_slots=n_slots,
                               steps=steps)


@dataclass
class Batch:
    keys: np.ndarray          # uint64 [N]
    offsets: np.ndarray       # int32  [n_bags + 1], offsets[0] = 0, offsets[-1] = N
    grads: np.ndarray         # float32 [n_bags, dim]
    ids: np.ndarray           # uint64 [N] the ids behind the keys (id < n_prefill: resident)

    @property
    def n_keys(self) -> int:
        return int(self.keys.shape[0])


class BatchStream:
    """Deterministic sequence of mini-batches for one Config."""

    def __init__(self, cfg: Config):
        self.cfg = cfg
        self._zipf = _Zipf(cfg.zipf_s, cfg.n_prefill, cfg.zipf_q)
        self._next_fresh = int(cfg.universe)   # "counter" mode
        self._step = 0
        self._lam = (_poisson_lambda_for_mean(cfg.bag_mean)
                     if cfg.bag_kind == "poisson" else None)

    @property
    def zipf(self) -> _Zipf:
        return self._zipf

    def next(self) -> Batch:
        cfg = self.cfg
        rng = np.random.default_rng([cfg.seed, self._step])
        self._step += 1
        nb = cfg.n_bags
        if cfg.bag_kind == "uniform":
            sizes = rng.integers(cfg.bag_lo, cfg.bag_hi + 1, size=nb, dtype=np.int64)
        elif cfg.bag_kind == "poisson":
            sizes = np.maximum(1, rng.poisson(self._lam, size=nb)).astype(np.int64)
        else:
            raise ValueError(cfg.bag_kind)
        offsets = np.zeros(nb + 1, dtype=np.int64)
        np.cumsum(sizes, out=offsets[1:])
        n = int(offsets[-1])
        assert n < (1 << 31)
        ids = (self._zipf.sample(rng, n) - 1).astype(np.uint64)
        if cfg.fresh_frac > 0.0:
            fresh = rng.random(n) < cfg.fresh_frac
            nf = int(fresh.sum())
            if cfg.fresh_mode == "universe":
                ids[fresh] = rng.integers(cfg.n_prefill, cfg.universe, size=nf,
                                          dtype=np.uint64)
            elif cfg.fresh_mode == "counter":
                ids[fresh] = np.arange(self._next_fresh, self._next_fresh + nf,
                                       dtype=np.uint64)
                self._next_fresh += nf
            else:
                raise ValueError(cfg.fresh_mode)
        keys = mix64(ids)
        grads = rng.normal(0.0, cfg.grad_std, size=(nb, cfg.dim)).astype(np.float32)
        return Batch(keys=keys, offsets=offsets.astype(np.int32), grads=grads, ids=ids)

    def __iter__(self) -> Iterator[Batch]:
        while True:
            yield self.next()


def resident_split(cfg: Config, batch: Batch) -> Tuple[np.ndarray, np.ndarray]:
    """(unique resident keys, unique fresh keys) of a batch, each ascending."""
    res = batch.ids < np.uint64(cfg.n_prefill)
    return np.unique(batch.keys[res]), np.unique(batch.keys[~res])
