"""Quantised integer laws delivered as uint32 threshold tables.

Every random quantity of a sample path (arrival count per slot, request class,
prompt length l, decode length o) is drawn by inverting one 32-bit uniform word
``u`` against a non-decreasing table of thresholds::

    value = lo + #{ i : u >= thr[i] }            thr[i] = floor(F(lo + i) * 2**32)

so ``P(value <= lo + i) = thr[i] / 2**32`` and the largest value ``lo + len(thr)``
carries the remaining mass.  The tables are *inputs*: they are built here once,
in float64, and handed unchanged to whichever simulator consumes them, so no
transcendental function is ever evaluated on a sampled path.

This module holds input construction only.  It contains none of the scheduling
method's arithmetic (no workload formula, no stability bound, no simulation).
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
from scipy import special as _sp

TWO32 = 4294967296.0
U32_MAX = 4294967295


def _quantise(cdf: np.ndarray) -> np.ndarray:
    """floor(F * 2^32) clipped to uint32 and forced non-decreasing."""
    cdf = np.asarray(cdf, dtype=np.float64)
    thr = np.floor(cdf * TWO32)
    thr = np.clip(thr, 0.0, float(U32_MAX))
    thr = np.maximum.accumulate(thr) if thr.size else thr
    return thr.astype(np.uint32)


@dataclasses.dataclass(frozen=True)
class Law:
    """Integer law on ``{lo, lo+1, ..., lo+len(thr)}`` given by thresholds."""

    lo: int
    thr: np.ndarray  # uint32, non-decreasing, may be empty (point mass at lo)
    name: str = ""

    def __post_init__(self):
        t = np.ascontiguousarray(self.thr, dtype=np.uint32)
        object.__setattr__(self, "thr", t)
        if t.size > 1 and np.any(t[1:] < t[:-1]):
            raise ValueError("thresholds must be non-decreasing")

    @property
    def hi(self) -> int:
        return self.lo + int(self.thr.size)

    def values(self) -> np.ndarray:
        return np.arange(self.lo, self.hi + 1, dtype=np.int64)

    def pmf(self) -> np.ndarray:
        """Exact probability of each value under the quantised table."""
        edges = np.concatenate(([0.0], self.thr.astype(np.float64), [TWO32]))
        return np.diff(edges) / TWO32

    def moment(self, k: int = 1) -> float:
        v = self.values().astype(np.float64)
        return float(np.sum(self.pmf() * v**k))

    def sample(self, u: np.ndarray) -> np.ndarray:
        """Table inversion of uint32 words (used by tests of the tables)."""
        u = np.asarray(u, dtype=np.uint32)
        return self.lo + np.searchsorted(self.thr, u, side="right").astype(np.int64)


def point(v: int) -> Law:
    return Law(int(v), np.zeros(0, np.uint32), f"point({v})")


def from_pmf(lo: int, pmf) -> Law:
    pmf = np.asarray(pmf, dtype=np.float64)
    if pmf.ndim != 1 or pmf.size < 1 or np.any(pmf < 0):
        raise ValueError("bad pmf")
    cdf = np.cumsum(pmf / pmf.sum())[:-1]
    return Law(int(lo), _quantise(cdf), "pmf")


def uniform_int(lo: int, hi: int) -> Law:
    """Uniform on the integers lo..hi inclusive."""
    n = hi - lo + 1
    if n < 1:
        raise ValueError("empty range")
    cdf = np.arange(1, n, dtype=np.float64) / float(n)
    return Law(int(lo), _quantise(cdf), f"uniform[{lo},{hi}]")


def geometric(mean: float, cap: int | None = None) -> Law:
    """Geometric on {1,2,...} with success probability 1/mean, X = min(G, cap)."""
    p = 1.0 / float(mean)
    if not (0.0 < p <= 1.0):
        raise ValueError("mean must be >= 1")
    if cap is None:
        # stop where the tail falls below the table resolution
        cap = 1 if p >= 1.0 else int(math.ceil(-33.0 * math.log(2.0) / math.log1p(-p))) + 1
    v = np.arange(1, cap, dtype=np.float64)  # values 1..cap-1 get thresholds
    cdf = -np.expm1(v * math.log1p(-p)) if p < 1.0 else np.ones_like(v)
    return Law(1, _quantise(cdf), f"geometric(mean={mean},cap={cap})")


def lognormal(mu: float, sigma: float, lo: int, hi: int) -> Law:
    """X = clip(floor(Y), lo, hi), ln Y ~ N(mu, sigma^2)."""
    if hi < lo or lo < 1:
        raise ValueError("bad clip range")
    v = np.arange(lo, hi, dtype=np.float64)  # P(X <= v) = P(Y < v + 1) for v < hi
    cdf = _sp.ndtr((np.log(v + 1.0) - mu) / sigma)
    return Law(int(lo), _quantise(cdf), f"lognormal({mu},{sigma})[{lo},{hi}]")


def pareto(alpha: float, xmin: float, cap: int) -> Law:
    """X = min(floor(Y), cap), P(Y > y) = (xmin / y)^alpha for y >= xmin."""
    lo = int(math.floor(xmin))
    if cap < lo:
        raise ValueError("cap below xmin")
    v = np.arange(lo, cap, dtype=np.float64)
    cdf = 1.0 - np.power(xmin / np.maximum(v + 1.0, xmin), alpha)
    return Law(lo, _quantise(cdf), f"pareto({alpha},{xmin})cap{cap}")


def poisson_counts(lam: float) -> Law:
    """Number of arrivals in one slot, Poisson(lam), truncated at table resolution."""
    if not (lam >= 0.0) or lam > 64.0:
        raise ValueError("lam out of range for a count table")
    if lam == 0.0:
        return Law(0, np.zeros(0, np.uint32), "poisson(0)")
    cdf = []
    term = math.exp(-lam)
    acc = term
    k = 0
    while True:
        cdf.append(acc)
        if acc * TWO32 >= TWO32 - 0.5 or k > 400:
            break
        k += 1
        term *= lam / k
        acc += term
    thr = _quantise(np.minimum(np.array(cdf), 1.0))
    return Law(0, thr, f"poisson({lam!r})")


def bernoulli_counts(p: float) -> Law:
    if not (0.0 <= p <= 1.0):
        raise ValueError("p out of range")
    return Law(0, _quantise(np.array([1.0 - p])), f"bernoulli({p})")


def frac_threshold(frac: float) -> int:
    """uint32 threshold t with P(u < t) = floor(frac * 2^32) / 2^32."""
    if not (0.0 <= frac < 1.0):
        raise ValueError("fraction must be in [0,1)")
    return int(min(math.floor(frac * TWO32), U32_MAX))


@dataclasses.dataclass(frozen=True)
class RequestClass:
    weight: float
    prompt: Law
    decode: Law


@dataclasses.dataclass(frozen=True)
class Mixture:
    """The joint law nu of (l, o): a class mixture with l and o independent within a class."""

    classes: tuple

    def __post_init__(self):
        object.__setattr__(self, "classes", tuple(self.classes))
        if not self.classes:
            raise ValueError("need at least one class")

    @property
    def class_thr(self) -> np.ndarray:
        w = np.array([c.weight for c in self.classes], dtype=np.float64)
        return _quantise(np.cumsum(w / w.sum())[:-1])

    def class_prob(self) -> np.ndarray:
        edges = np.concatenate(([0.0], self.class_thr.astype(np.float64), [TWO32]))
        return np.diff(edges) / TWO32

    @property
    def l_max(self) -> int:
        return max(c.prompt.hi for c in self.classes)

    @property
    def o_max(self) -> int:
        return max(c.decode.hi for c in self.classes)


def single(prompt: Law, decode: Law) -> Mixture:
    return Mixture((RequestClass(1.0, prompt, decode),))
