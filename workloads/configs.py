"""Seeded synthetic workloads: the five benchmark configurations and small variants.

A :class:`Workload` is a complete, simulator-agnostic description of one run:
capacity M, token budget, prefill chunk, the length mixture nu, a list of
arrival-count laws, and a list of *cells* (policy, arrival law, activation
budget b) that all share the same random streams.  Each cell is simulated for
``n_replicas`` independent sample paths of ``n_steps`` slots.

The arrival rates of most configurations are stated as multiples of the paper's
necessary-condition bound (Proposition 2, eq. 3).  That bound is part of the
method, so it is *not* computed here: the caller passes ``stability_bound``, a
function ``(Mixture, capacity) -> float``.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Callable, Sequence

import numpy as np

from . import laws
from .laws import Law, Mixture, RequestClass

FLOW = 0     # Algorithm 2: rate-limited activation, LIFO eviction on overflow
GREEDY = 1   # b -> infinity limit with a memory fit test: admit while it fits, evict newest
CLASSES = 2  # Algorithm 1: known lengths, one FIFO, arrival stream and integer budget b_k per class
ALPHA = 3    # alpha-protection greedy (Section 4.1): admit while it fits (1 - alpha) M, evict all on overflow
MC = 4       # memory-check benchmark (Section 4.1): FCFS, admit only if the predicted future usage stays within M


@dataclasses.dataclass(frozen=True)
class Cell:
    policy: int
    arrival: int          # index into Workload.arrival_laws
    b_floor: int          # B_t = b_floor + [u < b_frac_thr]   (ignored by GREEDY)
    b_frac_thr: int
    label: str = ""
    class_arrival: tuple = ()   # CLASSES: per class, index into Workload.arrival_laws
    class_budget: tuple = ()    # CLASSES: per class, integer budget b_k
    alpha: float = 0.0          # ALPHA: protected share of the memory
    budget_law: int = -1        # FLOW, if >= 0: B_t is drawn from Workload.arrival_laws[budget_law]
    credit_b16: int = 0         # FLOW, if > 0: B_t = floor(t b) - floor((t - 1) b), b = credit_b16 / 2^16
    assumed_o: int = 0          # MC: output length every request is taken to reach (the longest possible one)


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    capacity: int
    token_budget: int
    prefill_chunk: int
    mixture: Mixture
    arrival_laws: tuple
    cells: tuple
    n_replicas: int
    n_steps: int
    seed: int
    trace_every: int = 0
    hist_bins: int = 0
    hist_shift: int = 0
    max_requests: int = 0      # per-path capacity of the per-request record arrays (0 = off)
    time_model: tuple = (0, 0, 0)  # (c0, cp, cd): a slot lasts c0 + cp * prompt tokens + cd * output tokens
                                   # time units, arrivals come per unit; all 0: every slot lasts one unit
    notes: str = ""

    def scaled(self, n_replicas: int | None = None, n_steps: int | None = None, **kw) -> "Workload":
        d = {}
        if n_replicas is not None:
            d["n_replicas"] = int(n_replicas)
        if n_steps is not None:
            d["n_steps"] = int(n_steps)
        d.update(kw)
        return dataclasses.replace(self, **d)

    @property
    def n_paths(self) -> int:
        return len(self.cells) * self.n_replicas


def split_b(b: float):
    """b -> (floor(b), threshold of the fractional part): B_t = floor + Bernoulli(frac)."""
    fl = int(math.floor(b))
    return fl, laws.frac_threshold(b - fl)


def default_b(lam: float, lam_star: float) -> float:
    """Midpoint between the arrival rate and the bound while below it, the bound itself otherwise."""
    return 0.5 * (lam + lam_star) if lam < lam_star else lam_star


def flow_cell(arrival: int, b: float, label: str = "") -> Cell:
    fl, th = split_b(b)
    return Cell(FLOW, arrival, fl, th, label or f"flow(b={b:.6g})")


def flow_law_cell(arrival: int, budget_law: int, label: str = "") -> Cell:
    """FLOW with B_t i.i.d. from a count law of the workload (Theorem 2: any bounded integer law)."""
    return Cell(FLOW, arrival, 0, 0, label or f"flow(B~law {budget_law})", budget_law=int(budget_law))


def flow_credit_cell(arrival: int, b: float, label: str = "") -> Cell:
    """FLOW with the deterministic budget of a credit accumulator: floor(t b) - floor((t - 1) b)."""
    b16 = int(round(b * 65536.0))
    if b16 <= 0:
        raise ValueError("b must be at least 2^-16")
    return Cell(FLOW, arrival, 0, 0, label or f"flow(credit b={b16 / 65536.0:.6g})", credit_b16=b16)


def greedy_cell(arrival: int, label: str = "greedy") -> Cell:
    return Cell(GREEDY, arrival, 0, 0, label)


def alpha_cell(arrival: int, alpha: float, label: str = "") -> Cell:
    if not 0.0 <= alpha < 1.0:
        raise ValueError("alpha in [0, 1)")
    return Cell(ALPHA, arrival, 0, 0, label or f"alpha-protection({alpha:.6g})", alpha=float(alpha))


def mc_cell(arrival: int, assumed_o: int, label: str = "") -> Cell:
    """The memory-check benchmark with every output taken as `assumed_o` tokens long (Section 4.1: with
    unknown types the longest possible value, `longest_output(mixture)`)."""
    return Cell(MC, arrival, 0, 0, label or f"mc(o_hat={assumed_o})", assumed_o=int(assumed_o))


def mc_known_cell(arrival: int, label: str = "mc(known types)") -> Cell:
    """The memory-check benchmark with known request types (Section 4.1, first study): every request is
    predicted to produce its own output length."""
    return Cell(MC, arrival, 0, 0, label, assumed_o=0)


def longest_output(mixture: Mixture) -> int:
    return max(c.decode.hi for c in mixture.classes)


def classes_cell(class_arrival, class_budget, label: str = "") -> Cell:
    class_arrival = tuple(int(a) for a in class_arrival)
    class_budget = tuple(int(b) for b in class_budget)
    if len(class_arrival) != len(class_budget):
        raise ValueError("one arrival law and one budget per class")
    return Cell(CLASSES, class_arrival[0], 0, 0, label or f"classes(b={class_budget})", class_arrival, class_budget)


Bound = Callable[[Mixture, int], float]


def config0(bound: Bound) -> Workload:
    M = 16384
    mix = laws.single(laws.uniform_int(16, 256), laws.geometric(128.0, cap=1024))
    lam = 0.05
    ls = bound(mix, M)
    return Workload(
        name="cfg0-tiny-flow", capacity=M, token_budget=512, prefill_chunk=512, mixture=mix,
        arrival_laws=(laws.bernoulli_counts(lam),),
        cells=(flow_cell(0, default_b(lam, ls)),),
        n_replicas=64, n_steps=10_000, seed=1, max_requests=1024,
        notes=f"lambda={lam}, bound={ls:.6g}")


def config1(bound: Bound) -> Workload:
    M = 262144
    mix = laws.single(laws.lognormal(6.0, 0.8, 8, 8192), laws.lognormal(5.5, 1.0, 1, 16384))
    ls = bound(mix, M)
    lam = 0.9 * ls
    return Workload(
        name="cfg1-flow-vs-greedy", capacity=M, token_budget=2048, prefill_chunk=512, mixture=mix,
        arrival_laws=(laws.poisson_counts(lam),),
        cells=(flow_cell(0, default_b(lam, ls)), greedy_cell(0)),
        n_replicas=1024, n_steps=100_000, seed=2, hist_bins=0,
        notes=f"lambda={lam:.6g} (0.9 x bound {ls:.6g})")


def config2(bound: Bound) -> Workload:
    M = 524288
    mix = laws.single(laws.uniform_int(64, 4096), laws.pareto(1.5, 32.0, 32768))
    ls = bound(mix, M)
    factors = (0.8, 0.95, 1.05)
    arr = tuple(laws.poisson_counts(f * ls) for f in factors)
    cells = tuple(flow_cell(i, default_b(f * ls, ls), f"flow(lambda={f}xbound)") for i, f in enumerate(factors))
    return Workload(
        name="cfg2-heavy-tail", capacity=M, token_budget=4096, prefill_chunk=1024, mixture=mix,
        arrival_laws=arr, cells=cells, n_replicas=4096, n_steps=200_000, seed=3, trace_every=1000,
        notes=f"bound={ls:.6g}")


def config3(bound: Bound, n_lambda: int = 64, n_b: int = 32) -> Workload:
    M = 131072
    mix = laws.single(laws.geometric(512.0), laws.geometric(256.0))
    ls = bound(mix, M)
    lam_f = np.linspace(0.5, 1.1, n_lambda)
    b_f = np.linspace(0.5, 1.5, n_b)
    arr = tuple(laws.poisson_counts(float(f) * ls) for f in lam_f)
    cells = []
    for i, f in enumerate(lam_f):
        for g in b_f:
            cells.append(flow_cell(i, float(g) * ls, f"flow(lambda={f:.4f}x,b={g:.4f}x)"))
    return Workload(
        name="cfg3-grid", capacity=M, token_budget=1024, prefill_chunk=256, mixture=mix,
        arrival_laws=arr, cells=tuple(cells), n_replicas=128, n_steps=50_000, seed=4,
        hist_bins=4096, hist_shift=1, notes=f"bound={ls:.6g}")


def config4(bound: Bound) -> Workload:
    M = 2097152
    short = RequestClass(0.7, laws.lognormal(5.0, 0.5, 1, 32768), laws.geometric(64.0))
    long_ = RequestClass(0.3, laws.lognormal(8.0, 0.5, 1, 32768), laws.lognormal(7.0, 1.0, 1, 65536))
    mix = Mixture((short, long_))
    ls = bound(mix, M)
    lam = 0.95 * ls
    return Workload(
        name="cfg4-large-memory", capacity=M, token_budget=8192, prefill_chunk=2048, mixture=mix,
        arrival_laws=(laws.poisson_counts(lam),),
        cells=(flow_cell(0, default_b(lam, ls)),),
        n_replicas=512, n_steps=1_000_000, seed=5,
        notes=f"lambda={lam:.6g} (0.95 x bound {ls:.6g})")


CONFIGS = (config0, config1, config2, config3, config4)


def make(index: int, bound: Bound) -> Workload:
    return CONFIGS[index](bound)


def three_class(lam_per_class: float, capacity: int = 16492, b: float = 12.0,
                n_replicas: int = 8, n_steps: int = 2000, seed: int = 7) -> Workload:
    """The paper's synthetic study shape (Section 4.1): l=10, o in {20,40,60}, equal Poisson rates."""
    cls = tuple(RequestClass(1.0, laws.point(10), laws.point(o)) for o in (20, 40, 60))
    mix = Mixture(cls)
    return Workload(
        name="three-class", capacity=capacity, token_budget=1 << 20, prefill_chunk=1 << 20, mixture=mix,
        arrival_laws=(laws.poisson_counts(3.0 * lam_per_class),),
        cells=(flow_cell(0, b), greedy_cell(0)),
        n_replicas=n_replicas, n_steps=n_steps, seed=seed, max_requests=1 << 16)


def known_classes(lam_per_class=(5.0, 5.0, 5.0), budgets=(4, 4, 4), lengths=((10, 20), (10, 40), (10, 60)),
                  capacity: int = 16492, token_budget: int = 1 << 30, prefill_chunk: int = 1 << 30,
                  n_replicas: int = 1024, n_steps: int = 10_000, seed: int = 8, **kw) -> Workload:
    """The paper's synthetic study with known lengths (Section 4.1 under Algorithm 1): classes
    (l, o) = (10, 20), (10, 40), (10, 60), Poisson arrivals per class, M = 16492, b = (4, 4, 4).
    The printed rate of 5 per class overloads it (b_k < lambda_k); rates below 4 are stable."""
    cls = tuple(RequestClass(1.0, laws.point(l), laws.point(o)) for l, o in lengths)
    rates = tuple(float(x) for x in lam_per_class)
    distinct = sorted(set(rates))
    arr = tuple(laws.poisson_counts(r) for r in distinct)
    cell = classes_cell([distinct.index(r) for r in rates], budgets)
    return Workload(
        name="known-classes", capacity=capacity, token_budget=token_budget, prefill_chunk=prefill_chunk,
        mixture=Mixture(cls), arrival_laws=arr, cells=(cell,), n_replicas=n_replicas, n_steps=n_steps,
        seed=seed, **kw)


def budget_forms(bound: Bound, n_replicas: int = 1024, n_steps: int = 100_000) -> Workload:
    """Configuration 1's workload under Algorithm 2 with three forms of the activation budget of the same
    mean b: floor(b) + Bernoulli, a three-point law (Theorem 2 allows any bounded i.i.d. integer law), and
    the deterministic credit accumulator."""
    base = config1(bound)
    lam_cell = base.cells[0]
    b = lam_cell.b_floor + lam_cell.b_frac_thr / laws.TWO32
    fl = int(math.floor(b))
    frac = b - fl
    # masses on {fl - 1, fl, fl + 1} (or {fl, fl + 1, fl + 2} when fl = 0) with mean b
    lo = max(fl - 1, 0)
    shift = b - (lo + 1)                   # mean relative to the middle point, in (-1, 1)
    pmf = np.array([0.25 - shift / 2.0, 0.5, 0.25 + shift / 2.0])
    cells = (lam_cell, flow_law_cell(0, 1, f"flow(B~3-point, mean {b:.6g})"), flow_credit_cell(0, b))
    return dataclasses.replace(base, name="budget-forms", arrival_laws=base.arrival_laws + (laws.from_pmf(lo, pmf),),
                               cells=cells, n_replicas=n_replicas, n_steps=n_steps, seed=10)


def alpha_sweep(alphas=(0.0, 0.05, 0.1, 0.15), lam_per_class: float = 3.3, capacity: int = 16492,
                n_replicas: int = 1024, n_steps: int = 10_000, seed: int = 9, **kw) -> Workload:
    """The paper's synthetic study with unknown types (Section 4.1) under the alpha-protection greedy
    baseline, one cell per alpha (the paper searches a grid of alpha), plus the greedy / evict-newest
    baseline on the same arrivals: classes (10, 20), (10, 40), (10, 60) in equal shares, Poisson arrivals."""
    cls = tuple(RequestClass(1.0, laws.point(10), laws.point(o)) for o in (20, 40, 60))
    cells = tuple(alpha_cell(0, a) for a in alphas) + (greedy_cell(0),)
    return Workload(
        name="alpha-sweep", capacity=capacity, token_budget=kw.pop("token_budget", 1 << 30),
        prefill_chunk=kw.pop("prefill_chunk", 1 << 30), mixture=Mixture(cls),
        arrival_laws=(laws.poisson_counts(3.0 * lam_per_class),), cells=cells, n_replicas=n_replicas,
        n_steps=n_steps, seed=seed, **kw)


def unknown_types(lam_per_class: float = 3.3, b: float = 11.0, alpha: float = 0.05, capacity: int = 16492,
                  n_replicas: int = 1024, n_steps: int = 10_000, seed: int = 12, **kw) -> Workload:
    """The paper's synthetic study with unknown request types (Section 4.1, second row of its figure): classes
    (10, 20), (10, 40), (10, 60) in equal shares, Poisson arrivals, M = 16492, under Algorithm 2, the
    alpha-protection greedy baseline, the MC benchmark with the longest possible output (60), and the
    greedy / evict-newest baseline, all on the same arrivals."""
    cls = tuple(RequestClass(1.0, laws.point(10), laws.point(o)) for o in (20, 40, 60))
    mix = Mixture(cls)
    cells = (flow_cell(0, b), alpha_cell(0, alpha), mc_cell(0, longest_output(mix)), greedy_cell(0))
    return Workload(
        name="unknown-types", capacity=capacity, token_budget=1 << 30, prefill_chunk=1 << 30, mixture=mix,
        arrival_laws=(laws.poisson_counts(3.0 * lam_per_class),), cells=cells, n_replicas=n_replicas,
        n_steps=n_steps, seed=seed, **kw)


def known_types(lam_per_class: float = 3.3, budgets=(4, 4, 4), alpha: float = 0.05, capacity: int = 16492,
                n_replicas: int = 1024, n_steps: int = 10_000, seed: int = 14, **kw) -> Workload:
    """The paper's synthetic study with known request types (Section 4.1, first row of its figure): classes
    (10, 20), (10, 40), (10, 60), Poisson arrivals per class, M = 16492, under Algorithm 1 with b = (4, 4, 4),
    the alpha-protection greedy baseline, the MC benchmark with every request predicted at its own length, and
    the greedy / evict-newest baseline.  Algorithm 1 draws one arrival stream per class; the other three share
    one stream of the summed rate whose requests fall into the classes with equal shares."""
    cls = tuple(RequestClass(1.0, laws.point(10), laws.point(o)) for o in (20, 40, 60))
    arr = (laws.poisson_counts(lam_per_class), laws.poisson_counts(3.0 * lam_per_class))
    cells = (classes_cell([0, 0, 0], budgets), alpha_cell(1, alpha), mc_known_cell(1), greedy_cell(1))
    return Workload(
        name="known-types", capacity=capacity, token_budget=1 << 30, prefill_chunk=1 << 30, mixture=Mixture(cls),
        arrival_laws=arr, cells=cells, n_replicas=n_replicas, n_steps=n_steps, seed=seed, **kw)


def timed_study(bound: Bound, time_model=(40, 1, 1), n_replicas: int = 1024, n_steps: int = 10_000) -> Workload:
    """Configuration 1's request mix and memory under Algorithm 2 and the greedy baseline with slots of variable
    duration (a linear stand-in for the batch times of Section 4.2): a slot lasts 40 + prompt tokens + output
    tokens time units, requests arrive per unit at 0.9 of the rate the slot model would carry if every slot
    took the duration of a typical one."""
    base = config1(bound)
    lam_slot = 0.9 * bound(base.mixture, base.capacity)              # per slot, as in configuration 1
    typical = time_model[0] + time_model[1] * 300 + time_model[2] * 215  # prompt and output tokens of a typical slot
    lam_unit = lam_slot / typical
    b = default_b(lam_slot, bound(base.mixture, base.capacity))
    return dataclasses.replace(base, name="timed-study", arrival_laws=(laws.poisson_counts(lam_unit),),
                               cells=(flow_cell(0, b), greedy_cell(0)), n_replicas=n_replicas, n_steps=n_steps,
                               seed=13, time_model=tuple(time_model))


def toy(capacity: int = 600, token_budget: int = 96, prefill_chunk: int = 32, lam: float = 0.6,
        b: float = 0.8, l_range=(4, 60), o_mean: float = 12.0, o_cap: int = 80,
        n_replicas: int = 16, n_steps: int = 400, seed: int = 11,
        policies: Sequence[int] = (FLOW, GREEDY), **kw) -> Workload:
    """A small, eviction-heavy workload for exhaustive checks."""
    mix = laws.single(laws.uniform_int(*l_range), laws.geometric(o_mean, cap=o_cap))
    cells = []
    for p in policies:
        cells.append(flow_cell(0, b) if p == FLOW else greedy_cell(0))
    return Workload(
        name="toy", capacity=capacity, token_budget=token_budget, prefill_chunk=prefill_chunk, mixture=mix,
        arrival_laws=(laws.poisson_counts(lam),), cells=tuple(cells), n_replicas=n_replicas,
        n_steps=n_steps, seed=seed, trace_every=kw.pop("trace_every", 10),
        hist_bins=kw.pop("hist_bins", 256), hist_shift=kw.pop("hist_shift", 0),
        max_requests=kw.pop("max_requests", 2048), **kw)
