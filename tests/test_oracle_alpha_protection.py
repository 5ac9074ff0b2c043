"""Pins of the oracle's alpha-protection greedy baseline (Section 4.1): CPU only."""
import dataclasses
import json
import os

import numpy as np

import oracle
from workloads import ALPHA, GREEDY, configs, laws
from workloads.configs import Workload, alpha_cell, greedy_cell

HERE = os.path.dirname(os.path.abspath(__file__))
INF = 1 << 30


def _workload(cells, capacity, lam, T, n_replicas=4, seed=40, l=(4, 40), o_mean=20.0, o_cap=200, **kw):
    mix = laws.single(laws.uniform_int(*l), laws.geometric(o_mean, cap=o_cap))
    return Workload(name="alpha-pin", capacity=capacity, token_budget=kw.pop("token_budget", INF),
                    prefill_chunk=kw.pop("prefill_chunk", INF), mixture=mix,
                    arrival_laws=(laws.poisson_counts(lam),), cells=tuple(cells), n_replicas=n_replicas,
                    n_steps=T, seed=seed, max_requests=kw.pop("max_requests", 1 << 14), **kw)


def test_hand_trajectory_with_two_overflows():
    g = json.load(open(os.path.join(HERE, "golden", "alpha_protection_trajectory.json")))
    wl = _workload([alpha_cell(0, g["alpha"])], g["capacity"], 1.0, g["n_steps"], n_replicas=1)
    a = g["arrivals"]
    r = oracle.run_cell(wl, 0, per_step=True, forced=(a["t"], a["l"], a["o"]))
    assert oracle.protect_limit(g["alpha"], g["capacity"]) == 15
    assert r["step_u"][0].tolist() == g["U"]
    assert r["step_p"][0].tolist() == g["P"]
    assert r["step_q"][0].tolist() == g["Q"]
    c = {k: int(v[0]) for k, v in r["counters"].items()}
    for k in ("evictions", "overflow_steps", "activations", "completed", "sum_latency"):
        assert c[k] == g[k], k
    assert r["completion_step"][0][:3].tolist() == g["completion_step"]


def test_without_overflow_alpha_zero_is_the_greedy_baseline():
    # memory so large that nothing ever overflows: the two policies differ only in what an overflow does
    wl = _workload([alpha_cell(0, 0.0), greedy_cell(0)], 200_000, 1.0, 1500)
    a, g = oracle.run_cell(wl, 0), oracle.run_cell(wl, 1)
    assert not a["counters"]["overflow_steps"].any() and not g["counters"]["overflow_steps"].any()
    for k in a["counters"]:
        assert np.array_equal(a["counters"][k], g["counters"][k]), k
    assert np.array_equal(a["completion_step"], g["completion_step"])


def test_limit_is_respected_and_overflow_empties_the_active_set():
    wl = _workload([alpha_cell(0, 0.3)], 1500, 0.9, 3000, o_mean=40.0)
    limit = oracle.protect_limit(0.3, 1500)
    assert limit == 1050
    r = oracle.run_cell(wl, 0, per_step=True)
    c = r["counters"]
    assert c["overflow_steps"].sum() > 0
    U, P, Q, N = (r[k].astype(np.int64) for k in ("step_u", "step_p", "step_q", "step_n"))
    assert U.max() <= 1500
    for i in range(U.shape[0]):
        first = r["first_activation"][i]
        last = r["last_activation"][i]
        known = first > 0
        # a slot that activates somebody ends (all prompts taken whole, one token each) with a usage of
        # at most the limit: the fit test counted l + 1 for every active request
        act = np.unique(np.concatenate([first[known], last[known]]))
        assert np.all(U[i][act - 1] <= limit)
        # an overflow slot leaves nobody active, and the queue grows by more than the arrivals: everything
        # that was active went back (a slot emptied by completions alone leaves the queue as it was)
        empty = (P[i] == 0) & (U[i] == 0)
        went_back = empty[1:] & (P[i][:-1] > 0) & (Q[i][1:] >= Q[i][:-1] + N[i][1:] + 1)
        assert int(went_back.sum()) == int(c["overflow_steps"][i])
    # conservation
    assert np.array_equal(c["arrived"], c["completed"] + c["final_p"] + c["final_q"])
    assert np.array_equal(c["activations"], c["completed"] + c["final_p"] + c["evictions"])
    assert np.all(c["evictions"] >= c["overflow_steps"])


def test_everything_protected_means_nobody_is_admitted():
    # (1 - alpha) M below the smallest l + 1: the queue is the arrival count
    wl = _workload([alpha_cell(0, 0.999)], 4000, 0.5, 400, l=(4, 40))
    assert oracle.protect_limit(0.999, 4000) == 4
    c = oracle.run_cell(wl, 0)["counters"]
    assert not c["activations"].any() and not c["completed"].any()
    assert np.array_equal(c["arrived"], c["final_q"])


def test_more_protection_means_fewer_overflows_on_average():
    # the protected share exists to absorb growth: over many replicas overflows fall as alpha rises
    cells = [alpha_cell(0, a) for a in (0.0, 0.2, 0.4)]
    wl = _workload(cells, 2500, 0.8, 3000, n_replicas=16, o_mean=50.0, o_cap=400)
    ov = [int(oracle.run_cell(wl, i, n_threads=4)["counters"]["overflow_steps"].sum()) for i in range(3)]
    assert ov[0] > ov[1] > ov[2], ov
