"""Pins of the oracle's slots of variable duration (a linear stand-in for the batch times of Section 4.2):
CPU only."""
import json
import os

import numpy as np

import oracle
from workloads import configs, laws
from workloads.configs import Workload, flow_cell, greedy_cell

HERE = os.path.dirname(os.path.abspath(__file__))
INF = 1 << 30


def _workload(cells, time_model, lam=0.05, T=3000, capacity=4000, n_replicas=4, seed=90, **kw):
    mix = laws.single(laws.uniform_int(4, 40), laws.geometric(12.0, cap=80))
    return Workload(name="timed-pin", capacity=capacity, token_budget=kw.pop("token_budget", 256),
                    prefill_chunk=kw.pop("prefill_chunk", 64), mixture=mix,
                    arrival_laws=(laws.poisson_counts(lam),), cells=tuple(cells), n_replicas=n_replicas,
                    n_steps=T, seed=seed, max_requests=1 << 14, time_model=tuple(time_model), **kw)


def test_hand_trajectory():
    g = json.load(open(os.path.join(HERE, "golden", "timed_trajectory.json")))
    wl = _workload([flow_cell(0, 1.0)], g["time_model"], T=g["n_steps"], capacity=1000, n_replicas=1,
                   token_budget=INF, prefill_chunk=INF)
    a = g["arrivals"]
    r = oracle.run_cell(wl, 0, per_step=True, forced=(a["t"], a["l"], a["o"]), forced_B=[1])
    assert r["step_u"][0].tolist() == g["U"]
    assert r["step_p"][0].tolist() == g["P"]
    assert r["step_q"][0].tolist() == g["Q"]
    assert r["step_n"][0].tolist() == g["N"]
    assert r["completion_step"][0][:3].tolist() == g["completion_time"]
    c = {k: int(v[0]) for k, v in r["counters"].items()}
    assert (c["sum_latency"], c["max_latency"], c["elapsed"]) == (g["sum_latency"], g["max_latency"], g["elapsed"])


def test_unit_slots_are_the_special_case():
    # d_t = 1 + 0 + 0: the same path as without a time model, counter for counter
    for cells in ([flow_cell(0, 0.9)], [greedy_cell(0)]):
        a = oracle.run_cell(_workload(cells, (0, 0, 0), lam=0.8, capacity=600), 0)
        b = oracle.run_cell(_workload(cells, (1, 0, 0), lam=0.8, capacity=600), 0)
        for k in a["counters"]:
            assert np.array_equal(a["counters"][k], b["counters"][k]), k
        assert np.array_equal(a["completion_step"], b["completion_step"])
        assert np.all(a["counters"]["elapsed"] == 3000)


def test_time_is_the_sum_of_the_slot_durations_and_arrivals_follow_it():
    c0, cp, cd = 3, 1, 2
    wl = _workload([greedy_cell(0)], (c0, cp, cd), lam=0.04, T=4000)
    r = oracle.run_cell(wl, 0, per_step=True)
    c = r["counters"]
    # elapsed = sum over slots of c0 + cp * prompt tokens + cd * output tokens
    want = 4000 * c0 + cp * c["prefill_tokens"].astype(np.int64) + cd * c["decode_tokens"].astype(np.int64)
    assert np.array_equal(c["elapsed"].astype(np.int64), want)
    # arrivals: a Poisson stream per time unit; what has joined by the last slot is the stream up to its start
    key = (wl.seed & 0xffffffff, wl.seed >> 32)
    for i, rep in enumerate(r["replica_ids"][:2]):
        arr = r["arrival_step"][i]
        arr = arr[:int(c["arrived"][i])]
        assert np.all(np.diff(arr) >= 0) and arr[0] >= 1                       # ids in order of arrival time
        words = np.array([oracle.philox([0, u, int(rep), 0], key)[0] for u in range(1, 400)], np.uint32)
        n_u = oracle.invert(wl.arrival_laws[0], words)
        got = np.bincount(arr[arr < 400], minlength=400)[1:400]
        assert np.array_equal(got, n_u[:399])
    # rate: arrivals per elapsed unit is the mean of the count law
    rate = c["arrived"].sum() / c["elapsed"].sum()
    assert abs(rate - 0.04) < 0.004


def test_latencies_are_in_time_units():
    # long stable run
    c0, cp, cd = 2, 1, 1
    wl = _workload([flow_cell(0, 1.5)], (c0, cp, cd), lam=0.02, T=30000, n_replicas=8)
    r = oracle.run_cell(wl, 0, per_step=True, n_threads=8)
    c = r["counters"]
    assert not c["evictions"].any()
    # latencies are in time units: completion unit - arrival unit + 1, per request
    done = c["completed"].astype(np.float64)
    mean_lat = c["sum_latency"].sum() / done.sum()
    lam_eff = done.sum() / c["elapsed"].sum()
    for i in range(2):
        comp = r["completion_step"][i].astype(np.int64)
        arr = r["arrival_step"][i].astype(np.int64)
        ok = comp > 0
        assert int(c["sum_latency"][i]) == int((comp[ok] - arr[ok] + 1).sum())
        assert int(c["max_latency"][i]) == int((comp[ok] - arr[ok] + 1).max())
        assert np.all(comp[ok] <= int(c["elapsed"][i]))
    # stable: what completes per unit of time is what arrives per unit of time
    assert abs(lam_eff - 0.02) < 0.002 and mean_lat > c0


def test_longer_batches_mean_more_arrivals_per_slot():
    base = _workload([greedy_cell(0)], (1, 0, 0), lam=0.05, T=3000)
    slow = _workload([greedy_cell(0)], (4, 0, 0), lam=0.05, T=3000)
    a, b = oracle.run_cell(base, 0)["counters"], oracle.run_cell(slow, 0)["counters"]
    assert np.all(b["elapsed"] == 4 * a["elapsed"])
    assert abs(b["arrived"].sum() / a["arrived"].sum() - 4.0) < 0.4
