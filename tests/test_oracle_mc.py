"""Pins of the oracle's memory-check (MC) benchmark of Section 4.1: CPU only."""
import json
import os

import numpy as np

import oracle
from workloads import configs, laws
from workloads.configs import Workload, greedy_cell, longest_output, mc_cell

HERE = os.path.dirname(os.path.abspath(__file__))
INF = 1 << 30


def _workload(cells, mix, capacity, lam, T, n_replicas=4, seed=70):
    return Workload(name="mc-pin", capacity=capacity, token_budget=INF, prefill_chunk=INF, mixture=mix,
                    arrival_laws=(laws.poisson_counts(lam),), cells=tuple(cells), n_replicas=n_replicas,
                    n_steps=T, seed=seed, max_requests=1 << 14)


def test_hand_trajectory_with_a_refused_and_a_tight_admission():
    g = json.load(open(os.path.join(HERE, "golden", "mc_trajectory.json")))
    mix = laws.single(laws.uniform_int(4, 8), laws.uniform_int(1, 4))
    assert longest_output(mix) == g["assumed_o"]
    wl = _workload([mc_cell(0, g["assumed_o"])], mix, g["capacity"], 1.0, g["n_steps"], n_replicas=1)
    a = g["arrivals"]
    r = oracle.run_cell(wl, 0, per_step=True, forced=(a["t"], a["l"], a["o"]))
    assert r["step_u"][0].tolist() == g["U"]
    assert r["step_p"][0].tolist() == g["P"]
    assert r["step_q"][0].tolist() == g["Q"]
    assert r["completion_step"][0][:4].tolist() == g["completion_step"]
    assert r["first_activation"][0][:4].tolist() == g["first_activation"]
    c = r["counters"]
    assert int(c["sum_latency"][0]) == g["sum_latency"] and not c["evictions"].any()


def test_the_memory_is_never_exceeded_under_overload():
    # far more load than the memory carries: the queue explodes, nothing is ever evicted
    mix = laws.single(laws.uniform_int(4, 40), laws.geometric(20.0, cap=100))
    wl = _workload([mc_cell(0, longest_output(mix))], mix, 1500, 2.0, 2500)
    r = oracle.run_cell(wl, 0, per_step=True)
    c = r["counters"]
    assert not c["evictions"].any() and not c["overflow_steps"].any()
    assert r["step_u"].max() <= 1500 and np.all(c["max_u"] <= 1500)
    assert np.all(c["final_q"] > 1000)
    assert np.array_equal(c["activations"], c["completed"] + c["final_p"])      # nobody is activated twice
    # first come first served: requests are activated in the order of their ids
    for i in range(4):
        fa = r["first_activation"][i]
        fa = fa[:int(c["activations"][i])]
        assert np.all(fa > 0) and np.all(np.diff(fa) >= 0)


def test_with_exact_lengths_the_memory_is_filled_to_within_one_request():
    # every output really has the assumed length: the prediction is exact, so whenever the head is kept
    # waiting some future slot would pass M with it, and without later help that slot comes within one
    # request of M.  (A rule that reserved l + o_hat for everybody would stay far below.)
    l_hi, o_hat, M = 12, 30, 1200
    mix = laws.single(laws.uniform_int(3, l_hi), laws.point(o_hat))
    wl = _workload([mc_cell(0, o_hat)], mix, M, 3.0, 1500)
    c = oracle.run_cell(wl, 0)["counters"]
    assert np.all(c["final_q"] > 100)                       # saturated
    assert np.all(c["max_u"] <= M) and np.all(c["max_u"] > M - (l_hi + o_hat))
    reserved_peak = (M // (3 + o_hat)) * (l_hi + o_hat)     # what static reservations could ever hold ...
    assert reserved_peak >= M - (l_hi + o_hat)              # ... is not the reason: look at the mean
    assert np.all(c["sum_u"] / 1500 > 0.6 * M)              # staggered requests fill the memory on average


def test_with_room_for_everybody_it_is_the_greedy_baseline():
    mix = laws.single(laws.uniform_int(4, 40), laws.geometric(20.0, cap=100))
    wl = _workload([mc_cell(0, 100), greedy_cell(0)], mix, 1 << 22, 1.5, 1500)
    a, g = oracle.run_cell(wl, 0), oracle.run_cell(wl, 1)
    for k in a["counters"]:
        assert np.array_equal(a["counters"][k], g["counters"][k]), k
    assert np.array_equal(a["completion_step"], g["completion_step"])


def test_a_longer_assumed_output_admits_less():
    mix = laws.single(laws.uniform_int(4, 40), laws.geometric(20.0, cap=100))
    wl = _workload([mc_cell(0, 100), mc_cell(0, 200), mc_cell(0, 400)], mix, 2500, 1.6, 2500)
    q = [float(oracle.run_cell(wl, i)["counters"]["sum_q"].sum()) for i in range(3)]
    assert q[0] < q[1] < q[2], q


# ---- known request types: every request predicted at its own output length (first study of Section 4.1) ----

def test_known_types_hand_trajectory():
    from workloads.configs import mc_known_cell
    g = json.load(open(os.path.join(HERE, "golden", "mc_known_trajectory.json")))
    mix = laws.single(laws.uniform_int(4, 8), laws.uniform_int(1, 5))
    a = g["arrivals"]
    wl = _workload([mc_known_cell(0), mc_cell(0, 5)], mix, g["capacity"], 1.0, g["n_steps"], n_replicas=1)
    r = oracle.run_cell(wl, 0, per_step=True, forced=(a["t"], a["l"], a["o"]))
    assert r["step_u"][0].tolist() == g["U"]
    assert r["step_p"][0].tolist() == g["P"]
    assert r["step_q"][0].tolist() == g["Q"]
    assert r["completion_step"][0][:3].tolist() == g["completion_step"]
    assert r["first_activation"][0][:3].tolist() == g["first_activation"]
    assert int(r["counters"]["sum_latency"][0]) == g["sum_latency"] and not r["counters"]["evictions"].any()
    # the same arrivals under one common assumed length (the longest, 5): B is kept out of slot 1
    u = oracle.run_cell(wl, 1, per_step=True, forced=(a["t"], a["l"], a["o"]))
    assert u["first_activation"][0][1] > 1


def test_known_types_fill_the_memory_and_never_pass_it():
    from workloads.configs import mc_known_cell
    mix = laws.single(laws.uniform_int(4, 40), laws.geometric(20.0, cap=100))
    M = 1500
    wl = _workload([mc_known_cell(0), mc_cell(0, longest_output(mix))], mix, M, 2.0, 2500)
    k = oracle.run_cell(wl, 0, per_step=True)
    c = k["counters"]
    assert not c["evictions"].any() and not c["overflow_steps"].any()
    assert k["step_u"].max() <= M and np.all(c["final_q"] > 200)
    assert np.array_equal(c["activations"], c["completed"] + c["final_p"])
    # the prediction is exact, so a head that waits would really have passed M: the memory comes within one
    # request of M again and again
    assert np.all(c["max_u"] > M - (40 + 100))
    # knowing the lengths admits more than assuming the longest for everybody
    u = oracle.run_cell(wl, 1)["counters"]
    assert np.all(c["completed"] > u["completed"]) and c["sum_q"].sum() < u["sum_q"].sum()
    # the prediction made at activation is what happens: usage in a request's last slot, re-summed from the
    # requests then active, stays within M (brute force over the records)
    for i in range(2):
        n = int(c["arrived"][i])
        s, l, o, e = (k[x][i][:n].astype(np.int64) for x in ("first_activation", "req_l", "req_o", "completion_step"))
        on = s > 0
        assert np.array_equal(e[on & (e > 0)], (s + o - 1)[on & (e > 0)])       # alive exactly o slots
        for t in range(1, wl.n_steps + 1, 97):
            act = on & (s <= t) & (s + o - 1 >= t)
            assert int((l[act] + t - s[act] + 1).sum()) == int(k["step_u"][i][t - 1])


def test_known_types_with_one_output_length_equal_the_assumed_length_rule():
    from workloads.configs import mc_known_cell
    mix = laws.single(laws.uniform_int(3, 12), laws.point(30))
    wl = _workload([mc_known_cell(0), mc_cell(0, 30)], mix, 1200, 3.0, 1500)
    a, b = oracle.run_cell(wl, 0), oracle.run_cell(wl, 1)
    for name in a["counters"]:
        assert np.array_equal(a["counters"][name], b["counters"][name]), name
    assert np.array_equal(a["completion_step"], b["completion_step"])
