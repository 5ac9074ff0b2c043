"""Pins of the oracle's Algorithm 1 (Section 3.2: known lengths, per-class budgets b_k) against things
fixed outside it: a hand-computed trajectory, the memory bound and the Lindley recursion of the proof
of Theorem 1, the closed form of a request's life in the pure model, and the one-class special case,
which is Algorithm 2 with a constant budget."""
import json
import os

import numpy as np

import oracle
from workloads import configs, laws
from workloads.configs import Workload, classes_cell, flow_cell
from workloads.laws import Mixture, RequestClass

INF = 1 << 30


def _class_workload(lengths, budgets, rates, M, T, n_replicas=1, seed=3, **kw):
    cls = tuple(RequestClass(1.0, laws.point(l), laws.point(o)) for l, o in lengths)
    distinct = sorted(set(rates))
    arr = tuple(laws.poisson_counts(r) for r in distinct)
    cell = classes_cell([distinct.index(r) for r in rates], budgets)
    return Workload(name="alg1", capacity=M, token_budget=INF, prefill_chunk=INF, mixture=Mixture(cls),
                    arrival_laws=arr, cells=(cell,), n_replicas=n_replicas, n_steps=T, seed=seed, **kw)


def test_hand_trajectory(golden_dir):
    with open(os.path.join(golden_dir, "algorithm1_trajectory.json")) as f:
        g = json.load(f)
    wl = _class_workload(g["classes"], g["budgets"], [0.0, 0.0], g["M"], g["T"], max_requests=16)
    arr = np.array(g["arrivals"], dtype=np.int32)
    r = oracle.run_cell(wl, 0, replica_ids=[0], per_step=True, forced=(arr[:, 0], arr[:, 1]))
    assert r["step_u"][0].tolist() == g["U"]
    assert r["step_p"][0].tolist() == g["P"]
    assert r["step_q"][0].tolist() == g["Q"]
    for rid, t in g["completion_by_id"].items():
        assert int(r["completion_step"][0, int(rid)]) == t, rid
    c = r["counters"]
    assert int(c["sum_latency"][0]) == g["latency_sum"]
    assert int(c["sum_u"][0]) == sum(g["U"]) and int(c["sum_p"][0]) == sum(g["P"]) and int(c["sum_q"][0]) == sum(g["Q"])
    for k, v in g["counters"].items():
        assert int(c[k][0]) == v, k


def _class_arrivals(wl, replica, T):
    """n_{t,k} recomputed from the published counter layout: Philox (k, t, replica, 2), word 0."""
    cell = wl.cells[0]
    key = [wl.seed & 0xFFFFFFFF, wl.seed >> 32]
    n = np.zeros((T, len(cell.class_arrival)), np.int64)
    for k, a in enumerate(cell.class_arrival):
        words = np.array([oracle.philox([k, t, replica, 2], key)[0] for t in range(1, T + 1)], np.uint32)
        n[:, k] = oracle.invert(wl.arrival_laws[a], words)
    return n


def test_memory_bound_and_lindley_queues_of_theorem_1():
    # proof of Theorem 1: U_t <= sum_k b_k w_k at all times, no overflow, and each class queue obeys
    # Q_{t,k} = (Q_{t-1,k} + n_{t,k} - b_k)^+ whatever the lengths are
    lengths, budgets = ((10, 20), (10, 40), (10, 60)), (4, 4, 4)
    bound = sum(b * int(oracle.workload(l, o)) for (l, o), b in zip(lengths, budgets))
    assert bound == 16240 < 16492
    T = 600
    for rates, saturated in (((5.0, 5.0, 5.0), True), ((3.0, 3.5, 2.5), False)):
        wl = _class_workload(lengths, budgets, rates, 16492, T, n_replicas=3)
        r = oracle.run_cell(wl, 0, per_step=True)
        c = r["counters"]
        assert np.all(c["overflow_steps"] == 0) and np.all(c["evictions"] == 0)
        assert np.all(c["max_u"] <= bound)
        if saturated:  # every class queue is busy for good after a while: the bound is attained
            assert np.all(c["max_u"] == bound)
        for i, rep in enumerate(r["replica_ids"]):
            n = _class_arrivals(wl, int(rep), T)
            assert np.array_equal(n.sum(axis=1), r["step_n"][i])
            q = np.zeros(len(budgets), np.int64)
            trace = []
            for t in range(T):
                q = np.maximum(q + n[t] - np.array(budgets), 0)
                trace.append(int(q.sum()))
            assert trace == r["step_q"][i].tolist()
            assert int(c["final_q"][i]) == trace[-1] and int(c["max_q"][i]) == max(trace)


def test_each_request_lives_o_slots_after_a_fifo_wait():
    # pure model (chunk >= l, unlimited token budget): a class-k request activated at slot s completes
    # at s + o_k - 1; s follows from serving each class FIFO at b_k per slot
    lengths, budgets, rates = ((3, 5), (7, 2), (1, 9)), (2, 1, 3), (1.6, 0.8, 2.9)
    T = 400
    wl = _class_workload(lengths, budgets, rates, 100000, T, max_requests=4096)
    r = oracle.run_cell(wl, 0, replica_ids=[0])
    n = _class_arrivals(wl, 0, T)
    m = len(lengths)
    lat_sum = done = 0
    for k in range(m):
        arrival_slots = np.repeat(np.arange(1, T + 1), n[:, k])
        served_before = 0
        for t in range(1, T + 1):
            waiting = int((arrival_slots <= t).sum()) - served_before
            take = min(budgets[k], waiting)
            for j in range(served_before, served_before + take):
                rid = j * m + k
                done_at = t + lengths[k][1] - 1
                assert int(r["arrival_step"][0, rid]) == int(arrival_slots[j])
                assert int(r["first_activation"][0, rid]) == t
                assert int(r["completion_step"][0, rid]) == (done_at if done_at <= T else 0)
                if done_at <= T:
                    lat_sum += done_at - int(arrival_slots[j]) + 1
                    done += 1
            served_before += take
    assert int(r["counters"]["completed"][0]) == done
    assert int(r["counters"]["sum_latency"][0]) == lat_sum


def test_one_class_is_algorithm_2_with_a_constant_budget():
    # with a single class, Algorithm 1 and Algorithm 2 with B_t = b move the same requests
    rng = np.random.default_rng(5)
    T, b = 300, 2
    per_slot = rng.poisson(1.7, T)
    slots = np.repeat(np.arange(1, T + 1), per_slot).astype(np.int32)
    l, o = 6, 11
    known = _class_workload(((l, o),), (b,), (0.0,), 100000, T, max_requests=2048)
    flow = Workload(name="flow", capacity=100000, token_budget=INF, prefill_chunk=INF,
                    mixture=laws.single(laws.point(l), laws.point(o)), arrival_laws=(laws.poisson_counts(0.0),),
                    cells=(flow_cell(0, float(b)),), n_replicas=1, n_steps=T, seed=3, max_requests=2048)
    ra = oracle.run_cell(known, 0, replica_ids=[0], per_step=True, forced=(slots, np.zeros_like(slots)))
    rb = oracle.run_cell(flow, 0, replica_ids=[0], per_step=True,
                         forced=(slots, np.full_like(slots, l), np.full_like(slots, o)), forced_B=[b])
    for k in ra["counters"]:
        if k != "digest":
            assert np.array_equal(ra["counters"][k], rb["counters"][k]), k
    for k in ("step_u", "step_p", "step_q", "completion_step", "first_activation"):
        assert np.array_equal(ra[k], rb[k]), k


def test_overflow_is_counted_not_resolved():
    # Algorithm 1 has no eviction step: when sum_k b_k w_k exceeds M the usage simply exceeds M
    wl = _class_workload(((10, 60),), (8,), (9.0,), 5000, 300)
    c = oracle.run_cell(wl, 0, replica_ids=[0])["counters"]
    assert int(c["evictions"][0]) == 0 and int(c["overflow_steps"][0]) > 0 and int(c["max_u"][0]) > 5000
