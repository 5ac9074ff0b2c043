"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle is checked against things other than itself: published Philox
vectors, numpy's searchsorted for table inversion, values the paper prints,
hand-computed trajectories, the Lindley recursion of the proof of Theorem 1,
conservation identities, Little's law and the direction of Proposition 2.
"""
import json
import math
import os

import numpy as np
import pytest

import oracle
from workloads import FLOW, GREEDY, configs, laws
from workloads.configs import Workload, flow_cell, greedy_cell

INF = 1 << 30


# ---------------------------------------------------------------- Philox ----

def test_philox_known_answers(golden_dir):
    rows = 0
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            out = oracle.philox(w[0:4], w[4:6])
            assert [int(x) for x in out] == w[6:10]
            rows += 1
    assert rows == 3


def test_philox_counter_sensitivity():
    # flipping any single counter or key word changes the block (catches an unused word)
    base = oracle.philox([1, 2, 3, 4], [5, 6])
    for i in range(4):
        c = [1, 2, 3, 4]
        c[i] ^= 1
        assert not np.array_equal(oracle.philox(c, [5, 6]), base)
    assert not np.array_equal(oracle.philox([1, 2, 3, 4], [4, 6]), base)
    assert not np.array_equal(oracle.philox([1, 2, 3, 4], [5, 7]), base)


# ------------------------------------------------------- table inversion ----

@pytest.mark.parametrize("law", [
    laws.uniform_int(16, 256), laws.geometric(128.0, cap=1024), laws.lognormal(6.0, 0.8, 8, 8192),
    laws.pareto(1.5, 32.0, 32768), laws.poisson_counts(2.13), laws.bernoulli_counts(0.05), laws.point(7),
])
def test_inversion_matches_searchsorted(law):
    rng = np.random.default_rng(3)
    u = rng.integers(0, 1 << 32, size=20000, dtype=np.uint64).astype(np.uint32)
    edge = [0, 1, (1 << 32) - 1, (1 << 32) - 2]
    for t in law.thr[:: max(1, law.thr.size // 50)]:
        edge += [int(t), max(int(t) - 1, 0), min(int(t) + 1, (1 << 32) - 1)]
    u = np.concatenate([u, np.array(edge, dtype=np.uint32)])
    got = oracle.invert(law, u)
    assert np.array_equal(got, law.sample(u))
    assert got.min() >= law.lo and got.max() <= law.hi


def test_table_masses_match_the_continuous_laws():
    # the quantised tables reproduce textbook moments of the laws they discretise
    assert abs(laws.uniform_int(16, 256).moment(1) - 136.0) < 1e-6
    g = laws.geometric(256.0)
    assert abs(g.moment(1) - 256.0) < 1e-4
    assert abs(g.moment(2) - (2 - 1 / 256.0) * 256.0**2) / 256.0**2 < 1e-6
    p = laws.poisson_counts(0.9)
    assert abs(p.moment(1) - 0.9) < 1e-7 and abs(p.moment(2) - (0.9 + 0.81)) < 1e-6
    assert abs(laws.bernoulli_counts(0.05).moment(1) - 0.05) < 1e-9


# ------------------------------------------------------------ closed forms --

def test_paper_closed_forms(golden_dir):
    with open(os.path.join(golden_dir, "paper_closed_forms.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    ws = {}
    for r in rows:
        if r[0] == "w":
            l, o, w = int(r[1]), int(r[2]), int(r[3])
            assert oracle.workload(l, o) == w
            assert sum(l + j for j in range(1, o + 1)) == w
            ws[o] = w
        elif r[0] == "eq2":
            b = [int(x) for x in r[1:4]]
            M, total = int(r[4]), int(r[5])
            assert sum(bk * w for bk, w in zip(b, [ws[20], ws[40], ws[60]])) == total < M
    # equal-rate three-class mixture: E[w] = 4060/3
    wl = configs.three_class(1.0)
    assert abs(oracle.expected_workload(wl.mixture) - 4060.0 / 3.0) < 1e-6
    assert abs(oracle.stability_bound(wl.mixture, 16492) - 3 * 16492 / 4060.0) < 1e-8


def test_expected_workload_equals_brute_force_double_sum():
    rng = np.random.default_rng(5)
    a = laws.from_pmf(3, rng.random(17))
    b = laws.from_pmf(1, rng.random(23))
    c = laws.from_pmf(9, rng.random(5))
    d = laws.from_pmf(2, rng.random(11))
    mix = laws.Mixture((laws.RequestClass(0.3, a, b), laws.RequestClass(0.7, c, d)))
    brute = 0.0
    for pc, cl in zip(mix.class_prob(), mix.classes):
        for l, pl in zip(cl.prompt.values(), cl.prompt.pmf()):
            for o, po in zip(cl.decode.values(), cl.decode.pmf()):
                brute += pc * pl * po * sum(int(l) + j for j in range(1, int(o) + 1))
    assert abs(oracle.expected_workload(mix) - brute) / brute < 1e-12


# ----------------------------------------------------- hand trajectories ----

def _cases(golden_dir):
    with open(os.path.join(golden_dir, "trajectories.json")) as f:
        return json.load(f)["cases"]


def _case_workload(case):
    M = case["M"]
    tau = INF if case["tau"] == "inf" else case["tau"]
    c = INF if case["c"] == "inf" else case["c"]
    cell = flow_cell(0, 1.0) if case["policy"] == "FLOW" else greedy_cell(0)
    mix = laws.single(laws.point(1), laws.point(1))  # unused: arrivals are forced
    return Workload(name=case["name"], capacity=M, token_budget=tau, prefill_chunk=c, mixture=mix,
                    arrival_laws=(laws.poisson_counts(0.0),), cells=(cell,), n_replicas=1,
                    n_steps=case["T"], seed=1, max_requests=16)


def test_hand_trajectories(golden_dir):
    cases = _cases(golden_dir)
    assert len(cases) >= 8
    for case in cases:
        wl = _case_workload(case)
        req = np.array(case["requests"], dtype=np.int32)
        r = oracle.run_cell(wl, 0, replica_ids=[0], per_step=True,
                            forced=(req[:, 0], req[:, 1], req[:, 2]), forced_B=case["B"])
        name = case["name"]
        assert r["step_u"][0].tolist() == case["U"], name
        assert r["step_p"][0].tolist() == case["P"], name
        assert r["step_q"][0].tolist() == case["Q"], name
        n = len(case["requests"])
        assert r["completion_step"][0, :n].tolist() == case["completion"], name
        lat = (r["completion_step"][0, :n] - r["arrival_step"][0, :n] + 1).tolist()
        assert lat == case["latency"], name
        cnt = r["counters"]
        assert int(cnt["sum_latency"][0]) == sum(case["latency"]), name
        assert int(cnt["completed"][0]) == n and int(cnt["arrived"][0]) == n, name
        assert int(cnt["sum_u"][0]) == sum(case["U"]) and int(cnt["sum_p"][0]) == sum(case["P"]), name
        assert int(cnt["sum_q"][0]) == sum(case["Q"]), name
        assert int(cnt["max_u"][0]) == max(case["U"]), name
        for k, v in case["counters"].items():
            assert int(cnt[k][0]) == v, (name, k)


# ------------------------------------- Lindley recursion / pure-model timing --

def test_flow_queue_is_lindley_and_requests_live_o_slots():
    # Huge M: no eviction, so Q_t = (Q_{t-1} + n_t - B_t)^+ (proof of Theorem 1) and, with one-chunk
    # prefill and no token budget, a request activated at s completes at s + o - 1 (proof of Theorem 2).
    mix = laws.single(laws.uniform_int(4, 60), laws.geometric(12.0, cap=80))
    wl = Workload(name="lindley", capacity=1 << 28, token_budget=INF, prefill_chunk=INF, mixture=mix,
                  arrival_laws=(laws.poisson_counts(0.7),), cells=(flow_cell(0, 0.8),),
                  n_replicas=6, n_steps=3000, seed=21, max_requests=4096)
    r = oracle.run_cell(wl, 0, per_step=True)
    assert r["counters"]["evictions"].sum() == 0
    for i in range(wl.n_replicas):
        q = 0
        n, b = r["step_n"][i], r["step_b"][i]
        for t in range(wl.n_steps):
            q = max(q + int(n[t]) - int(b[t]), 0)
            assert q == r["step_q"][i, t]
        done = r["completion_step"][i] > 0
        assert done.sum() > 1000
        assert np.array_equal(r["completion_step"][i][done],
                              (r["first_activation"][i] + r["req_o"][i] - 1)[done])
        assert np.array_equal(r["first_activation"][i][done], r["last_activation"][i][done])
        # usage by the closed expression in the proof of Theorem 2
        act, l, o = r["first_activation"][i], r["req_l"][i], r["req_o"][i]
        started = act > 0
        for t in (1, 7, 500, 1777, 3000):
            age = t - act[started] + 1
            alive = (age >= 1) & (o[started] >= age)
            assert int(np.sum((l[started] + age)[alive])) == r["step_u"][i, t - 1]


def test_draws_follow_the_tables():
    # empirical frequencies of n_t, B_t, l, o against the table masses (5-sigma bands), and
    # independence of l and o (they must come from different words of the block)
    mix = laws.single(laws.uniform_int(4, 60), laws.geometric(12.0, cap=80))
    lam, b = 0.9, 1.3
    wl = Workload(name="draws", capacity=1 << 28, token_budget=INF, prefill_chunk=INF, mixture=mix,
                  arrival_laws=(laws.poisson_counts(lam),), cells=(flow_cell(0, b),),
                  n_replicas=8, n_steps=20000, seed=33, max_requests=1 << 15)
    r = oracle.run_cell(wl, 0, per_step=True)
    n = r["step_n"].ravel().astype(np.float64)
    N = n.size
    assert abs(n.mean() - lam) < 5 * math.sqrt(lam / N)
    assert abs(n.var() - lam) < 0.03
    pm = wl.arrival_laws[0].pmf()
    for k in range(4):
        f = np.mean(n == k)
        assert abs(f - pm[k]) < 5 * math.sqrt(pm[k] * (1 - pm[k]) / N)
    bt = r["step_b"].ravel()
    assert set(np.unique(bt)) == {1, 2}
    assert abs(np.mean(bt == 2) - 0.3) < 5 * math.sqrt(0.21 / N)
    # n_t and B_t come from different words: uncorrelated
    assert abs(np.corrcoef(n, bt)[0, 1]) < 5 / math.sqrt(N)
    have = r["arrival_step"] > 0
    l = r["req_l"][have].astype(np.float64)
    o = r["req_o"][have].astype(np.float64)
    K = l.size
    L, O = mix.classes[0].prompt, mix.classes[0].decode
    assert abs(l.mean() - L.moment(1)) < 5 * math.sqrt((L.moment(2) - L.moment(1) ** 2) / K)
    assert abs(o.mean() - O.moment(1)) < 5 * math.sqrt((O.moment(2) - O.moment(1) ** 2) / K)
    assert abs(np.corrcoef(l, o)[0, 1]) < 5 / math.sqrt(K)
    # different replicas and different arrivals of one slot see different words
    assert not np.array_equal(r["step_n"][0], r["step_n"][1])
    same_slot = np.nonzero(r["step_n"][0] >= 2)[0]
    assert same_slot.size > 100
    ids = np.cumsum(r["step_n"][0]) - r["step_n"][0]
    pairs = np.array([(r["req_l"][0, ids[t]], r["req_l"][0, ids[t] + 1]) for t in same_slot])
    assert np.mean(pairs[:, 0] == pairs[:, 1]) < 0.2


def test_two_class_mixture_draws():
    short = laws.RequestClass(0.7, laws.point(5), laws.point(3))
    long_ = laws.RequestClass(0.3, laws.point(50), laws.point(9))
    wl = Workload(name="mix", capacity=1 << 28, token_budget=INF, prefill_chunk=INF,
                  mixture=laws.Mixture((short, long_)), arrival_laws=(laws.poisson_counts(0.5),),
                  cells=(flow_cell(0, 3.0),), n_replicas=4, n_steps=20000, seed=9, max_requests=1 << 15)
    r = oracle.run_cell(wl, 0)
    have = r["arrival_step"] > 0
    l, o = r["req_l"][have], r["req_o"][have]
    assert set(np.unique(l)) == {5, 50}
    assert np.array_equal(o[l == 5], np.full((l == 5).sum(), 3))
    assert np.array_equal(o[l == 50], np.full((l == 50).sum(), 9))
    f = np.mean(l == 50)
    assert abs(f - 0.3) < 5 * math.sqrt(0.21 / l.size)


# ------------------------------------------------------------ conservation --

def _toy_runs():
    wl = configs.toy()
    for ci in range(len(wl.cells)):
        yield wl, ci, oracle.run_cell(wl, ci, per_step=True)
    wl2 = configs.toy(capacity=300, token_budget=40, prefill_chunk=8, lam=0.9, b=1.5, seed=12)
    for ci in range(len(wl2.cells)):
        yield wl2, ci, oracle.run_cell(wl2, ci, per_step=True)


def test_conservation_and_bounds_on_eviction_heavy_runs():
    saw_evictions = saw_stalls = False
    for wl, ci, r in _toy_runs():
        c = {k: v.astype(np.int64) for k, v in r["counters"].items()}
        T, M = wl.n_steps, wl.capacity
        assert np.array_equal(c["arrived"], c["final_q"] + c["final_p"] + c["completed"])
        assert np.all(c["max_u"] <= M) and np.all(c["sum_u"] <= M * T)
        assert np.all(r["step_u"] + r["step_p"] * 0 <= M)
        assert np.array_equal(c["activations"], c["completed"] + c["evictions"] + c["final_p"])
        assert np.array_equal(c["arrived"], r["step_n"].sum(axis=1))
        assert np.array_equal(c["sum_p"], r["step_p"].sum(axis=1))
        # every slot spends at most tau budget tokens; first tokens ride on the last chunk for free
        assert np.all(c["prefill_tokens"] + c["decode_tokens"] - c["activations"] <= wl.token_budget * T)
        # a request in P either gets a token, stalls, or is still prefilling
        assert np.all(c["decode_tokens"] + c["stalled"] <= c["sum_p"])
        for i in range(wl.n_replicas):
            arr, comp = r["arrival_step"][i], r["completion_step"][i]
            n = int(c["arrived"][i])
            assert n <= wl.max_requests
            arr, comp = arr[:n].astype(np.int64), comp[:n].astype(np.int64)
            l, o = r["req_l"][i][:n].astype(np.int64), r["req_o"][i][:n].astype(np.int64)
            assert np.all(arr >= 1) and np.all(np.diff(arr) >= 0)
            done = comp > 0
            assert done.sum() == c["completed"][i]
            # Little's law, exact sample-path form: sum_t N_t = sum_i sojourn_i (truncated at T)
            sojourn = np.where(done, comp, T) - arr + 1
            assert sojourn.sum() == c["sum_p"][i] + c["sum_q"][i]
            assert c["sum_latency"][i] == sojourn[done].sum()
            assert c["useful_tokens"][i] == o[done].sum()
            # proof of Proposition 1: completed work fits in the M*T budget, and each completed
            # request held at least w_i of it
            w = l * o + o * (o + 1) // 2
            assert w[done].sum() <= c["sum_u"][i] <= M * T
            # nobody finishes faster than its chunked prefill plus o - 1 further tokens
            fastest = -(-l // wl.prefill_chunk) + o - 1
            assert np.all((comp - arr + 1)[done] >= fastest[done])
            # under GREEDY nothing is admitted that does not fit (l + 1 on top of provisioned usage)
        saw_evictions |= bool(c["evictions"].sum() > 0)
        saw_stalls |= bool(c["stalled"].sum() > 0)
    assert saw_evictions and saw_stalls


def test_final_state_digest_distinguishes_runs():
    wl = configs.toy()
    a = oracle.run_cell(wl, 0)["counters"]["digest"]
    b = oracle.run_cell(wl, 0)["counters"]["digest"]
    c = oracle.run_cell(wl, 0, seed=wl.seed + 1)["counters"]["digest"]
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert np.unique(a).size == a.size


def test_policies_share_random_streams():
    wl = configs.toy()
    f = oracle.run_cell(wl, 0, per_step=True)
    g = oracle.run_cell(wl, 1, per_step=True)
    assert np.array_equal(f["step_n"], g["step_n"])
    assert np.array_equal(f["req_l"], g["req_l"]) and np.array_equal(f["req_o"], g["req_o"])
    assert not np.array_equal(f["step_u"], g["step_u"])


def test_replica_subset_equals_full_run():
    wl = configs.toy(n_replicas=12)
    full = oracle.run_cell(wl, 0)
    sub = oracle.run_cell(wl, 0, replica_ids=[3, 7, 11], n_threads=2)
    for k, v in full["counters"].items():
        assert np.array_equal(v[[3, 7, 11]], sub["counters"][k]), k
    assert np.array_equal(full["trace_u"][[3, 7, 11]], sub["trace_u"])


def test_histogram_percentile_is_nearest_rank():
    wl = configs.toy(hist_bins=4096, hist_shift=0, n_steps=3000)
    r = oracle.run_cell(wl, 0)
    for i in range(wl.n_replicas):
        done = r["completion_step"][i] > 0
        lat = np.sort((r["completion_step"][i] - r["arrival_step"][i] + 1)[done])
        assert lat.size == r["hist"][i].sum() and lat.size > 100
        for num, den in ((99, 100), (95, 100), (1, 2)):
            k = -(-num * lat.size // den)
            val, sat = oracle.percentile_from_hist(r["hist"][i], num, den, 0)
            assert not sat and val == lat[k - 1]


def test_trace_samples_every_k_steps():
    wl = configs.toy(trace_every=25, n_steps=400)
    r = oracle.run_cell(wl, 1, per_step=True)
    assert r["trace_u"].shape == (wl.n_replicas, 16)
    assert np.array_equal(r["trace_u"], r["step_u"][:, 24::25])
    assert np.array_equal(r["trace_q"], r["step_q"][:, 24::25])


# ------------------------------------------------------------- stability ----

def test_single_class_flow_never_overflows_when_b_w_below_M():
    # Theorem 1 with one class: b*w < M and b > lambda => usage never exceeds b*w, no eviction,
    # and the waiting queue is the Lindley recursion.  (l,o) = (10,60): w = 2430, b = 6.
    mix = laws.single(laws.point(10), laws.point(60))
    wl = Workload(name="thm1", capacity=16492, token_budget=INF, prefill_chunk=INF, mixture=mix,
                  arrival_laws=(laws.poisson_counts(5.0),), cells=(flow_cell(0, 6.0),),
                  n_replicas=4, n_steps=5000, seed=3, max_requests=0)
    r = oracle.run_cell(wl, 0, per_step=True)
    assert r["counters"]["evictions"].sum() == 0
    assert r["counters"]["max_u"].max() <= 6 * 2430
    assert r["counters"]["max_u"].max() > 0.7 * 6 * 2430       # and the bound is nearly attained
    for i in range(wl.n_replicas):
        q = 0
        for t in range(wl.n_steps):
            q = max(q + int(r["step_n"][i, t]) - 6, 0)
            assert q == r["step_q"][i, t]
    assert r["step_q"][:, -1].max() < 200                        # positive recurrent, not drifting


def test_queue_explodes_above_the_bound_under_both_policies():
    # Proposition 1/2: lambda*E[w] > M  =>  unfinished requests grow at least delta/w_max per slot.
    # Paper's synthetic set-up with lambda = 5 per class: delta = 20300 - 16492, w_max = 2430.
    wl = configs.three_class(5.0, n_replicas=4, n_steps=6000)
    rate_floor = (5 * 4060 - 16492) / 2430.0
    for ci in range(2):
        c = oracle.run_cell(wl, ci)["counters"]
        growth = (c["arrived"].astype(np.float64) - c["completed"]) / wl.n_steps
        # the finite-horizon slack of the proof is at most one active set's worth of requests
        assert np.all(growth > rate_floor - 0.05), (ci, growth, rate_floor)
        # and completed work respects the capacity budget
        assert np.all(c["sum_u"] <= 16492 * wl.n_steps)


def test_little_law_long_run():
    wl = configs.config0(oracle.stability_bound).scaled(n_replicas=8, n_steps=60000)
    c = oracle.run_cell(wl, 0, n_threads=4)["counters"]
    T = wl.n_steps
    mean_n = (c["sum_p"].sum() + c["sum_q"].sum()) / (8.0 * T)
    thr = c["completed"].sum() / (8.0 * T)
    lat = c["sum_latency"].sum() / c["completed"].sum()
    assert abs(mean_n - thr * lat) / mean_n < 0.01
    assert abs(thr - 0.05) < 0.002
