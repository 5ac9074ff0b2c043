"""More pins for the CPU oracle (no GPU): the latency histogram with a bucket shift, the sample-path bound
of the proof of Theorem 2, and the whole oracle replayed under the host compiler's sanitizers."""
import json
import os

import numpy as np
import pytest

import oracle
from workloads import configs, laws
from workloads.configs import Workload, flow_cell, greedy_cell

INF = 1 << 30


# ------------------------------------------------- histogram with a shift ----

@pytest.mark.parametrize("shift,bins", [(1, 4096), (3, 512), (1, 24), (3, 7)])
def test_histogram_buckets_and_percentiles_with_a_shift(shift, bins):
    # bucket = min(latency >> shift, bins - 1); the percentile is the lower edge of the bucket of the
    # ceil(q n)-th smallest latency, flagged when that is the last bucket.  The small bin counts saturate.
    wl = configs.toy(hist_bins=bins, hist_shift=shift, n_steps=3000)
    for ci in range(len(wl.cells)):
        r = oracle.run_cell(wl, ci)
        for i in range(wl.n_replicas):
            done = r["completion_step"][i] > 0
            lat = np.sort((r["completion_step"][i] - r["arrival_step"][i] + 1)[done].astype(np.int64))
            assert lat.size > 100
            want = np.bincount(np.minimum(lat >> shift, bins - 1), minlength=bins)
            assert np.array_equal(r["hist"][i], want)
            for num, den in ((99, 100), (95, 100), (1, 2), (1, 100), (1, 1)):
                k = max(-(-num * lat.size // den), 1)
                bucket = min(int(lat[k - 1]) >> shift, bins - 1)
                val, sat = oracle.percentile_from_hist(r["hist"][i], num, den, shift)
                assert val == bucket << shift and sat == (bucket == bins - 1), (num, den, val, bucket)
    if bins <= 24:
        assert r["hist"][:, -1].sum() > 0      # the last bucket really collected the tail


# ------------------------------------------- proof of Theorem 2: U_t <= U^_t ----

def test_usage_is_dominated_by_the_usage_of_full_budgets():
    # Proof of Theorem 2: with a_s <= B_s requests activated at slot s and nobody evicted,
    #   U_t = sum_s sum_{p <= a_s} (l_{s,p} + t - s + 1) 1(o_{s,p} >= t - s + 1)
    # and filling every slot up to B_s requests with further draws from nu gives U^_t >= U_t with
    # E[U^_t] = b E[l o + (o + o^2)/2] once t exceeds the longest output.
    o_cap = 80
    mix = laws.single(laws.uniform_int(4, 60), laws.geometric(12.0, cap=o_cap))
    b = 0.8
    wl = Workload(name="u-hat", capacity=1 << 28, token_budget=INF, prefill_chunk=INF, mixture=mix,
                  arrival_laws=(laws.poisson_counts(0.7),), cells=(flow_cell(0, b),),
                  n_replicas=8, n_steps=6000, seed=33, max_requests=8192)
    r = oracle.run_cell(wl, 0, per_step=True)
    assert r["counters"]["evictions"].sum() == 0
    T = wl.n_steps
    rng = np.random.default_rng(7)
    cls = mix.classes[0]
    means = []
    for i in range(wl.n_replicas):
        n = int(r["counters"]["arrived"][i])
        act, l, o = r["first_activation"][i][:n], r["req_l"][i][:n], r["req_o"][i][:n]
        on = act > 0
        assert np.array_equal(act[on], r["last_activation"][i][:n][on])   # nobody is activated twice
        a = np.bincount(act[on], minlength=T + 1)[1:T + 1]
        B = r["step_b"][i].astype(np.int64)
        assert np.all(a <= B)
        # the real requests, then the fictitious ones that fill B_s - a_s
        fs = np.repeat(np.arange(1, T + 1), B - a)
        u32 = rng.integers(0, 1 << 32, size=(2, fs.size), dtype=np.uint64).astype(np.uint32)
        fl, fo = cls.prompt.sample(u32[0]), cls.decode.sample(u32[1])

        def usage(starts, ls, os_):
            u = np.zeros(T + 2 + o_cap, np.int64)
            for q in range(1, o_cap + 1):           # token q is held in slot s + q - 1 by requests with o >= q
                m = os_ >= q
                np.add.at(u, starts[m] + q - 1, ls[m] + q)
            return u[1:T + 1]

        real = usage(act[on].astype(np.int64), l[on].astype(np.int64), o[on].astype(np.int64))
        assert np.array_equal(real, r["step_u"][i])                       # the expression for U_t itself
        hat = real + usage(fs, fl.astype(np.int64), fo.astype(np.int64))
        assert np.all(r["step_u"][i] <= hat)
        full = np.convolve((a == B).astype(np.int64), np.ones(o_cap, np.int64))[:T] == np.minimum(np.arange(1, T + 1), o_cap)
        assert np.array_equal(hat[full], r["step_u"][i][full])            # equality where every budget was used
        means.append(hat[o_cap:].mean())
    want = b * oracle.expected_workload(mix)
    # the replicas are independent: their means scatter around b E[w] with the standard error seen
    se = np.std(means, ddof=1) / np.sqrt(len(means))
    assert abs(np.mean(means) - want) < 4.0 * se + 0.01 * want, (np.mean(means), want, se)


# ------------------------------------------- the oracle under ASan and UBSan ----

@pytest.fixture(scope="module")
def sanitized(tmp_path_factory):
    return oracle.build_sanitized(str(tmp_path_factory.mktemp("asan")))


def _same(rows, ref, label):
    for i, (cnt, comp, hist) in enumerate(rows):
        for k, v in cnt.items():
            assert int(ref["counters"][k][i]) == v, (label, k, i)
        if "completion_step" in ref:
            assert np.array_equal(comp, ref["completion_step"][i]), (label, "completion", i)
        if "hist" in ref:
            assert np.array_equal(hist, ref["hist"][i]), (label, "hist", i)


def test_sanitized_replay_of_the_hand_trajectories(sanitized, golden_dir):
    with open(os.path.join(golden_dir, "trajectories.json")) as f:
        cases = json.load(f)["cases"]
    for case in cases:
        tau = INF if case["tau"] == "inf" else case["tau"]
        c = INF if case["c"] == "inf" else case["c"]
        cell = flow_cell(0, 1.0) if case["policy"] == "FLOW" else greedy_cell(0)
        wl = Workload(name=case["name"], capacity=case["M"], token_budget=tau, prefill_chunk=c,
                      mixture=laws.single(laws.point(1), laws.point(1)), arrival_laws=(laws.poisson_counts(0.0),),
                      cells=(cell,), n_replicas=1, n_steps=case["T"], seed=1, max_requests=16)
        req = np.array(case["requests"], dtype=np.int32)
        forced = (req[:, 0], req[:, 1], req[:, 2])
        rows = oracle.replay(sanitized, oracle.case_tokens(wl, 0, [0], forced=forced, forced_B=case["B"]))
        n = len(case["requests"])
        assert rows[0][1][:n].tolist() == case["completion"], case["name"]
        assert rows[0][0]["sum_u"] == sum(case["U"]) and rows[0][0]["sum_p"] == sum(case["P"]), case["name"]
        for k, v in case["counters"].items():
            assert rows[0][0][k] == v, (case["name"], k)


def test_sanitized_replay_of_every_policy(sanitized):
    # no address or undefined-behaviour report on eviction-heavy, stalling, chunked, overloaded runs of every
    # policy, budget form and the time model, and the same numbers as the shared library gives
    obs = dict(trace_every=25, hist_bins=64, hist_shift=1, max_requests=2048)
    toy = configs.toy(n_replicas=3, n_steps=500)
    cases = [
        toy,
        configs.toy(capacity=300, token_budget=40, prefill_chunk=8, lam=0.9, b=1.5, seed=12, n_replicas=2, n_steps=500),
        toy.scaled(cells=(configs.flow_law_cell(0, 0), configs.flow_credit_cell(0, 1.3))),
        toy.scaled(time_model=(2, 1, 1)),
        configs.known_classes(n_replicas=2, n_steps=300, **obs),
        configs.known_classes(lam_per_class=(0.3, 0.2, 0.25), budgets=(1, 1, 2), lengths=((37, 5), (9, 30), (64, 1)),
                              token_budget=48, prefill_chunk=16, capacity=4000, n_replicas=2, n_steps=600, seed=22, **obs),
        configs.alpha_sweep(n_replicas=2, n_steps=300, **obs),
        configs.unknown_types(n_replicas=2, n_steps=200, **obs),
    ]
    for wl in cases:
        ids = list(range(wl.n_replicas))
        for ci in range(len(wl.cells)):
            rows = oracle.replay(sanitized, oracle.case_tokens(wl, ci, ids))
            _same(rows, oracle.run_cell(wl, ci), f"{wl.name} cell {ci}")
