"""Pins of the oracle's other forms of the activation budget B_t of Algorithm 2 (Theorem 2: any i.i.d.
bounded nonnegative integer law with mean b; and a deterministic credit accumulator): CPU only."""
from fractions import Fraction

import numpy as np

import oracle
from workloads import configs, laws
from workloads.configs import Workload, flow_cell, flow_credit_cell, flow_law_cell

INF = 1 << 30


def _workload(cells, extra_laws=(), lam=1.1, T=4000, n_replicas=6, seed=60, capacity=1 << 28):
    mix = laws.single(laws.uniform_int(4, 40), laws.geometric(20.0, cap=200))
    return Workload(name="budget-pin", capacity=capacity, token_budget=INF, prefill_chunk=INF, mixture=mix,
                    arrival_laws=(laws.poisson_counts(lam),) + tuple(extra_laws), cells=tuple(cells),
                    n_replicas=n_replicas, n_steps=T, seed=seed)


def _lindley(r):
    """Q_t = (Q_{t-1} + n_t - B_t)^+ with the oracle's own per-slot n_t and B_t (memory never binds)."""
    n, b, q = (r[k].astype(np.int64) for k in ("step_n", "step_b", "step_q"))
    prev = np.zeros(n.shape[0], np.int64)
    for t in range(n.shape[1]):
        prev = np.maximum(prev + n[:, t] - b[:, t], 0)
        assert np.array_equal(prev, q[:, t]), t


def test_credit_accumulator_is_floor_of_t_b_differences():
    for b in (1.25, 0.3, 2.0, 1.1):
        cell = flow_credit_cell(0, b)
        bq = Fraction(cell.credit_b16, 65536)
        wl = _workload([cell], T=3000, n_replicas=3)
        r = oracle.run_cell(wl, 0, per_step=True)
        want = [int(t * bq) - int((t - 1) * bq) for t in range(1, 3001)]     # Fraction -> int floors
        for i in range(3):
            assert r["step_b"][i].tolist() == want                          # the same on every replica
        assert np.array_equal(np.cumsum(want), [int(t * bq) for t in range(1, 3001)])
        assert set(want) <= {int(bq), int(bq) + 1}
        assert not r["counters"]["evictions"].any()
        _lindley(r)
    first = oracle.run_cell(_workload([flow_credit_cell(0, 1.25)], T=8), 0, per_step=True)["step_b"][0]
    assert first.tolist() == [1, 1, 1, 2, 1, 1, 1, 2]


def test_budget_from_a_bounded_law_is_iid_with_that_law():
    pmf = np.array([0.15, 0.35, 0.2, 0.05, 0.25])          # on {0, ..., 4}: mean 1.9, A = 4
    law = laws.from_pmf(0, pmf)
    wl = _workload([flow_law_cell(0, 1)], extra_laws=(law,), lam=1.6, T=20000, n_replicas=8)
    r = oracle.run_cell(wl, 0, per_step=True, n_threads=8)
    b = r["step_b"].astype(np.int64)
    n = r["step_n"].astype(np.int64)
    assert b.min() >= 0 and b.max() == 4
    N = b.size
    freq = np.bincount(b.ravel(), minlength=5) / N
    assert np.all(np.abs(freq - pmf) < 5 * np.sqrt(pmf * (1 - pmf) / N))
    # independent of the arrivals of the same slot (the two come from different words of one block) and
    # of the budget of the next slot
    for x, y in ((b.ravel(), n.ravel()), (b[:, :-1].ravel(), b[:, 1:].ravel())):
        assert abs(np.corrcoef(x, y)[0, 1]) < 5 / np.sqrt(N)
    # replicas draw different sequences
    assert not np.array_equal(b[0], b[1])
    # word 1 of the slot's block against the law's table, value = lo + #{thr <= u}
    key = (wl.seed & 0xffffffff, wl.seed >> 32)
    for t in (1, 2, 777):
        u = np.array([oracle.philox([0, t, 3, 0], key)[1]], np.uint32)
        assert int(oracle.invert(law, u)[0]) == int(b[3, t - 1])
    _lindley(r)


def test_bernoulli_split_is_the_two_point_case_in_law():
    # B = floor(b) + Bernoulli(frac) and the two-point law with the same masses: same law of B_t, and
    # the same long-run queue (not the same path: the two read the random word from opposite ends)
    b = 1.3
    two_point = laws.from_pmf(1, np.array([0.7, 0.3]))
    wl = _workload([flow_cell(0, b), flow_law_cell(0, 1)], extra_laws=(two_point,), lam=1.2, T=30000,
                   n_replicas=8)
    a, c = (oracle.run_cell(wl, i, per_step=True, n_threads=8) for i in (0, 1))
    ma, mc = a["step_b"].mean(), c["step_b"].mean()
    assert abs(ma - b) < 0.01 and abs(mc - b) < 0.01
    qa, qc = a["step_q"].mean(), c["step_q"].mean()
    assert abs(qa - qc) < 0.25 * max(qa, qc)


def test_overflow_events_fall_as_the_memory_grows_at_a_fixed_margin():
    # Theorem 2: with b E[w] <= (1 - eps) M the expected number of overflow events is below T exp(-C M^2).
    # The constant is not given, so only the direction is checked: same eps and lambda / b, growing M
    # (b and lambda grow with it), and a larger margin at one M.
    mix = laws.single(laws.uniform_int(4, 40), laws.geometric(20.0, cap=120))
    ew = oracle.expected_workload(mix)

    def overflows(M, eps):
        b = (1.0 - eps) * M / ew
        wl = Workload(name="thm2", capacity=M, token_budget=INF, prefill_chunk=INF, mixture=mix,
                      arrival_laws=(laws.poisson_counts(0.97 * b),), cells=(flow_cell(0, b),), n_replicas=16,
                      n_steps=20000, seed=80)
        return int(oracle.run_cell(wl, 0, n_threads=8)["counters"]["overflow_steps"].sum())

    counts = [overflows(M, 0.1) for M in (1500, 3000, 6000, 12000)]
    assert counts[0] > counts[1] > counts[2] > counts[3] > 0, counts
    assert counts[3] < 0.2 * counts[0]
    assert overflows(6000, 0.3) < 0.2 * counts[2]
