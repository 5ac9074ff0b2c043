"""Element-by-element comparison of a GPU run with the CPU oracle on the same seeded inputs."""
import numpy as np

import oracle

# integer state compared bit-exactly; the engine's extra counters (error, error_step) are checked apart
SHARED = None


def shared_counters(got):
    return [n for n in oracle.counter_names() if n in got]


def compare(engine, wl, replica_ids=None, n_threads=8, check_requests=True, label=""):
    """Runs the oracle for the given replicas of every cell and asserts equality with the engine."""
    got, summary = engine.stats()
    R, T = engine.n_replicas, engine.n_steps
    ids = np.arange(R) if replica_ids is None else np.asarray(replica_ids)
    assert not np.any(got["error"]), (label, got["error"].nonzero())
    names = shared_counters(got)
    assert len(names) == len(oracle.counter_names()), "engine lacks an oracle counter"
    trace_q = engine.trace_q.cpu().numpy() if engine.trace_q is not None else None
    trace_u = engine.trace_u.cpu().numpy() if engine.trace_u is not None else None
    hist = engine.hist.cpu().numpy().view(np.uint32) if engine.hist is not None else None
    arr = engine.arrival_step.cpu().numpy() if engine.arrival_step is not None else None
    comp = engine.completion_step.cpu().numpy() if engine.completion_step is not None else None
    if hist is not None:
        p99, sat = engine.percentile(99, 100)
        p50, _ = engine.percentile(1, 2)
    totals = {}
    for ci in range(len(wl.cells)):
        ref = oracle.run_cell(wl, ci, replica_ids=ids, n_steps=T, n_threads=n_threads)
        rows = ci * R + ids
        for name in names:
            a, b = ref["counters"][name], got[name][rows]
            assert np.array_equal(a, b), (label, "cell", ci, name, np.nonzero(a != b)[0][:5], a[:4], b[:4])
        if trace_q is not None:
            assert np.array_equal(ref["trace_q"], trace_q[rows]), (label, ci, "trace_q")
            assert np.array_equal(ref["trace_u"], trace_u[rows]), (label, ci, "trace_u")
        if hist is not None:
            assert np.array_equal(ref["hist"], hist[rows]), (label, ci, "hist")
            for k, r in enumerate(rows):
                v, s = oracle.percentile_from_hist(ref["hist"][k], 99, 100, wl.hist_shift)
                assert (v, s) == (int(p99[r]), bool(sat[r])), (label, ci, "p99", r)
                v, s = oracle.percentile_from_hist(ref["hist"][k], 1, 2, wl.hist_shift)
                assert v == int(p50[r]), (label, ci, "p50", r)
        if arr is not None and check_requests:
            assert np.array_equal(ref["arrival_step"], arr[rows]), (label, ci, "arrival_step")
            assert np.array_equal(ref["completion_step"], comp[rows]), (label, ci, "completion_step")
        totals[ci] = ref
    return got, summary, totals


def check_summary(engine, wl, got, rel=1e-9):
    """Derived floating-point statistics against the same ratios formed from oracle-checked integers."""
    R, T, M = engine.n_replicas, engine.n_steps, wl.capacity
    for ci in list(range(len(wl.cells))) + [-1]:
        _, s = engine.stats(cell=ci)
        rows = slice(None) if ci < 0 else slice(ci * R, (ci + 1) * R)
        n = got["sum_p"][rows].size
        f = lambda name: float(np.sum(got[name][rows].astype(np.float64)))
        done = f("completed")
        want = {
            "mean_latency": f("sum_latency") / done if done else 0.0,
            "kv_utilisation": f("sum_u") / (n * T * M),
            "token_throughput": f("useful_tokens") / (n * T),
            "prompt_throughput": done / (n * T),
            "mean_queue": f("sum_q") / (n * T),
            "mean_active": f("sum_p") / (n * T),
        }
        for k, v in want.items():
            assert abs(s[k] - v) <= rel * max(abs(v), 1e-300), (ci, k, s[k], v)
        assert s["request_steps"] == int(got["sum_p"][rows].sum())
