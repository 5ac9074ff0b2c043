"""fcs_run_static (the entry point that allocates nothing) against fcs_bind + fcs_run, through the C ABI.

Every output array of the two entry points must agree bit for bit: counters (the digest of the final
state among them), traces, histograms, per-request arrival and completion slots.  Two calls in a row share
the library's device array, the second with a smaller input and another engine's tables.
"""
import numpy as np
import pytest

import oracle
import paper_2604_11001_amd as fcs
from workloads import configs, laws
from workloads.configs import Workload, flow_cell, greedy_cell

pytestmark = pytest.mark.gpu


def _outputs(eng):
    got, _ = eng.stats()
    out = dict(got)
    for name in ("trace_q", "trace_u", "hist", "arrival_step", "completion_step"):
        t = getattr(eng, name)
        if t is not None:
            out[name] = t.cpu().numpy()
    return out


def _same(wl, **kw):
    a = fcs.Engine(wl, **kw)
    a.run()
    want = _outputs(a)
    b = fcs.Engine(wl, static_workspace=True, **kw)
    assert b.workspace is None
    b.run()
    got = _outputs(b)
    assert want.keys() == got.keys()
    for k in want:
        assert np.array_equal(want[k], got[k]), (wl.name, k)
    assert not np.any(got["error"])
    assert a.geometry() == b.geometry()
    return b, got


def _spilling(n_replicas=6, n_steps=3000):
    mix = laws.single(laws.uniform_int(1, 8), laws.geometric(40.0, cap=200))
    return Workload(name="static-spill", capacity=12000, token_budget=2000, prefill_chunk=4, mixture=mix,
                    arrival_laws=(laws.poisson_counts(10.0),), cells=(flow_cell(0, 10.6), greedy_cell(0)),
                    n_replicas=n_replicas, n_steps=n_steps, seed=5, trace_every=100, hist_bins=512,
                    max_requests=1 << 15)


def test_static_workspace_matches_a_bound_one_on_two_calls_in_a_row():
    # first call: the active set leaves LDS, so the spill regions inside the library's array are in use
    big = _spilling()
    eng_big, got_big = _same(big, lds_slots=256, max_active=2048)
    assert got_big["max_p"].max() > 300 and got_big["evictions"].sum() > 0
    # second call: a smaller input of another engine (its tables replace the first one's in the array)
    small = configs.toy(n_replicas=3, n_steps=129)
    eng_small, got_small = _same(small)
    assert got_small["arrived"].sum() > 0
    # the first engine again, fewer slots: tables uploaded anew, contents left by the other call ignored
    eng_big.run(n_steps=1000)
    again = _outputs(eng_big)
    ref = fcs.Engine(big, lds_slots=256, max_active=2048)
    ref.run(n_steps=1000)
    want = _outputs(ref)
    for k in ("arrived", "completed", "evictions", "sum_u", "sum_p", "sum_q", "digest", "max_u"):
        assert np.array_equal(want[k], again[k]), k
    # and the same engine twice in a row without an upload in between
    eng_big.run(n_steps=1000)
    twice = _outputs(eng_big)
    for k in again:
        assert np.array_equal(again[k], twice[k]), k
    # the oracle agrees with what the static entry point produced
    ref0 = oracle.run_cell(small, 0)
    for name in oracle.counter_names():
        assert np.array_equal(ref0["counters"][name], got_small[name][: small.n_replicas]), name


def test_static_workspace_refuses_what_does_not_fit():
    wl = configs.config1(oracle.stability_bound).scaled(max_requests=0)   # about 600 MB of spill regions
    eng = fcs.Engine(wl, static_workspace=True)
    with pytest.raises(fcs.FcsError) as e:
        eng.run()
    assert e.value.code == fcs.binding.FCS_ENOMEM
    # with the active set bounded so that it stays in LDS the same engine fits
    eng2 = fcs.Engine(wl.scaled(n_replicas=64, n_steps=2000), static_workspace=True, max_active=1024)
    eng2.run()
    got, _ = eng2.stats()
    assert not np.any(got["error"]) and got["sum_p"].sum() > 0
