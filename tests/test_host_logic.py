"""Host-side checks that need no GPU: the library loads, exports its ABI, validates parameters."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2604_11001_amd as fcs
from paper_2604_11001_amd import binding
from workloads import configs, laws

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "fcs.h")) as f:
        text = f.read()
    declared = set(re.findall(r"\b(fcs_[a-z_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    L = fcs.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_counter_names_cover_the_oracle():
    names = fcs.counter_names()
    assert len(names) == fcs.lib().fcs_n_counters() and len(set(names)) == len(names)
    assert set(oracle.counter_names()) <= set(names)


def test_stability_bound_matches_the_oracle_closed_form():
    for i in range(5):
        wl = configs.make(i, oracle.stability_bound)
        a = oracle.stability_bound(wl.mixture, wl.capacity)
        b = fcs.stability_bound(wl.mixture, wl.capacity)
        assert abs(a - b) <= 1e-12 * a
    assert abs(fcs.stability_bound(configs.three_class(1.0).mixture, 16492) - 3 * 16492 / 4060.0) < 1e-7   # class weights are quantised to 2^-32


def _create(wl, **kw):
    p, keep = binding.make_params(wl, **kw)
    h = C.c_void_p()
    rc = fcs.lib().fcs_create(C.byref(p), C.byref(h))
    if rc == 0:
        fcs.lib().fcs_destroy(h)
    return rc


def test_protect_limit_against_the_oracle_and_exact_arithmetic():
    # floor((1 - alpha) M): the library's C double arithmetic, the oracle's, and exact rationals on decimal alphas
    from fractions import Fraction
    rng = np.random.default_rng(11)
    for M in (20, 1500, 4000, 16492, 262144, 1 << 30):
        for a in list(rng.random(200)) + [0.0, 1.0, 0.05, 0.1, 0.15, 0.25, 0.3, 0.999, 0.5]:
            assert binding.protect_limit(a, M) == oracle.protect_limit(a, M), (a, M)
    for M in (20, 16492, 100000):
        for k in range(0, 101):
            exact = (1 - Fraction(k, 100)) * M
            got = binding.protect_limit(k / 100.0, M)
            # a decimal alpha is not a binary fraction: where (1 - alpha) M is a whole number the double
            # product may land just below it
            assert got == exact.numerator // exact.denominator or (exact.denominator == 1 and got == exact - 1), (k, M)
    out = C.c_int32(0)
    for a, M in ((-0.1, 10), (1.1, 10), (float("nan"), 10), (0.5, 0), (0.5, (1 << 30) + 1)):
        assert fcs.lib().fcs_protect_limit(a, M, C.byref(out)) == -1
    assert fcs.lib().fcs_protect_limit(0.5, 10, None) == -1


def test_create_validates_parameters():
    ok = configs.toy()
    assert _create(ok) == 0
    assert _create(ok.scaled(capacity=0)) == -1
    assert _create(ok.scaled(token_budget=0)) == -1
    assert _create(ok.scaled(prefill_chunk=0)) == -1
    assert _create(ok.scaled(capacity=100)) == -1            # max l + max o = 140 > M
    assert _create(ok, lds_slots=100) == -1
    # LDS slots per path: 256 to 512 in steps of 64, then in steps of 256; the kernels of the other policies
    # and of slots of variable duration take steps of 256 only
    for slots, rc in ((256, 0), (320, 0), (448, 0), (512, 0), (576, -1), (768, 0), (4096, 0), (4352, -1), (192, -1)):
        assert _create(ok, lds_slots=slots) == rc, slots
    assert _create(configs.alpha_sweep(n_replicas=2, n_steps=10), lds_slots=320) == -1
    assert _create(configs.alpha_sweep(n_replicas=2, n_steps=10), lds_slots=512) == 0
    assert _create(ok.scaled(time_model=(2, 1, 1)), lds_slots=384) == -1
    bad = laws.Law.__new__(laws.Law)
    object.__setattr__(bad, "lo", 1)
    object.__setattr__(bad, "thr", np.array([5, 3], np.uint32))
    object.__setattr__(bad, "name", "decreasing")
    assert _create(ok.scaled(mixture=laws.single(bad, laws.point(3)))) == -1
    assert _create(ok.scaled(mixture=laws.single(laws.point(0), laws.point(3)))) == -1   # l >= 1
    assert _create(ok.scaled(cells=(configs.Cell(7, 0, 0, 0),))) == -1
    assert _create(ok.scaled(cells=(configs.Cell(0, 3, 0, 0),))) == -1
    assert _create(ok.scaled(arrival_laws=(laws.uniform_int(0, 100),))) == -1            # > 63 thresholds


def test_create_validates_the_other_policies():
    import dataclasses
    kc = configs.known_classes(n_replicas=2, n_steps=10)
    assert _create(kc) == 0
    cell = kc.cells[0]
    with_cell = lambda **kw: kc.scaled(cells=(dataclasses.replace(cell, **kw),))
    assert _create(with_cell(class_budget=(40, 20, 5))) == -1            # budgets sum to more than 64
    assert _create(with_cell(class_budget=(4, -1, 4))) == -1
    assert _create(with_cell(class_arrival=(0, 0, 9))) == -1             # no such arrival law
    mixed = laws.Mixture((laws.RequestClass(1.0, laws.uniform_int(4, 9), laws.point(5)),) + kc.mixture.classes[1:])
    assert _create(kc.scaled(mixture=mixed)) == -1                       # Algorithm 1 needs known lengths
    # alpha-protection: the limit lies in [0, M]
    al = configs.alpha_sweep(n_replicas=2, n_steps=10)
    assert _create(al) == 0
    p, keep = fcs.binding.make_params(al)
    h = C.c_void_p()
    for bad in (-0.01, 1.5, float("nan")):
        p.cells[0].alpha = bad
        assert fcs.lib().fcs_create(C.byref(p), C.byref(h)) == -1
    # MC benchmark: the slot model without chunking or token budget, an assumed length that covers every output
    ut = configs.unknown_types(n_replicas=2, n_steps=10)
    assert _create(ut) == 0
    assert _create(ut.scaled(prefill_chunk=8)) == -1
    assert _create(ut.scaled(token_budget=4096)) == -1
    assert _create(ut.scaled(cells=(configs.mc_cell(0, 59),))) == -1     # a class produces 60 tokens
    assert _create(ut.scaled(cells=(configs.mc_cell(0, 60),), capacity=69)) == -1
    assert _create(ut.scaled(cells=(configs.mc_known_cell(0),))) == 0        # known request types
    long_out = laws.single(laws.point(10), laws.uniform_int(1, 1025))
    assert _create(ut.scaled(cells=(configs.mc_known_cell(0),), mixture=long_out)) == -1   # outputs beyond the wheel
    # slots of variable duration: c0 >= 1, not with Algorithm 1 cells
    toy = configs.toy()
    assert _create(toy.scaled(time_model=(2, 1, 1))) == 0
    assert _create(toy.scaled(time_model=(0, 1, 1))) == -1
    assert _create(toy.scaled(time_model=(1, -1, 0))) == -1
    assert _create(kc.scaled(time_model=(1, 0, 0))) == -1
    # forms of B_t: only for FLOW cells, the law must exist, b in (0, 30000]
    toy = configs.toy()
    ok = toy.scaled(cells=(configs.flow_law_cell(0, 0), configs.flow_credit_cell(0, 1.5)))
    assert _create(ok) == 0
    assert _create(toy.scaled(cells=(configs.flow_law_cell(0, 5),))) == -1
    assert _create(toy.scaled(cells=(dataclasses.replace(configs.greedy_cell(0), credit_b16=65536),))) == -1
    assert _create(toy.scaled(cells=(dataclasses.replace(configs.flow_cell(0, 1.0), credit_b16=(30001 << 16)),))) == -1


def test_calls_out_of_order_and_null_arguments():
    L = fcs.lib()
    p, keep = binding.make_params(configs.toy())
    h = C.c_void_p()
    assert L.fcs_create(C.byref(p), C.byref(h)) == 0
    n = C.c_size_t(0)
    assert L.fcs_workspace_bytes(h, 16, C.byref(n)) == 0 and n.value > 0
    assert L.fcs_workspace_bytes(h, 0, C.byref(n)) == -1
    assert L.fcs_run(h, 16, 100, 1, None) == -3            # not bound
    assert L.fcs_stats(h, -1, None, None) == -3            # nothing ran
    assert L.fcs_create(None, C.byref(h)) == -1
    assert L.fcs_strerror(-4).decode().startswith("a path outgrew")
    L.fcs_destroy(h)
    # a mixture of several classes without its class thresholds
    p3, keep3 = binding.make_params(configs.three_class(1.0))
    out = C.c_double(0.0)
    assert L.fcs_stability_bound(C.byref(p3), C.byref(out)) == 0
    p3.class_thr = None
    assert L.fcs_stability_bound(C.byref(p3), C.byref(out)) == -1
    assert L.fcs_create(C.byref(p3), C.byref(h)) == -1
    assert L.fcs_stability_bound(C.byref(p3), None) == -1


def test_engine_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(RuntimeError):
        fcs.Engine(configs.toy())
