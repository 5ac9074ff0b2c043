"""CPU oracle (test infrastructure, not part of the product).

Thin ctypes access to ``fcs_oracle.cpp`` plus the closed forms of the paper
written out in numpy.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; it imports nothing from the GPU
engine and the engine imports nothing from here.
"""
from __future__ import annotations

import ctypes as C
import os
import math
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fcs_oracle.cpp")
_LIB = os.path.join(_HERE, "libfcs_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


class _Law(C.Structure):
    _fields_ = [("lo", C.c_int32), ("n_thr", C.c_int32), ("thr", C.POINTER(C.c_uint32))]


class _Config(C.Structure):
    _fields_ = [
        ("policy", C.c_int32), ("n_classes", C.c_int32),
        ("capacity", C.c_int64), ("token_budget", C.c_int64), ("prefill_chunk", C.c_int64),
        ("b_floor", C.c_int32), ("b_frac_thr", C.c_uint32),
        ("arrivals", _Law),
        ("class_thr", C.POINTER(C.c_uint32)), ("prompt", C.POINTER(_Law)), ("decode", C.POINTER(_Law)),
        ("trace_every", C.c_int32), ("hist_bins", C.c_int32), ("hist_shift", C.c_int32),
        ("reserved", C.c_int32), ("max_requests", C.c_int64),
        ("n_forced", C.c_int64),
        ("forced_t", C.POINTER(C.c_int32)), ("forced_l", C.POINTER(C.c_int32)),
        ("forced_o", C.POINTER(C.c_int32)),
        ("n_forced_B", C.c_int64), ("forced_B", C.POINTER(C.c_int32)),
        ("class_arrivals", C.POINTER(_Law)), ("class_budget", C.POINTER(C.c_int32)),
        ("forced_cls", C.POINTER(C.c_int32)),
        ("protect_limit", C.c_int64),
        ("budget_mode", C.c_int32), ("reserved2", C.c_int32), ("budget_law", _Law), ("budget_b16", C.c_int64),
        ("assumed_o", C.c_int64),
        ("time_c0", C.c_int64), ("time_cp", C.c_int64), ("time_cd", C.c_int64),
    ]


_OUT_I32 = ["trace_q", "trace_u"]
_OUT_REQ = ["arrival_step", "completion_step", "first_activation", "last_activation", "req_l", "req_o"]
_OUT_STEP = ["step_u", "step_p", "step_q", "step_n", "step_b"]


class _Outputs(C.Structure):
    _fields_ = ([("counters", C.POINTER(C.c_uint64)), ("trace_q", C.POINTER(C.c_int32)),
                 ("trace_u", C.POINTER(C.c_int32)), ("hist", C.POINTER(C.c_uint32))]
                + [(n, C.POINTER(C.c_int32)) for n in _OUT_REQ]
                + [(n, C.POINTER(C.c_int32)) for n in _OUT_STEP])


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.fo_counter_name.restype = C.c_char_p
        _lib.fo_run.argtypes = [C.POINTER(_Config), C.c_int64, C.POINTER(C.c_int64), C.c_int64,
                                C.c_uint64, C.c_int32, C.POINTER(_Outputs)]
        _lib.fo_invert.argtypes = [C.POINTER(_Law), C.POINTER(C.c_uint32), C.c_int64, C.POINTER(C.c_int64)]
    return _lib


def protect_limit(alpha, capacity):
    """Section 4.1, alpha-protection greedy: admission may fill (1 - alpha) M, here rounded down."""
    return int(math.floor((1.0 - float(alpha)) * int(capacity)))


def counter_names():
    L = lib()
    return [L.fo_counter_name(i).decode() for i in range(L.fo_n_counters())]


def _p(arr, ctype):
    return arr.ctypes.data_as(C.POINTER(ctype))


def _law(law, keep):
    thr = np.ascontiguousarray(law.thr, dtype=np.uint32)
    keep.append(thr)
    return _Law(int(law.lo), int(thr.size), _p(thr, C.c_uint32))


def philox(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    o = np.zeros(4, np.uint32)
    lib().fo_philox(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(o, C.c_uint32))
    return o


def invert(law, u):
    keep = []
    L = _law(law, keep)
    u = np.ascontiguousarray(u, dtype=np.uint32)
    out = np.zeros(u.size, np.int64)
    rc = lib().fo_invert(C.byref(L), _p(u, C.c_uint32), u.size, _p(out, C.c_int64))
    if rc != 0:
        raise RuntimeError("oracle search routines disagree")
    return out


def run_cell(wl, cell_index, replica_ids=None, n_steps=None, seed=None, n_threads=1,
             per_step=False, per_request=None, forced=None, forced_B=None):
    """Simulate one cell of a workload for the listed replicas.

    Returns a dict: ``counters`` maps counter name -> uint64 array over the
    replicas; optional arrays ``trace_q``, ``trace_u``, ``hist``,
    ``arrival_step``, ``completion_step`` and (oracle-only) ``first_activation``,
    ``last_activation``, ``req_l``, ``req_o``, ``step_*``.
    ``forced`` = (t, l, o) arrays replaces the random arrival stream and
    ``forced_B`` the random activation budgets (hand-computed trajectories); for a
    CLASSES cell ``forced`` = (t, class) arrays.
    """
    cell = wl.cells[cell_index]
    T = int(wl.n_steps if n_steps is None else n_steps)
    if replica_ids is None:
        replica_ids = np.arange(wl.n_replicas)
    ids = np.ascontiguousarray(replica_ids, dtype=np.int64)
    n = int(ids.size)
    keep = []
    mix = wl.mixture
    nc = len(mix.classes)
    prompt = (_Law * nc)(*[_law(c.prompt, keep) for c in mix.classes])
    decode = (_Law * nc)(*[_law(c.decode, keep) for c in mix.classes])
    cthr = np.ascontiguousarray(mix.class_thr, dtype=np.uint32)
    max_req = int(wl.max_requests if per_request is None else per_request)
    cfg = _Config()
    cfg.policy = int(cell.policy)
    cfg.n_classes = nc
    cfg.capacity = int(wl.capacity)
    cfg.token_budget = int(wl.token_budget)
    cfg.prefill_chunk = int(wl.prefill_chunk)
    cfg.b_floor = int(cell.b_floor)
    cfg.b_frac_thr = int(cell.b_frac_thr)
    cfg.arrivals = _law(wl.arrival_laws[cell.arrival], keep)
    cfg.class_thr = _p(cthr, C.c_uint32)
    cfg.prompt = prompt
    cfg.decode = decode
    cfg.trace_every = int(wl.trace_every)
    cfg.hist_bins = int(wl.hist_bins)
    cfg.hist_shift = int(wl.hist_shift)
    cfg.max_requests = max_req
    cfg.n_forced = -1
    if cell.policy == 3:
        cfg.protect_limit = protect_limit(cell.alpha, wl.capacity)
    if cell.policy == 4:
        cfg.assumed_o = int(cell.assumed_o)
    cfg.time_c0, cfg.time_cp, cfg.time_cd = (int(v) for v in getattr(wl, "time_model", (0, 0, 0)))
    if cell.budget_law >= 0:
        cfg.budget_mode = 1
        cfg.budget_law = _law(wl.arrival_laws[cell.budget_law], keep)
    elif cell.credit_b16 > 0:
        cfg.budget_mode = 2
        cfg.budget_b16 = int(cell.credit_b16)
    if cell.policy == 2:
        ca = (_Law * nc)(*[_law(wl.arrival_laws[a], keep) for a in cell.class_arrival])
        cb = np.ascontiguousarray(cell.class_budget, dtype=np.int32)
        keep += [ca, cb]
        cfg.class_arrivals = ca
        cfg.class_budget = _p(cb, C.c_int32)
        if forced is not None:
            ft, fc = (np.ascontiguousarray(a, dtype=np.int32) for a in forced)
            if np.any(np.diff(ft) < 0):
                raise ValueError("forced arrivals must be sorted by slot")
            keep += [ft, fc]
            cfg.n_forced = int(ft.size)
            cfg.forced_t, cfg.forced_cls = _p(ft, C.c_int32), _p(fc, C.c_int32)
    elif forced is not None:
        ft, fl, fo = (np.ascontiguousarray(a, dtype=np.int32) for a in forced)
        if np.any(np.diff(ft) < 0):
            raise ValueError("forced arrivals must be sorted by slot")
        keep += [ft, fl, fo]
        cfg.n_forced = int(ft.size)
        cfg.forced_t, cfg.forced_l, cfg.forced_o = (_p(a, C.c_int32) for a in (ft, fl, fo))
    if forced_B is not None:
        fb = np.ascontiguousarray(forced_B, dtype=np.int32)
        keep.append(fb)
        cfg.n_forced_B = int(fb.size)
        cfg.forced_B = _p(fb, C.c_int32)

    L = lib()
    NC = L.fo_n_counters()
    res = {}
    out = _Outputs()
    counters = np.zeros((n, NC), np.uint64)
    out.counters = _p(counters, C.c_uint64)
    if wl.trace_every > 0:
        nt = T // wl.trace_every
        for name in _OUT_I32:
            res[name] = np.zeros((n, nt), np.int32)
            setattr(out, name, _p(res[name], C.c_int32))
    if wl.hist_bins > 0:
        res["hist"] = np.zeros((n, wl.hist_bins), np.uint32)
        out.hist = _p(res["hist"], C.c_uint32)
    if max_req > 0:
        for name in _OUT_REQ:
            res[name] = np.zeros((n, max_req), np.int32)
            setattr(out, name, _p(res[name], C.c_int32))
    if per_step:
        for name in _OUT_STEP:
            res[name] = np.zeros((n, T), np.int32)
            setattr(out, name, _p(res[name], C.c_int32))
    seed = int(wl.seed if seed is None else seed)
    rc = L.fo_run(C.byref(cfg), n, _p(ids, C.c_int64), T, seed, int(n_threads), C.byref(out))
    if rc != 0:
        raise RuntimeError(f"oracle rejected the configuration (rc={rc})")
    res["counters"] = {name: counters[:, i].copy() for i, name in enumerate(counter_names())}
    res["replica_ids"] = ids
    return res


# ---- closed forms -----------------------------------------------------------------

def workload(l, o):
    """Minimum KV-slot-tokens one request occupies: w = sum_{j=1..o} (l + j) (proof of Proposition 1)."""
    l = np.asarray(l, dtype=np.float64)
    o = np.asarray(o, dtype=np.float64)
    return l * o + 0.5 * (o + o * o)


def expected_workload(mix) -> float:
    """E_nu[l o + (o + o^2)/2] with l and o independent within a class (eq. 3)."""
    total = 0.0
    for pc, c in zip(mix.class_prob(), mix.classes):
        el = c.prompt.moment(1)
        eo = c.decode.moment(1)
        eo2 = c.decode.moment(2)
        total += pc * (el * eo + 0.5 * (eo + eo2))
    return float(total)


def stability_bound(mix, capacity) -> float:
    """Largest arrival rate not excluded by Proposition 2: lambda* = M / E[w]."""
    return float(capacity) / expected_workload(mix)


def percentile_from_hist(hist, num, den, shift=0):
    """Nearest-rank percentile on a latency histogram: bucket of the ceil(q n)-th smallest.

    Returns (value, saturated): value = bucket << shift; saturated if it is the last bucket.
    """
    hist = np.asarray(hist, dtype=np.int64)
    n = int(hist.sum())
    if n == 0:
        return 0, False
    k = (num * n + den - 1) // den
    k = max(k, 1)
    cum = np.cumsum(hist)
    b = int(np.searchsorted(cum, k, side="left"))
    return b << shift, b == hist.size - 1


# ---- the oracle under the host compiler's sanitizers ------------------------------------------------

def case_tokens(wl, cell_index, replica_ids, n_steps=None, forced=None, forced_B=None):
    """One case as the flat list of integers that replay_main.cpp reads (the fields of fo_config in order)."""
    cell = wl.cells[cell_index]
    mix = wl.mixture
    nc = len(mix.classes)

    def law(L):
        thr = [int(v) for v in np.asarray(L.thr, dtype=np.uint32)]
        return [int(L.lo), len(thr)] + thr

    t = [int(cell.policy), nc, int(wl.capacity), int(wl.token_budget), int(wl.prefill_chunk), int(cell.b_floor),
         int(cell.b_frac_thr)]
    t += law(wl.arrival_laws[cell.arrival])
    t += [int(v) for v in np.asarray(mix.class_thr, dtype=np.uint32)][: max(nc - 1, 0)]
    for c in mix.classes:
        t += law(c.prompt)
    for c in mix.classes:
        t += law(c.decode)
    t += [int(wl.trace_every), int(wl.hist_bins), int(wl.hist_shift), int(wl.max_requests)]
    if forced is None:
        t += [-1]
    else:
        cols = [list(map(int, a)) for a in forced]
        n = len(cols[0])
        if cell.policy == 2:  # (slot, class)
            cols = [cols[0], [0] * n, [0] * n, cols[1]]
        else:                 # (slot, l, o)
            cols = cols + [[0] * n]
        t += [n] + cols[0] + cols[1] + cols[2] + cols[3]
    fb = [] if forced_B is None else [int(v) for v in forced_B]
    t += [len(fb)] + fb
    if cell.policy == 2:
        t += [1]
        for a in cell.class_arrival:
            t += law(wl.arrival_laws[a])
        t += [int(b) for b in cell.class_budget]
    else:
        t += [0]
    t += [protect_limit(cell.alpha, wl.capacity) if cell.policy == 3 else 0]
    if cell.budget_law >= 0:
        t += [1] + law(wl.arrival_laws[cell.budget_law]) + [0]
    elif cell.credit_b16 > 0:
        t += [2, 0, 0, int(cell.credit_b16)]
    else:
        t += [0, 0, 0, 0]
    t += [int(cell.assumed_o) if cell.policy == 4 else 0]
    t += [int(v) for v in getattr(wl, "time_model", (0, 0, 0))]
    ids = [int(v) for v in replica_ids]
    t += [len(ids)] + ids + [int(wl.n_steps if n_steps is None else n_steps), int(wl.seed)]
    return t


def build_sanitized(out_dir) -> str:
    """replay_main.cpp with the address and undefined-behaviour sanitizers of the host compiler."""
    exe = os.path.join(out_dir, "fcs_oracle_replay_asan")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-pthread", "-o", exe, os.path.join(_HERE, "replay_main.cpp")]
    subprocess.run(cmd, check=True)
    return exe


def replay(exe, tokens):
    """Runs the driver on one case; returns a list of (counters dict, completion slots, histogram) per replica."""
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], input=" ".join(map(str, tokens)), capture_output=True, text=True, env=env)
    if r.returncode != 0:
        raise RuntimeError(f"sanitized oracle failed (rc={r.returncode}):\n{r.stderr[-4000:]}")
    names = counter_names()
    rows, cur = [], None
    for ln in r.stdout.splitlines():
        kind, *vals = ln.split()
        if kind == "counters":
            cur = [dict(zip(names, map(int, vals))), None, None]
            rows.append(cur)
        elif kind == "completion":
            cur[1] = np.array(list(map(int, vals)), dtype=np.int32)
        elif kind == "hist":
            cur[2] = np.array(list(map(int, vals)), dtype=np.uint32)
    return rows
