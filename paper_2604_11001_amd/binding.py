"""ctypes binding of libfcs (argument marshalling only).

Function names mirror the C ABI of ``include/fcs.h``.  PyTorch is used for
device buffers and the stream handle, nothing else; every step of a sample
path runs inside the HIP kernel.  There is no CPU fallback: importing works
without a GPU (so the exported symbols can be checked), but creating an
:class:`Engine` without one raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfcs.so")

FCS_OK, FCS_EINVAL, FCS_ENOMEM, FCS_ESTATE, FCS_EOVERFLOW, FCS_EDEVICE = 0, -1, -2, -3, -4, -5
POLICY_FLOW, POLICY_GREEDY = 0, 1
FLAG_SKIP_IDLE, FLAG_GENERAL_CODE = 1, 2
# counters that describe the run on the device, not the sample path: they differ from launch to launch
PROFILING_COUNTERS = ("clock_start", "clock_end")


class FcsError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


class fcs_law(C.Structure):
    _fields_ = [("lo", C.c_int32), ("n_thr", C.c_int32), ("thr", C.POINTER(C.c_uint32))]


class fcs_cell(C.Structure):
    _fields_ = [("policy", C.c_int32), ("arrival", C.c_int32), ("b_floor", C.c_int32),
                ("b_frac_thr", C.c_uint32),
                ("class_arrival", C.POINTER(C.c_int32)), ("class_budget", C.POINTER(C.c_int32)),
                ("alpha", C.c_double), ("budget_mode", C.c_int32), ("budget_law", C.c_int32),
                ("budget_b16", C.c_uint32), ("assumed_o", C.c_int32)]


class fcs_params(C.Structure):
    _fields_ = [
        ("capacity", C.c_int32), ("token_budget", C.c_int32), ("prefill_chunk", C.c_int32),
        ("n_classes", C.c_int32), ("class_thr", C.POINTER(C.c_uint32)),
        ("prompt", C.POINTER(fcs_law)), ("decode", C.POINTER(fcs_law)),
        ("n_arrival_laws", C.c_int32), ("arrival", C.POINTER(fcs_law)),
        ("n_cells", C.c_int32), ("cells", C.POINTER(fcs_cell)),
        ("trace_every", C.c_int32), ("hist_bins", C.c_int32), ("hist_shift", C.c_int32),
        ("max_requests", C.c_int32), ("max_active", C.c_int32), ("lds_slots", C.c_int32),
        ("time_c0", C.c_int32), ("time_cp", C.c_int32), ("time_cd", C.c_int32),
        ("flags", C.c_int32),
    ]


class fcs_outputs(C.Structure):
    _fields_ = [("counters", C.c_void_p), ("trace_q", C.c_void_p), ("trace_u", C.c_void_p),
                ("hist", C.c_void_p), ("arrival_step", C.c_void_p), ("completion_step", C.c_void_p),
                ("trace_entries", C.c_int64)]


class fcs_summary(C.Structure):
    _fields_ = [
        ("n_paths", C.c_int64), ("n_steps", C.c_int64), ("request_steps", C.c_uint64),
        ("arrived", C.c_uint64), ("completed", C.c_uint64), ("evictions", C.c_uint64),
        ("overflow_steps", C.c_uint64), ("mean_latency", C.c_double), ("kv_utilisation", C.c_double),
        ("token_throughput", C.c_double), ("prompt_throughput", C.c_double), ("mean_queue", C.c_double),
        ("mean_active", C.c_double), ("first_error_path", C.c_int64), ("error_code", C.c_int32),
        ("reserved", C.c_int32),
    ]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_ if n != "reserved"}


EXPORTS = ["fcs_create", "fcs_workspace_bytes", "fcs_bind", "fcs_run", "fcs_run_from", "fcs_run_static", "fcs_stats",
           "fcs_percentile", "fcs_stability_bound", "fcs_protect_limit", "fcs_geometry", "fcs_destroy", "fcs_strerror",
           "fcs_n_counters", "fcs_counter_name"]

_lib = None


def lib():
    """Loads the built library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2604_11001_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.fcs_create.argtypes = [C.POINTER(fcs_params), C.POINTER(C.c_void_p)]
        L.fcs_workspace_bytes.argtypes = [C.c_void_p, C.c_int64, C.POINTER(C.c_size_t)]
        L.fcs_bind.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int64, C.POINTER(fcs_outputs), C.c_void_p]
        L.fcs_run.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_uint64, C.c_void_p]
        L.fcs_run_from.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_uint64, C.c_void_p]
        L.fcs_run_static.argtypes = [C.c_void_p, C.POINTER(fcs_outputs), C.c_int64, C.c_int64, C.c_uint64, C.c_void_p]
        L.fcs_stats.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(fcs_summary)]
        L.fcs_percentile.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
        L.fcs_stability_bound.argtypes = [C.POINTER(fcs_params), C.POINTER(C.c_double)]
        L.fcs_protect_limit.argtypes = [C.c_double, C.c_int32, C.POINTER(C.c_int32)]
        L.fcs_geometry.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.fcs_destroy.argtypes = [C.c_void_p]
        L.fcs_destroy.restype = None
        L.fcs_strerror.argtypes = [C.c_int]
        L.fcs_strerror.restype = C.c_char_p
        L.fcs_counter_name.argtypes = [C.c_int]
        L.fcs_counter_name.restype = C.c_char_p
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().fcs_strerror(int(code)).decode()


def counter_names():
    L = lib()
    return [L.fcs_counter_name(i).decode() for i in range(L.fcs_n_counters())]


def _check(rc, what):
    if rc != FCS_OK:
        raise FcsError(rc, what)


def _law(law, keep):
    thr = np.ascontiguousarray(law.thr, dtype=np.uint32)
    keep.append(thr)
    return fcs_law(int(law.lo), int(thr.size), thr.ctypes.data_as(C.POINTER(C.c_uint32)))


def make_params(wl, max_active: int = 0, lds_slots: int = 0, flags: int = 0):
    """Marshals a workload description into fcs_params; returns (params, keep-alive list)."""
    keep = []
    mix = wl.mixture
    nc = len(mix.classes)
    prompt = (fcs_law * nc)(*[_law(c.prompt, keep) for c in mix.classes])
    decode = (fcs_law * nc)(*[_law(c.decode, keep) for c in mix.classes])
    na = len(wl.arrival_laws)
    arrival = (fcs_law * na)(*[_law(a, keep) for a in wl.arrival_laws])
    cthr = np.ascontiguousarray(mix.class_thr, dtype=np.uint32)
    ncell = len(wl.cells)
    cells = (fcs_cell * ncell)()
    for i, c in enumerate(wl.cells):
        cells[i].policy, cells[i].arrival = int(c.policy), int(c.arrival)
        cells[i].b_floor, cells[i].b_frac_thr = int(c.b_floor), int(c.b_frac_thr)
        if getattr(c, "budget_law", -1) >= 0:      # B_t drawn from one of the count laws
            cells[i].budget_mode, cells[i].budget_law = 1, int(c.budget_law)
        elif getattr(c, "credit_b16", 0) > 0:      # B_t of a credit accumulator
            cells[i].budget_mode, cells[i].budget_b16 = 2, int(c.credit_b16)
        if int(c.policy) == 4:  # memory-check benchmark
            cells[i].assumed_o = int(c.assumed_o)
        if int(c.policy) == 3:  # alpha-protection greedy: the protected share of the memory
            cells[i].alpha = float(c.alpha)
        if getattr(c, "class_arrival", ()):  # per-class arrival laws and budgets (Algorithm 1)
            ca = np.ascontiguousarray(c.class_arrival, dtype=np.int32)
            cb = np.ascontiguousarray(c.class_budget, dtype=np.int32)
            keep += [ca, cb]
            cells[i].class_arrival = ca.ctypes.data_as(C.POINTER(C.c_int32))
            cells[i].class_budget = cb.ctypes.data_as(C.POINTER(C.c_int32))
    keep += [prompt, decode, arrival, cthr, cells]
    p = fcs_params()
    p.capacity, p.token_budget, p.prefill_chunk = int(wl.capacity), int(wl.token_budget), int(wl.prefill_chunk)
    p.n_classes = nc
    p.class_thr = cthr.ctypes.data_as(C.POINTER(C.c_uint32))
    p.prompt, p.decode = prompt, decode
    p.n_arrival_laws, p.arrival = na, arrival
    p.n_cells, p.cells = ncell, cells
    p.trace_every, p.hist_bins, p.hist_shift = int(wl.trace_every), int(wl.hist_bins), int(wl.hist_shift)
    p.max_requests, p.max_active, p.lds_slots = int(wl.max_requests), int(max_active), int(lds_slots)
    p.time_c0, p.time_cp, p.time_cd = (int(v) for v in getattr(wl, "time_model", (0, 0, 0)))
    p.flags = int(flags)
    return p, keep


def protect_limit(alpha, capacity) -> int:
    """fcs_protect_limit (host only, no GPU needed)."""
    out = C.c_int32(0)
    _check(lib().fcs_protect_limit(float(alpha), int(capacity), C.byref(out)), "fcs_protect_limit")
    return int(out.value)


def stability_bound(mixture, capacity) -> float:
    """fcs_stability_bound for a mixture (host only, no GPU needed)."""
    import types
    wl = types.SimpleNamespace(mixture=mixture, capacity=capacity, token_budget=1, prefill_chunk=1,
                               arrival_laws=(), cells=(), trace_every=0, hist_bins=0, hist_shift=0,
                               max_requests=0)
    p, keep = make_params(wl)
    out = C.c_double(0.0)
    _check(lib().fcs_stability_bound(C.byref(p), C.byref(out)), "fcs_stability_bound")
    return float(out.value)


class Engine:
    """Owns one fcs handle plus the torch device buffers bound to it."""

    def __init__(self, wl, n_replicas=None, n_steps=None, device="cuda:0", max_active=0, lds_slots=0,
                 static_workspace=False, skip_idle=False, general_code=False):
        """static_workspace: no workspace is allocated or bound; ``run`` goes through fcs_run_static, on
        the device memory that the library itself holds."""
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("libfcs needs a HIP device; there is no CPU fallback")
        self.torch = torch
        self.device = torch.device(device)
        self.wl = wl
        self.n_replicas = int(wl.n_replicas if n_replicas is None else n_replicas)
        self.n_steps = int(wl.n_steps if n_steps is None else n_steps)
        self.n_cells = len(wl.cells)
        self.n_paths = self.n_cells * self.n_replicas
        self.bound_replicas = self.n_replicas
        self._h = C.c_void_p()
        params, keep = make_params(wl, max_active, lds_slots,
                                   (FLAG_SKIP_IDLE if skip_idle else 0) | (FLAG_GENERAL_CODE if general_code else 0))
        _check(lib().fcs_create(C.byref(params), C.byref(self._h)), "fcs_create")
        del keep
        nbytes = C.c_size_t(0)
        _check(lib().fcs_workspace_bytes(self._h, self.n_replicas, C.byref(nbytes)), "fcs_workspace_bytes")
        dev = self.device
        self.static_workspace = bool(static_workspace)
        with torch.cuda.device(dev):
            self.workspace = None if static_workspace else torch.empty(nbytes.value, dtype=torch.uint8, device=dev)
            nc = lib().fcs_n_counters()
            self.counters = torch.zeros((self.n_paths, nc), dtype=torch.int64, device=dev)
            self.out = fcs_outputs()
            self.out.counters = self.counters.data_ptr()
            self.trace_q = self.trace_u = self.hist = self.arrival_step = self.completion_step = None
            if wl.trace_every > 0:
                nt = self.n_steps // wl.trace_every
                self.trace_q = torch.zeros((self.n_paths, nt), dtype=torch.int32, device=dev)
                self.trace_u = torch.zeros((self.n_paths, nt), dtype=torch.int32, device=dev)
                self.out.trace_q, self.out.trace_u = self.trace_q.data_ptr(), self.trace_u.data_ptr()
                self.out.trace_entries = self.trace_q.numel()
            if wl.hist_bins > 0:
                self.hist = torch.zeros((self.n_paths, wl.hist_bins), dtype=torch.int32, device=dev)
                self.out.hist = self.hist.data_ptr()
            if wl.max_requests > 0:
                self.arrival_step = torch.zeros((self.n_paths, wl.max_requests), dtype=torch.int32, device=dev)
                self.completion_step = torch.zeros_like(self.arrival_step)
                self.out.arrival_step = self.arrival_step.data_ptr()
                self.out.completion_step = self.completion_step.data_ptr()
            if not static_workspace:
                stream = torch.cuda.current_stream(dev).cuda_stream
                _check(lib().fcs_bind(self._h, self.workspace.data_ptr(), nbytes.value, self.n_replicas,
                                      C.byref(self.out), C.c_void_p(stream)), "fcs_bind")

    def geometry(self):
        a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
        _check(lib().fcs_geometry(self._h, C.byref(a), C.byref(b), C.byref(c)), "fcs_geometry")
        return {"lds_slots": a.value, "lds_bytes": b.value, "spill_slots": c.value}

    def run(self, seed=None, n_steps=None, replica_base=0, stream=None, n_replicas=None):
        """fcs_run_from on the current torch stream (asynchronous).  n_replicas: fewer replicas per cell than
        the engine was created for; the rows of every output array are then packed by that number."""
        torch = self.torch
        if n_replicas is not None:
            if not 1 <= int(n_replicas) <= self.bound_replicas:
                raise ValueError("n_replicas beyond what the engine was created for")
            self.n_replicas = int(n_replicas)
            self.n_paths = self.n_cells * self.n_replicas
        if stream is None:
            stream = torch.cuda.current_stream(self.device).cuda_stream
        seed = int(self.wl.seed if seed is None else seed)
        T = int(self.n_steps if n_steps is None else n_steps)
        if self.static_workspace:
            with torch.cuda.device(self.device):
                _check(lib().fcs_run_static(self._h, C.byref(self.out), self.n_replicas, T, seed, C.c_void_p(stream)),
                       "fcs_run_static")
            return
        _check(lib().fcs_run_from(self._h, int(replica_base), self.n_replicas, T, seed, C.c_void_p(stream)),
               "fcs_run_from")

    def stats(self, cell=-1, allow_overflow=False, profiling=False):
        """fcs_stats: returns (counters dict name -> uint64 array over paths, summary dict).  The counters that
        describe the run on the device rather than the sample path (PROFILING_COUNTERS) come with profiling=True."""
        L = lib()
        nc = L.fcs_n_counters()
        host = np.zeros((self.n_paths, nc), np.uint64)
        s = fcs_summary()
        rc = L.fcs_stats(self._h, int(cell), host.ctypes.data_as(C.c_void_p), C.byref(s))
        if rc != FCS_OK and not (allow_overflow and rc == FCS_EOVERFLOW):
            raise FcsError(rc, "fcs_stats")
        names = counter_names()
        return ({n: host[:, i].copy() for i, n in enumerate(names) if profiling or n not in PROFILING_COUNTERS},
                s.as_dict())

    def percentile(self, num, den):
        val = np.zeros(self.n_paths, np.int32)
        sat = np.zeros(self.n_paths, np.uint8)
        _check(lib().fcs_percentile(self._h, int(num), int(den), val.ctypes.data_as(C.c_void_p),
                                    sat.ctypes.data_as(C.c_void_p)), "fcs_percentile")
        return val, sat.astype(bool)

    def close(self):
        if self._h:
            lib().fcs_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
