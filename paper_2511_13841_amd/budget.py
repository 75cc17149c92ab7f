"""Thin ctypes binding of include/das_budget.h (host-side budget solver and length-class policy, Sec. 4.2).
Argument marshalling only; the arithmetic is in csrc/das_budget.cpp."""
import ctypes as C

import numpy as np

from .binding import lib


class das_request(C.Structure):
    _fields_ = [("length", C.c_double), ("alpha", C.c_double), ("cap", C.c_double)]


class BudgetError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__(f"{what}: {'invalid argument' if code == -1 else 'forward-pass count below a request floor'} ({code})")


def _reqs(requests):
    arr = (das_request * len(requests))()
    for i, (l, a, k) in enumerate(requests):
        arr[i] = das_request(float(l), float(a), float(k))
    return arr


def _chk(code, what):
    if code != 0:
        raise BudgetError(code, what)


def _f64(x):
    return np.ascontiguousarray(x, dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def accepted(request, p):
    out = C.c_double()
    f = lib().das_budget_accepted
    f.argtypes = [C.POINTER(das_request), C.c_double, C.POINTER(C.c_double)]
    _chk(f(_reqs([request]), float(p), C.byref(out)), "das_budget_accepted")
    return out.value


def forward_passes(requests, p):
    out = C.c_double()
    p = _f64(p)
    f = lib().das_budget_forward_passes
    f.argtypes = [C.POINTER(das_request), C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
    _chk(f(_reqs(requests), len(requests), _ptr(p), C.byref(out)), "das_budget_forward_passes")
    return out.value


def latency(requests, p, c_base, c_tok, c_other=0.0):
    out = C.c_double()
    p = _f64(p)
    f = lib().das_budget_latency
    f.argtypes = [C.POINTER(das_request), C.c_int32, C.c_void_p, C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double)]
    _chk(f(_reqs(requests), len(requests), _ptr(p), c_base, c_tok, c_other, C.byref(out)), "das_budget_latency")
    return out.value


def _tight(name, requests, n_fwd):
    p = np.empty(len(requests), np.float64)
    f = getattr(lib(), name)
    f.argtypes = [C.POINTER(das_request), C.c_int32, C.c_double, C.c_void_p]
    _chk(f(_reqs(requests), len(requests), float(n_fwd), _ptr(p)), name)
    return p


def tight(requests, n_fwd):
    return _tight("das_budget_tight", requests, n_fwd)


def tight_printed(requests, n_fwd):
    return _tight("das_budget_tight_printed", requests, n_fwd)


def slope(requests, c_base, c_tok, n_fwd):
    out = C.c_double()
    f = lib().das_budget_slope
    f.argtypes = [C.POINTER(das_request), C.c_int32, C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double)]
    _chk(f(_reqs(requests), len(requests), c_base, c_tok, float(n_fwd), C.byref(out)), "das_budget_slope")
    return out.value


def solve(requests, c_base, c_tok):
    """(N_fwd*, p*[n]) minimising the rollout latency model."""
    n_fwd = C.c_double()
    p = np.empty(len(requests), np.float64)
    f = lib().das_budget_solve
    f.argtypes = [C.POINTER(das_request), C.c_int32, C.c_double, C.c_double, C.POINTER(C.c_double), C.c_void_p]
    _chk(f(_reqs(requests), len(requests), c_base, c_tok, C.byref(n_fwd), _ptr(p)), "das_budget_solve")
    return n_fwd.value, p


def draft_lens(p, n_fwd, k_max):
    p = _f64(p)
    k = np.empty(p.size, np.int32)
    f = lib().das_budget_draft_lens
    f.argtypes = [C.c_void_p, C.c_int32, C.c_double, C.c_int32, C.c_void_p]
    _chk(f(_ptr(p), p.size, float(n_fwd), int(k_max), _ptr(k)), "das_budget_draft_lens")
    return k


def length_class(length, t_medium, t_long):
    out = C.c_int32()
    f = lib().das_length_class
    f.argtypes = [C.c_double, C.c_double, C.c_double, C.POINTER(C.c_int32)]
    _chk(f(float(length), float(t_medium), float(t_long), C.byref(out)), "das_length_class")
    return out.value


def class_init(counts):
    out = C.c_int32()
    c = np.ascontiguousarray(counts, dtype=np.int64)
    f = lib().das_length_class_init
    f.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
    _chk(f(_ptr(c), C.byref(out)), "das_length_class_init")
    return out.value


def class_update(hist_final_len, hist_init, t_medium, t_long, partial_len, init_cls):
    out = C.c_int32()
    fl, ini = _f64(hist_final_len), np.ascontiguousarray(hist_init, dtype=np.int32)
    f = lib().das_length_class_update
    f.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_double, C.c_double, C.c_double, C.c_int32, C.POINTER(C.c_int32)]
    _chk(f(_ptr(fl), _ptr(ini), fl.size, float(t_medium), float(t_long), float(partial_len), int(init_cls), C.byref(out)),
         "das_length_class_update")
    return out.value
