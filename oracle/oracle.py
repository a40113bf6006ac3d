"""ctypes access to the C oracle.  TEST INFRASTRUCTURE ONLY: nothing in the product path may
import this module; it exists so tests, the smoke check and the benchmark's cpu_baseline leg
can compute reference results on the CPU."""
from __future__ import annotations

import ctypes as C
import numpy as np

from . import build as _build

_lib = None


class SimParams(C.Structure):
    _fields_ = [("cap", C.c_int32), ("policy", C.c_int32), ("a_prefill", C.c_int64),
                ("b_decode", C.c_int64), ("c_prefill", C.c_int64), ("c_decode", C.c_int64),
                ("max_prefill_tokens", C.c_int64)]


TRACE_DTYPE = np.dtype([("kind", "<u4"), ("count", "<u4"), ("t_start", "<i8"), ("x", "<i8")])


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.oracle_brute_force_opt.restype = C.c_int64
        _lib.oracle_brute_force_opt_caps.restype = C.c_int64
        _lib.oracle_fnv1a64.restype = C.c_uint64
        _lib.oracle_fnv1a64.argtypes = [C.c_void_p, C.c_size_t, C.c_uint64]
        _lib.oracle_fnv1a64_init.restype = C.c_uint64
        _lib.oracle_prefill_time.restype = C.c_int64
        _lib.oracle_decode_time.restype = C.c_int64
        _lib.oracle_prefill_time.argtypes = [C.c_void_p, C.c_int64]
        _lib.oracle_decode_time.argtypes = [C.c_void_p, C.c_int64]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def local_search(cost, assign0, M, cap, max_passes, want_log=False, mode=-1):
    """mode: -1 = the library picks, 0 = threads over scenarios, 1 = threads inside one scenario's
    swap scan (same results; tests pin both)."""
    cost = np.ascontiguousarray(cost, dtype=np.int64)
    S, N = cost.shape
    assign = np.ascontiguousarray(assign0, dtype=np.int32).copy()
    load = np.zeros((S, M), np.int64)
    mk = np.zeros(S, np.int64)
    passes = np.zeros(S, np.int32)
    evals = np.zeros(S, np.uint64)
    status = np.zeros(S, np.int32)
    log = np.full((S, max(max_passes, 1)), np.iinfo(np.uint64).max, np.uint64) if want_log else None
    rc = lib().oracle_local_search_mode(_p(cost), S, N, M, cap, max_passes, _p(assign), _p(load), _p(mk),
                                        _p(passes), _p(evals), _p(log) if (want_log and max_passes > 0) else None,
                                        _p(status), int(mode))
    out = dict(rc=rc, assign=assign, load=load, makespan=mk, passes=passes, evals=evals, status=status)
    if want_log:
        out["log"] = log
    return out


def brute_force_opt(cost_row, M, cap) -> int:
    c = np.ascontiguousarray(cost_row, dtype=np.int64)
    return int(lib().oracle_brute_force_opt(_p(c), int(c.shape[0]), int(M), int(cap)))


def lower_bound(cost, M, prefill_tokens=None, ncap_L=0, tp_L=0):
    cost = np.ascontiguousarray(cost, dtype=np.int64)
    S, N = cost.shape
    lb = np.zeros(S, np.int64)
    status = np.zeros(S, np.int32)
    pt = None if prefill_tokens is None else np.ascontiguousarray(prefill_tokens, dtype=np.int32)
    rc = lib().oracle_lower_bound(_p(cost), S, N, M, _p(pt), C.c_int64(ncap_L), C.c_int64(tp_L),
                                  _p(lb), _p(status))
    return dict(rc=rc, lb=lb, status=status)


LB_RANK_LIMIT = 16384     # ranks the library's extended bound looks at (its documented limit, see include/mmbp.h)


def lower_bound_ex(cost, M, cap=None, kmax=0, prefill_tokens=None, ncap=None, tp=None, tp_form=0,
                   rank_limit=LB_RANK_LIMIT):
    cost = np.ascontiguousarray(cost, dtype=np.int64)
    S, N = cost.shape
    lb = np.zeros(S, np.int64)
    parts = np.zeros((S, 6), np.int64)
    status = np.zeros(S, np.int32)
    capa = None if cap is None else np.ascontiguousarray(cap, dtype=np.int32)
    pt = None if prefill_tokens is None else np.ascontiguousarray(prefill_tokens, dtype=np.int32)
    nc = None if ncap is None else np.ascontiguousarray(ncap, dtype=np.int64)
    tpa = None if tp is None else np.ascontiguousarray(tp, dtype=np.int64)
    nl = 0 if nc is None else int(nc.shape[0])
    rc = lib().oracle_lower_bound_ex(_p(cost), S, N, int(M), _p(capa), int(kmax), int(rank_limit), _p(pt), nl, _p(nc),
                                     _p(tpa), int(tp_form), _p(lb), _p(parts), _p(status))
    return dict(rc=rc, lb=lb, parts=parts, status=status)


def brute_force_opt_caps(cost_row, M, caps) -> int:
    c = np.ascontiguousarray(cost_row, dtype=np.int64)
    k = np.ascontiguousarray(caps, dtype=np.int32)
    return int(lib().oracle_brute_force_opt_caps(_p(c), int(c.shape[0]), int(M), _p(k)))


def lpt_start(cost, M, cap):
    cost = np.ascontiguousarray(cost, dtype=np.int64)
    S, N = cost.shape
    assign = np.zeros((S, N), np.int32)
    load = np.zeros((S, M), np.int64)
    order = np.zeros((S, N), np.int32)
    status = np.zeros(S, np.int32)
    rc = lib().oracle_lpt_start(_p(cost), S, N, int(M), int(cap), _p(assign), _p(load), _p(order), _p(status))
    return dict(rc=rc, assign=assign, load=load, order=order, status=status)


def make_params(cap, a_prefill, b_decode, c_prefill, c_decode, max_prefill_tokens=0, policy=0):
    return SimParams(cap, policy, a_prefill, b_decode, c_prefill, c_decode, max_prefill_tokens)


def online_iter_sim(arrival_us, in_len, out_len, params: dict, trace_scenarios=0, trace_capacity=0):
    arrival = np.ascontiguousarray(arrival_us, dtype=np.int64)
    in_len = np.ascontiguousarray(in_len, dtype=np.int32)
    out_len = np.ascontiguousarray(out_len, dtype=np.int32)
    S, N = arrival.shape
    p = make_params(**params)
    finish = np.zeros((S, N), np.int64)
    total = np.zeros(S, np.int64)
    busy = np.zeros(S, np.int64)
    npre = np.zeros(S, np.int32)
    ndec = np.zeros(S, np.int32)
    h = np.zeros(S, np.uint64)
    status = np.zeros(S, np.int32)
    tb = tl = None
    if trace_scenarios > 0 and trace_capacity > 0:
        tb = np.zeros((trace_scenarios, trace_capacity), TRACE_DTYPE)
        tl = np.zeros(trace_scenarios, np.int32)
    rc = lib().oracle_online_iter_sim(_p(arrival), _p(in_len), _p(out_len), S, N, C.byref(p), _p(finish),
                                      _p(total), _p(busy), _p(npre), _p(ndec), _p(h), _p(tb), _p(tl),
                                      int(trace_scenarios), int(trace_capacity), _p(status))
    return dict(rc=rc, finish_us=finish, total_us=total, busy_slot_us=busy, n_prefill_iter=npre,
                n_decode_iter=ndec, trace_hash=h, trace=tb, trace_len=tl, status=status)


def online_iter_sim_assigned(in_len, out_len, assign, params: dict, trace_scenarios=0, trace_capacity=0):
    in_len = np.ascontiguousarray(in_len, dtype=np.int32)
    out_len = np.ascontiguousarray(out_len, dtype=np.int32)
    assign = np.ascontiguousarray(assign, dtype=np.int32)
    S, N = in_len.shape
    p = make_params(**params)
    finish = np.zeros((S, N), np.int64)
    total = np.zeros(S, np.int64)
    busy = np.zeros(S, np.int64)
    npre = np.zeros(S, np.int32)
    ndec = np.zeros(S, np.int32)
    h = np.zeros(S, np.uint64)
    served = np.zeros((S, N), np.int32)
    start = np.zeros((S, N), np.int64)
    status = np.zeros(S, np.int32)
    tb = tl = None
    if trace_scenarios > 0 and trace_capacity > 0:
        tb = np.zeros((trace_scenarios, trace_capacity), TRACE_DTYPE)
        tl = np.zeros(trace_scenarios, np.int32)
    rc = lib().oracle_online_iter_sim_assigned(_p(in_len), _p(out_len), _p(assign), S, N, C.byref(p), _p(finish),
                                               _p(total), _p(busy), _p(npre), _p(ndec), _p(h), _p(served), _p(start), _p(tb),
                                               _p(tl), int(trace_scenarios), int(trace_capacity), _p(status))
    return dict(rc=rc, finish_us=finish, total_us=total, busy_slot_us=busy, n_prefill_iter=npre,
                n_decode_iter=ndec, trace_hash=h, served_by=served, start_us=start, trace=tb, trace_len=tl, status=status)


def fnv1a64(data: bytes) -> int:
    buf = (C.c_uint8 * len(data)).from_buffer_copy(data) if data else None
    return int(lib().oracle_fnv1a64(buf, len(data), lib().oracle_fnv1a64_init()))


def prefill_time(params: dict, tokens: int) -> int:
    p = make_params(**params)
    return int(lib().oracle_prefill_time(C.byref(p), tokens))


def decode_time(params: dict, seqs: int) -> int:
    p = make_params(**params)
    return int(lib().oracle_decode_time(C.byref(p), seqs))
