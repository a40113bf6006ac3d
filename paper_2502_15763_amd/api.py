"""Thin Python binding over libmmbp's C ABI (argument marshalling only).

Same names as the C entry points.  Tensors must be contiguous torch tensors on a CUDA/HIP
device; PyTorch is used for device memory and the current stream only.  Every computation
runs inside the library's HIP kernels; there is no CPU fallback: if the library is missing or
no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmmbp.so")

I32, I64 = 0, 1
POLICY_RULE, POLICY_PREFILL_FIRST, POLICY_PREFILL_FIRST_SINGLE = 0, 1, 2
ST_OK, ST_TRUNCATED, ST_BAD_ASSIGN, ST_BAD_COST, ST_BAD_SIM_INPUT = 0, 1, 2, 3, 4
EINVAL, EINFEASIBLE, EUNSUPPORTED, EWORKSPACE, EHIP = -1, -2, -3, -4, -5

GRID_MAX_PASSES = 4096
STATIC_SCRATCH_BYTES = 16 << 20

EXPORTS = ("mmbp_version", "mmbp_strerror", "mmbp_workspace_bytes", "mmbp_valu_probe", "mmbp_lower_bound", "mmbp_lower_bound_ex", "mmbp_lpt_start",
           "mmbp_local_search", "mmbp_local_search_pruned", "mmbp_local_search_static", "online_iter_sim",
           "online_iter_sim_assigned")


class SimParams(C.Structure):
    _fields_ = [("cap", C.c_int32), ("policy", C.c_int32), ("a_prefill", C.c_int64),
                ("b_decode", C.c_int64), ("c_prefill", C.c_int64), ("c_decode", C.c_int64),
                ("max_prefill_tokens", C.c_int64)]


class MmbpError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"libmmbp error {code}: {text}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Load libmmbp.so (built in-tree by paper_2502_15763_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2502_15763_amd.build`")
    # PyTorch brings its own copy of the HIP runtime; the library must bind to that copy (one runtime
    # per process: a second one sees no device), so torch is loaded before the library, always.
    _torch()
    lib = C.CDLL(LIB_PATH)
    vp, i, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
    lib.mmbp_version.restype = i
    lib.mmbp_strerror.restype = C.c_char_p
    lib.mmbp_strerror.argtypes = [i]
    lib.mmbp_workspace_bytes.restype = sz
    lib.mmbp_workspace_bytes.argtypes = [i, i, i]
    lib.mmbp_valu_probe.restype = i
    lib.mmbp_valu_probe.argtypes = [vp, i, i, C.POINTER(C.c_uint64), vp]
    lib.mmbp_lower_bound.restype = i
    lib.mmbp_lower_bound.argtypes = [vp, i, i, i, i, vp, i64, i64, vp, vp, vp]
    lib.mmbp_lower_bound_ex.restype = i
    lib.mmbp_lower_bound_ex.argtypes = [vp, i, i, i, i, C.POINTER(C.c_int32), i, vp, i, C.POINTER(i64), C.POINTER(i64), i,
                                        vp, vp, vp, vp]
    lib.mmbp_lpt_start.restype = i
    lib.mmbp_lpt_start.argtypes = [vp, i, i, i, i, i, vp, vp, vp, vp, vp]
    lib.mmbp_local_search.restype = i
    lib.mmbp_local_search.argtypes = [vp, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.mmbp_local_search_pruned.restype = i
    lib.mmbp_local_search_pruned.argtypes = lib.mmbp_local_search.argtypes
    lib.mmbp_local_search_static.restype = i
    lib.mmbp_local_search_static.argtypes = [vp, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.online_iter_sim.restype = i
    lib.online_iter_sim.argtypes = [vp, vp, vp, i, i, C.POINTER(SimParams), vp, vp, vp, vp, vp, vp, vp, vp, i, i,
                                    vp, vp]
    lib.online_iter_sim_assigned.restype = i
    lib.online_iter_sim_assigned.argtypes = [vp, vp, vp, i, i, C.POINTER(SimParams), vp, vp, vp, vp, vp, vp, vp, vp,
                                             vp, vp, i, i, vp, vp]
    _lib = lib
    return lib


def _torch():
    import torch
    return torch


def _ptr(t, dtype=None, shape=None, name="tensor"):
    if t is None:
        return None
    torch = _torch()
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    torch = _torch()
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(rc, raise_on_error):
    if rc != 0 and raise_on_error:
        raise MmbpError(rc, mmbp_strerror(rc))
    return rc


def mmbp_version() -> int:
    return int(load_library().mmbp_version())


def mmbp_strerror(code: int) -> str:
    return load_library().mmbp_strerror(int(code)).decode()


def mmbp_workspace_bytes(S: int, N: int, M: int) -> int:
    return int(load_library().mmbp_workspace_bytes(int(S), int(N), int(M)))


def mmbp_valu_probe(out, blocks, trips, stream=None, raise_on_error=True) -> int:
    """Enqueues the vector-ALU calibration loop; returns the 32-bit lane operations it issues."""
    torch = _torch()
    ops = C.c_uint64(0)
    rc = load_library().mmbp_valu_probe(_ptr(out, torch.int32, (int(blocks) * 256,), "out"), int(blocks), int(trips),
                                        C.byref(ops), _stream(stream))
    _check(rc, raise_on_error)
    return int(ops.value)


def _cost_dtype(cost):
    torch = _torch()
    if cost.dtype == torch.int32:
        return I32
    if cost.dtype == torch.int64:
        return I64
    raise ValueError("cost must be int32 or int64")


def mmbp_lower_bound(cost, M, lb_out, status_out, prefill_tokens=None, ncap_L=0, tp_L=0, stream=None,
                     raise_on_error=True) -> int:
    torch = _torch()
    S, N = cost.shape
    rc = load_library().mmbp_lower_bound(
        _ptr(cost, name="cost"), _cost_dtype(cost), S, N, int(M),
        _ptr(prefill_tokens, torch.int32, (S, N), "prefill_tokens"), int(ncap_L), int(tp_L),
        _ptr(lb_out, torch.int64, (S,), "lb_out"), _ptr(status_out, torch.int32, (S,), "status_out"),
        _stream(stream))
    return _check(rc, raise_on_error)


TP_FLOOR_LARGEST, TP_COVER = 0, 1
LB_RANK_LIMIT = 16384


def mmbp_lower_bound_ex(cost, M, lb_out, status_out, cap=None, kmax=0, prefill_tokens=None, ncap=None, tp=None,
                        tp_form=TP_FLOOR_LARGEST, parts_out=None, stream=None, raise_on_error=True) -> int:
    """cap: host sequence of M ints or None; ncap / tp: host sequences (the level table) or None."""
    torch = _torch()
    S, N = cost.shape
    cap_arr = (C.c_int32 * int(M))(*[int(x) for x in cap]) if cap is not None else None
    nl = len(ncap) if ncap is not None else 0
    ncap_arr = (C.c_int64 * nl)(*[int(x) for x in ncap]) if nl else None
    tp_arr = (C.c_int64 * nl)(*[int(x) for x in tp]) if nl else None
    rc = load_library().mmbp_lower_bound_ex(
        _ptr(cost, name="cost"), _cost_dtype(cost), S, N, int(M), cap_arr, int(kmax),
        _ptr(prefill_tokens, torch.int32, (S, N), "prefill_tokens"), nl, ncap_arr, tp_arr, int(tp_form),
        _ptr(lb_out, torch.int64, (S,), "lb_out"), _ptr(parts_out, torch.int64, (S, 6), "parts_out"),
        _ptr(status_out, torch.int32, (S,), "status_out"), _stream(stream))
    return _check(rc, raise_on_error)


LPT_MAX_N = 16384


def mmbp_lpt_start(cost, M, cap, assign_out, load_out, order_out, status_out, stream=None, raise_on_error=True) -> int:
    torch = _torch()
    S, N = cost.shape
    rc = load_library().mmbp_lpt_start(
        _ptr(cost, name="cost"), _cost_dtype(cost), S, N, int(M), int(cap),
        _ptr(assign_out, torch.int32, (S, N), "assign_out"), _ptr(load_out, torch.int64, (S, M), "load_out"),
        _ptr(order_out, torch.int32, (S, N), "order_out"), _ptr(status_out, torch.int32, (S,), "status_out"),
        _stream(stream))
    return _check(rc, raise_on_error)


def mmbp_local_search(cost, M, cap, max_passes, assign, load_out, makespan_out, passes_out, status_out,
                      evals_out=None, applied_log=None, workspace=None, stream=None, raise_on_error=True,
                      _entry="mmbp_local_search") -> int:
    torch = _torch()
    S, N = cost.shape
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = _ptr(workspace, name="workspace"), workspace.numel() * workspace.element_size()
    rc = getattr(load_library(), _entry)(
        _ptr(cost, name="cost"), _cost_dtype(cost), S, N, int(M), int(cap), int(max_passes),
        _ptr(assign, torch.int32, (S, N), "assign"), _ptr(load_out, torch.int64, (S, M), "load_out"),
        _ptr(makespan_out, torch.int64, (S,), "makespan_out"), _ptr(passes_out, torch.int32, (S,), "passes_out"),
        _ptr(evals_out, torch.int64, (S,), "evals_out"),
        _ptr(applied_log, torch.int64, (S, max(int(max_passes), 0)), "applied_log") if applied_log is not None else None,
        _ptr(status_out, torch.int32, (S,), "status_out"), ws_ptr, ws_bytes, _stream(stream))
    return _check(rc, raise_on_error)


def mmbp_local_search_pruned(cost, M, cap, max_passes, assign, load_out, makespan_out, passes_out, status_out,
                             evals_out=None, applied_log=None, workspace=None, stream=None, raise_on_error=True) -> int:
    return mmbp_local_search(cost, M, cap, max_passes, assign, load_out, makespan_out, passes_out, status_out,
                             evals_out=evals_out, applied_log=applied_log, workspace=workspace, stream=stream,
                             raise_on_error=raise_on_error, _entry="mmbp_local_search_pruned")


def mmbp_local_search_static(cost, M, cap, max_passes, assign, load_out, makespan_out, passes_out, status_out,
                             evals_out=None, applied_log=None, stream=None, raise_on_error=True) -> int:
    """The entry point that allocates nothing: scratch comes from the library's own device array."""
    torch = _torch()
    S, N = cost.shape
    rc = load_library().mmbp_local_search_static(
        _ptr(cost, name="cost"), _cost_dtype(cost), S, N, int(M), int(cap), int(max_passes),
        _ptr(assign, torch.int32, (S, N), "assign"), _ptr(load_out, torch.int64, (S, M), "load_out"),
        _ptr(makespan_out, torch.int64, (S,), "makespan_out"), _ptr(passes_out, torch.int32, (S,), "passes_out"),
        _ptr(evals_out, torch.int64, (S,), "evals_out"),
        _ptr(applied_log, torch.int64, (S, max(int(max_passes), 0)), "applied_log") if applied_log is not None else None,
        _ptr(status_out, torch.int32, (S,), "status_out"), _stream(stream))
    return _check(rc, raise_on_error)


def online_iter_sim(arrival_us, in_len, out_len, params: dict, finish_us, total_us, busy_slot_us,
                    n_prefill_iter, n_decode_iter, trace_hash, status_out, trace_buf=None, trace_len=None,
                    stream=None, raise_on_error=True) -> int:
    """trace_buf: optional uint8 tensor [trace_scenarios, trace_capacity, 24]."""
    torch = _torch()
    S, N = arrival_us.shape
    p = SimParams(int(params["cap"]), int(params.get("policy", 0)), int(params["a_prefill"]), int(params["b_decode"]),
                  int(params["c_prefill"]), int(params["c_decode"]), int(params.get("max_prefill_tokens", 0)))
    tsc = tcap = 0
    if trace_buf is not None:
        if trace_buf.dtype != torch.uint8 or trace_buf.dim() != 3 or trace_buf.shape[2] != 24:
            raise ValueError("trace_buf must be uint8 [scenarios, capacity, 24]")
        tsc, tcap = int(trace_buf.shape[0]), int(trace_buf.shape[1])
    rc = load_library().online_iter_sim(
        _ptr(arrival_us, torch.int64, (S, N), "arrival_us"), _ptr(in_len, torch.int32, (S, N), "in_len"),
        _ptr(out_len, torch.int32, (S, N), "out_len"), S, N, C.byref(p),
        _ptr(finish_us, torch.int64, (S, N), "finish_us"), _ptr(total_us, torch.int64, (S,), "total_us"),
        _ptr(busy_slot_us, torch.int64, (S,), "busy_slot_us"), _ptr(n_prefill_iter, torch.int32, (S,), "n_prefill_iter"),
        _ptr(n_decode_iter, torch.int32, (S,), "n_decode_iter"), _ptr(trace_hash, torch.int64, (S,), "trace_hash"),
        _ptr(trace_buf, name="trace_buf"), _ptr(trace_len, torch.int32, (tsc,), "trace_len") if trace_buf is not None else None,
        tsc, tcap, _ptr(status_out, torch.int32, (S,), "status_out"), _stream(stream))
    return _check(rc, raise_on_error)


# ------------------------------------------------------------------------------------------
# Convenience wrappers used by tests, the smoke check and the benchmark: allocate outputs with
# torch, call the entry point, hand back tensors.  They add no computation.
# ------------------------------------------------------------------------------------------
def _sim_params(params: dict) -> SimParams:
    return SimParams(int(params["cap"]), int(params.get("policy", 0)), int(params["a_prefill"]), int(params["b_decode"]),
                     int(params["c_prefill"]), int(params["c_decode"]), int(params.get("max_prefill_tokens", 0)))


def online_iter_sim_assigned(in_len, out_len, assign, params: dict, finish_us, total_us, busy_slot_us,
                             n_prefill_iter, n_decode_iter, trace_hash, status_out, served_by=None, start_us=None,
                             trace_buf=None, trace_len=None, stream=None, raise_on_error=True) -> int:
    """trace_buf: optional uint8 tensor [trace_scenarios, trace_capacity, 24]."""
    torch = _torch()
    S, N = in_len.shape
    p = _sim_params(params)
    tsc = tcap = 0
    if trace_buf is not None:
        if trace_buf.dtype != torch.uint8 or trace_buf.dim() != 3 or trace_buf.shape[2] != 24:
            raise ValueError("trace_buf must be uint8 [scenarios, capacity, 24]")
        tsc, tcap = int(trace_buf.shape[0]), int(trace_buf.shape[1])
    rc = load_library().online_iter_sim_assigned(
        _ptr(in_len, torch.int32, (S, N), "in_len"), _ptr(out_len, torch.int32, (S, N), "out_len"),
        _ptr(assign, torch.int32, (S, N), "assign"), S, N, C.byref(p),
        _ptr(finish_us, torch.int64, (S, N), "finish_us"), _ptr(total_us, torch.int64, (S,), "total_us"),
        _ptr(busy_slot_us, torch.int64, (S,), "busy_slot_us"), _ptr(n_prefill_iter, torch.int32, (S,), "n_prefill_iter"),
        _ptr(n_decode_iter, torch.int32, (S,), "n_decode_iter"), _ptr(trace_hash, torch.int64, (S,), "trace_hash"),
        _ptr(served_by, torch.int32, (S, N), "served_by") if served_by is not None else None,
        _ptr(start_us, torch.int64, (S, N), "start_us") if start_us is not None else None,
        _ptr(trace_buf, name="trace_buf"), _ptr(trace_len, torch.int32, (tsc,), "trace_len") if trace_buf is not None else None,
        tsc, tcap, _ptr(status_out, torch.int32, (S,), "status_out"), _stream(stream))
    return _check(rc, raise_on_error)


def run_local_search(cost, assign0, M, cap, max_passes, want_log=False, stream=None, raise_on_error=True,
                     pruned=False, use_workspace=True):
    torch = _torch()
    dev = cost.device
    S, N = cost.shape
    out = dict(assign=assign0.clone(), load=torch.empty((S, M), dtype=torch.int64, device=dev),
               makespan=torch.empty(S, dtype=torch.int64, device=dev),
               passes=torch.empty(S, dtype=torch.int32, device=dev),
               evals=torch.empty(S, dtype=torch.int64, device=dev),
               status=torch.empty(S, dtype=torch.int32, device=dev))
    log = None
    if want_log and max_passes > 0:
        log = torch.full((S, max_passes), -1, dtype=torch.int64, device=dev)
    ws_bytes = mmbp_workspace_bytes(S, N, M)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=dev) if ws_bytes and use_workspace else None
    fn = mmbp_local_search_pruned if pruned else mmbp_local_search
    rc = fn(cost, M, cap, max_passes, out["assign"], out["load"], out["makespan"], out["passes"],
            out["status"], evals_out=out["evals"], applied_log=log, workspace=ws, stream=stream,
            raise_on_error=raise_on_error)
    out["rc"] = rc
    out["log"] = log
    out["workspace"] = ws
    return out


def run_lower_bound(cost, M, prefill_tokens=None, ncap_L=0, tp_L=0, stream=None, raise_on_error=True):
    torch = _torch()
    S = cost.shape[0]
    lb = torch.empty(S, dtype=torch.int64, device=cost.device)
    st = torch.empty(S, dtype=torch.int32, device=cost.device)
    rc = mmbp_lower_bound(cost, M, lb, st, prefill_tokens, ncap_L, tp_L, stream=stream, raise_on_error=raise_on_error)
    return dict(rc=rc, lb=lb, status=st)


def run_lpt_start(cost, M, cap, stream=None, raise_on_error=True):
    torch = _torch()
    S, N = cost.shape
    dev = cost.device
    out = dict(assign=torch.empty((S, N), dtype=torch.int32, device=dev), load=torch.empty((S, M), dtype=torch.int64, device=dev),
               order=torch.empty((S, N), dtype=torch.int32, device=dev), status=torch.empty(S, dtype=torch.int32, device=dev))
    out["rc"] = mmbp_lpt_start(cost, M, cap, out["assign"], out["load"], out["order"], out["status"], stream=stream,
                               raise_on_error=raise_on_error)
    return out


def run_lower_bound_ex(cost, M, cap=None, kmax=0, prefill_tokens=None, ncap=None, tp=None, tp_form=TP_FLOOR_LARGEST,
                       stream=None, raise_on_error=True):
    torch = _torch()
    S = cost.shape[0]
    lb = torch.empty(S, dtype=torch.int64, device=cost.device)
    parts = torch.empty((S, 6), dtype=torch.int64, device=cost.device)
    st = torch.empty(S, dtype=torch.int32, device=cost.device)
    rc = mmbp_lower_bound_ex(cost, M, lb, st, cap=cap, kmax=kmax, prefill_tokens=prefill_tokens, ncap=ncap, tp=tp,
                             tp_form=tp_form, parts_out=parts, stream=stream, raise_on_error=raise_on_error)
    return dict(rc=rc, lb=lb, parts=parts, status=st)


def run_online_sim(arrival_us, in_len, out_len, params, trace_scenarios=0, trace_capacity=0, stream=None,
                   raise_on_error=True):
    torch = _torch()
    dev = arrival_us.device
    S, N = arrival_us.shape
    i64 = dict(dtype=torch.int64, device=dev)
    i32 = dict(dtype=torch.int32, device=dev)
    out = dict(finish_us=torch.empty((S, N), **i64), total_us=torch.empty(S, **i64),
               busy_slot_us=torch.empty(S, **i64), n_prefill_iter=torch.empty(S, **i32),
               n_decode_iter=torch.empty(S, **i32), trace_hash=torch.empty(S, **i64),
               status=torch.empty(S, **i32), trace=None, trace_len=None)
    if trace_scenarios > 0 and trace_capacity > 0:
        out["trace"] = torch.zeros((trace_scenarios, trace_capacity, 24), dtype=torch.uint8, device=dev)
        out["trace_len"] = torch.zeros(trace_scenarios, **i32)
    rc = online_iter_sim(arrival_us, in_len, out_len, params, out["finish_us"], out["total_us"],
                         out["busy_slot_us"], out["n_prefill_iter"], out["n_decode_iter"], out["trace_hash"],
                         out["status"], trace_buf=out["trace"], trace_len=out["trace_len"], stream=stream,
                         raise_on_error=raise_on_error)
    out["rc"] = rc
    return out


def run_online_sim_assigned(in_len, out_len, assign, params, trace_scenarios=0, trace_capacity=0, stream=None,
                            raise_on_error=True):
    torch = _torch()
    dev = in_len.device
    S, N = in_len.shape
    i64 = dict(dtype=torch.int64, device=dev)
    i32 = dict(dtype=torch.int32, device=dev)
    out = dict(finish_us=torch.empty((S, N), **i64), total_us=torch.empty(S, **i64),
               busy_slot_us=torch.empty(S, **i64), n_prefill_iter=torch.empty(S, **i32),
               n_decode_iter=torch.empty(S, **i32), trace_hash=torch.empty(S, **i64),
               served_by=torch.empty((S, N), **i32), start_us=torch.empty((S, N), **i64),
               status=torch.empty(S, **i32), trace=None, trace_len=None)
    if trace_scenarios > 0 and trace_capacity > 0:
        out["trace"] = torch.zeros((trace_scenarios, trace_capacity, 24), dtype=torch.uint8, device=dev)
        out["trace_len"] = torch.zeros(trace_scenarios, **i32)
    rc = online_iter_sim_assigned(in_len, out_len, assign, params, out["finish_us"], out["total_us"],
                                  out["busy_slot_us"], out["n_prefill_iter"], out["n_decode_iter"], out["trace_hash"],
                                  out["status"], served_by=out["served_by"], start_us=out["start_us"],
                                  trace_buf=out["trace"], trace_len=out["trace_len"], stream=stream,
                                  raise_on_error=raise_on_error)
    out["rc"] = rc
    return out
