"""Helpers for the GPU parity tests: move numpy inputs to the device, call the library through the
Python binding of its C ABI, and compare element by element with the CPU oracle."""
import sys

import numpy as np


def say(msg):
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def u64(t):
    return t.cpu().numpy().view(np.uint64)


def gpu_local_search(cost, assign0, M, cap, max_passes, want_log=True, pruned=False, use_workspace=True):
    """use_workspace=False: no workspace is passed, which keeps a shape that fits the LDS on the
    one-workgroup path even where the library would prefer the multi-workgroup one."""
    import torch
    from paper_2502_15763_amd import api
    r = api.run_local_search(to_dev(cost), to_dev(assign0.astype(np.int32)), M, cap, max_passes, want_log=want_log,
                             pruned=pruned, use_workspace=use_workspace)
    torch.cuda.synchronize()
    out = dict(rc=r["rc"], assign=r["assign"].cpu().numpy(), load=r["load"].cpu().numpy(),
               makespan=r["makespan"].cpu().numpy(), passes=r["passes"].cpu().numpy(), evals=u64(r["evals"]),
               status=r["status"].cpu().numpy())
    if r["log"] is not None:
        out["log"] = u64(r["log"])
    return out


def compare_ls(g, o, check_log=True, label=""):
    assert g["rc"] == 0 and o["rc"] == 0
    for key in ("status", "passes", "makespan", "evals", "load", "assign"):
        if not np.array_equal(g[key], o[key]):
            bad = np.argwhere(g[key].reshape(g[key].shape[0], -1) != o[key].reshape(o[key].shape[0], -1))
            s = int(bad[0][0])
            raise AssertionError(f"{label}: {key} differs in {len(set(bad[:, 0].tolist()))} scenarios; first s={s}: "
                                 f"gpu passes={g['passes'][s]} oracle passes={o['passes'][s]} "
                                 f"gpu mk={g['makespan'][s]} oracle mk={o['makespan'][s]} "
                                 f"gpu log={g.get('log', [[]])[s][:6] if 'log' in g else None} "
                                 f"oracle log={o.get('log', [[]])[s][:6] if 'log' in o else None}")
    if check_log and "log" in g and "log" in o:
        for s in range(g["passes"].shape[0]):
            p = int(o["passes"][s])
            assert np.array_equal(g["log"][s][:p], o["log"][s][:p]), f"{label}: applied ids differ in scenario {s}"


def gpu_lower_bound(cost, M, prefill_tokens=None, ncap_L=0, tp_L=0):
    import torch
    from paper_2502_15763_amd import api
    pt = to_dev(prefill_tokens.astype(np.int32)) if prefill_tokens is not None else None
    r = api.run_lower_bound(to_dev(cost), M, pt, ncap_L, tp_L)
    torch.cuda.synchronize()
    return dict(rc=r["rc"], lb=r["lb"].cpu().numpy(), status=r["status"].cpu().numpy())


def gpu_lower_bound_ex(cost, M, cap=None, kmax=0, prefill_tokens=None, ncap=None, tp=None, tp_form=0):
    import torch
    from paper_2502_15763_amd import api
    pt = to_dev(prefill_tokens.astype(np.int32)) if prefill_tokens is not None else None
    r = api.run_lower_bound_ex(to_dev(cost), M, cap=cap, kmax=kmax, prefill_tokens=pt, ncap=ncap, tp=tp, tp_form=tp_form,
                               raise_on_error=False)
    torch.cuda.synchronize()
    return dict(rc=r["rc"], lb=r["lb"].cpu().numpy(), parts=r["parts"].cpu().numpy(), status=r["status"].cpu().numpy())


def gpu_lpt_start(cost, M, cap):
    import torch
    from paper_2502_15763_amd import api
    r = api.run_lpt_start(to_dev(cost), M, cap, raise_on_error=False)
    torch.cuda.synchronize()
    return dict(rc=r["rc"], assign=r["assign"].cpu().numpy(), load=r["load"].cpu().numpy(), order=r["order"].cpu().numpy(),
                status=r["status"].cpu().numpy())


def gpu_online_sim(arrival, in_len, out_len, params, trace_scenarios=0, trace_capacity=0):
    import torch
    from paper_2502_15763_amd import api
    r = api.run_online_sim(to_dev(arrival.astype(np.int64)), to_dev(in_len.astype(np.int32)),
                           to_dev(out_len.astype(np.int32)), params, trace_scenarios, trace_capacity)
    torch.cuda.synchronize()
    out = dict(rc=r["rc"])
    for k in ("finish_us", "total_us", "busy_slot_us", "n_prefill_iter", "n_decode_iter", "status"):
        out[k] = r[k].cpu().numpy()
    out["trace_hash"] = u64(r["trace_hash"])
    if r["trace"] is not None:
        from oracle.oracle import TRACE_DTYPE
        out["trace"] = r["trace"].cpu().numpy().view(TRACE_DTYPE).reshape(trace_scenarios, trace_capacity)
        out["trace_len"] = r["trace_len"].cpu().numpy()
        # The library runs another kernel variant when no trace records are wanted (the one the benchmark
        # times): the same call without a trace buffer must give the same outputs, so whatever a test
        # establishes for `out` holds for that variant too.
        if r["rc"] == 0:
            r2 = api.run_online_sim(to_dev(arrival.astype(np.int64)), to_dev(in_len.astype(np.int32)),
                                    to_dev(out_len.astype(np.int32)), params, 0, 0)
            torch.cuda.synchronize()
            assert r2["rc"] == 0
            for k in ("finish_us", "total_us", "busy_slot_us", "n_prefill_iter", "n_decode_iter", "status"):
                assert np.array_equal(r2[k].cpu().numpy(), out[k]), f"untraced variant: {k} differs from the traced run"
            assert np.array_equal(u64(r2["trace_hash"]), out["trace_hash"]), "untraced variant: trace_hash differs"
    return out


def gpu_online_sim_assigned(in_len, out_len, assign, params, trace_scenarios=0, trace_capacity=0):
    import torch
    from paper_2502_15763_amd import api
    r = api.run_online_sim_assigned(to_dev(in_len.astype(np.int32)), to_dev(out_len.astype(np.int32)),
                                    to_dev(assign.astype(np.int32)), params, trace_scenarios, trace_capacity)
    torch.cuda.synchronize()
    out = dict(rc=r["rc"])
    for k in ("finish_us", "total_us", "busy_slot_us", "n_prefill_iter", "n_decode_iter", "status", "served_by", "start_us"):
        out[k] = r[k].cpu().numpy()
    out["trace_hash"] = u64(r["trace_hash"])
    if r["trace"] is not None:
        from oracle.oracle import TRACE_DTYPE
        out["trace"] = r["trace"].cpu().numpy().view(TRACE_DTYPE).reshape(trace_scenarios, trace_capacity)
        out["trace_len"] = r["trace_len"].cpu().numpy()
        if r["rc"] == 0:                                 # the variant without trace records, as in gpu_online_sim
            r2 = api.run_online_sim_assigned(to_dev(in_len.astype(np.int32)), to_dev(out_len.astype(np.int32)),
                                             to_dev(assign.astype(np.int32)), params, 0, 0)
            torch.cuda.synchronize()
            assert r2["rc"] == 0
            for k in ("finish_us", "total_us", "busy_slot_us", "n_prefill_iter", "n_decode_iter", "status", "served_by", "start_us"):
                assert np.array_equal(r2[k].cpu().numpy(), out[k]), f"untraced variant: {k} differs from the traced run"
            assert np.array_equal(u64(r2["trace_hash"]), out["trace_hash"]), "untraced variant: trace_hash differs"
    return out


def compare_sim(g, o, label=""):
    assert g["rc"] == 0 and o["rc"] == 0
    for k in ("status", "total_us", "busy_slot_us", "n_prefill_iter", "n_decode_iter", "trace_hash", "finish_us"):
        if not np.array_equal(g[k], o[k]):
            bad = np.argwhere(g[k].reshape(g[k].shape[0], -1) != o[k].reshape(o[k].shape[0], -1))
            raise AssertionError(f"{label}: {k} differs, first at {bad[0].tolist()}: gpu={g[k][tuple(bad[0]) if g[k].ndim > 1 else bad[0][0]]}")
    for k in ("served_by", "start_us"):
        if k in g and k in o:
            assert np.array_equal(g[k], o[k]), f"{label}: {k} differs"
    if "trace" in g and o.get("trace") is not None:
        assert np.array_equal(g["trace_len"], o["trace_len"]), f"{label}: trace_len"
        for s in range(g["trace"].shape[0]):
            n = min(int(o["trace_len"][s]), g["trace"].shape[1])
            assert np.array_equal(g["trace"][s][:n], o["trace"][s][:n]), f"{label}: trace records differ, scenario {s}"
