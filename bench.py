#!/usr/bin/env python3
"""Benchmark: one step = lower bound + full local search over the 1024 x 1024 (M = 8) batch.

Prints ONE JSON line.  `value` = candidate moves/swaps evaluated per second (sum of the library's
own evals_out counters / wall time of the timed steps, inputs resident in HBM).  `roofline`
prices the local-search kernel against the chip's int32 vector-ALU issue rate with the fixed
algorithmic op counts (5 per swap candidate, 3 per move candidate); `frac_issued` beside it uses the
2 vector ops per swap candidate that the kernel's inner loop really issues.  `cpu_baseline` times the
CPU oracle on the same batch on the host cores.  `online_sim` reports the second metric
(simulated scenarios per second on the 8192 x 2048 online configuration).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

ALU_PEAK_LANE_OPS = 256 * 64 * 2.4e9      # 256 CUs x 64 int32 lanes/clk x 2.4 GHz
OPS_PER_SWAP, OPS_PER_MOVE = 5, 3
ISSUED_PER_SWAP = 2                       # v_sub_u32 + half a v_min3_u32 + half a v_max3_u32
# HBM bytes of one ls_lds_kernel launch on this workload, from rocprofv3 FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0
# (factors from a 256 MiB device copy; profiles/ls_lds_kernel_c2_counters.md).  To be taken again, or
# set to None, whenever the kernel changes.
LS_LDS_HBM_BYTES_PER_LAUNCH = (4344 * 2.0 + 706 * 1.0) * 1024


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sim", action="store_true", help="skip the simulator and hybrid-pipeline legs")
    ap.add_argument("--no-pruned", action="store_true", help="skip the pruned-scan leg")
    ap.add_argument("--no-large", action="store_true", help="skip the one-large-scenario (multi-workgroup path) leg")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch one plain 256 MiB device copy (calibrates FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (scenarios are independent; see DESIGN.md for how "
              "the batch would shard); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2502_15763_amd import api, workloads as W

    api.load_library()
    torch.cuda.set_device(0)
    K, Wm = args.steps, args.warmup

    c = W.config2()
    cost = torch.from_numpy(c.cost).cuda()
    assign0 = torch.from_numpy(c.assign0).cuda()
    S, N, M = c.S, c.N, c.M
    dev = cost.device
    assigns = [assign0.clone() for _ in range(K + Wm)]
    load = torch.empty((S, M), dtype=torch.int64, device=dev)
    mk = torch.empty(S, dtype=torch.int64, device=dev)
    passes = torch.empty(S, dtype=torch.int32, device=dev)
    evals = torch.empty(S, dtype=torch.int64, device=dev)
    status = torch.empty(S, dtype=torch.int32, device=dev)
    lb = torch.empty(S, dtype=torch.int64, device=dev)
    lbst = torch.empty(S, dtype=torch.int32, device=dev)
    ws_bytes = api.mmbp_workspace_bytes(S, N, M)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=dev) if ws_bytes else None
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]

    def step(k, timed_idx=None):
        api.mmbp_lower_bound(cost, M, lb, lbst)
        if timed_idx is not None:
            ev[timed_idx][0].record()
        api.mmbp_local_search(cost, M, c.cap, c.max_passes, assigns[k], load, mk, passes, status,
                              evals_out=evals, workspace=ws)
        if timed_idx is not None:
            ev[timed_idx][1].record()

    if args.copy_probe:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for k in range(Wm):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        step(Wm + k, k)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall = t1 - t0
    ls_ms = [a.elapsed_time(b) for a, b in ev]
    ls_avg_s = sum(ls_ms) / len(ls_ms) / 1e3

    ev_np = evals.cpu().numpy().view(np.uint64)
    passes_np = passes.cpu().numpy()
    total_evals = int(ev_np.sum())
    scans = passes_np.astype(np.int64) + (status.cpu().numpy() == 0)
    move_evals = int((scans * (N * (M - 1))).sum())
    swap_evals = total_evals - move_evals
    value = total_evals * K / wall
    alg_ops = swap_evals * OPS_PER_SWAP + move_evals * OPS_PER_MOVE
    achieved = alg_ops / ls_avg_s

    out = {
        "metric": "candidate moves evaluated/sec (MMBP local search)",
        "value": value, "unit": "candidates/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": wall / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": "configs[1]: 1024 scenarios x N=1024 requests, M=8 instances, batch cap 64 "
                               "(capacity 128 per instance), lognormal lengths, int32 costs, search to "
                               "convergence (max_passes 1024); step = mmbp_lower_bound + mmbp_local_search",
                   "S": S, "N": N, "M": M, "cap": c.cap, "max_passes": c.max_passes,
                   "mean_passes": float(passes_np.mean()), "candidates_per_step": total_evals},
        "roofline": {"bound": "alu", "achieved": achieved / 1e12, "peak": ALU_PEAK_LANE_OPS / 1e12,
                     "unit": "Tops/s (int32 lane-ops priced at 5 per swap and 3 per move candidate; the kernel issues 2 per "
                             "swap candidate, see frac_issued)",
                     "frac": achieved / ALU_PEAK_LANE_OPS, "traffic": LS_LDS_HBM_BYTES_PER_LAUNCH,
                     "kernel": "ls_lds_kernel (the mmbp_local_search launch)", "kernel_ms": ls_avg_s * 1e3,
                     "frac_issued": swap_evals * ISSUED_PER_SWAP / ls_avg_s / ALU_PEAK_LANE_OPS},
    }

    # the same search with the pruned scan (identical results): reported on its own, never mixed
    # into `value` or the roofline, which count evaluated candidates only
    if not args.no_pruned:
      pr_assign = [assign0.clone() for _ in range(K)]
      api.mmbp_local_search_pruned(cost, M, c.cap, c.max_passes, assign0.clone(), load, mk, passes, status,
                                   evals_out=evals, workspace=ws)
      torch.cuda.synchronize()
      t0 = time.perf_counter()
      for k in range(K):
          api.mmbp_local_search_pruned(cost, M, c.cap, c.max_passes, pr_assign[k], load, mk, passes, status,
                                       evals_out=evals, workspace=ws)
      torch.cuda.synchronize()
      pr_s = (time.perf_counter() - t0) / K
      out["pruned_scan"] = {"entry": "mmbp_local_search_pruned", "ms_per_call": pr_s * 1e3,
                            "passes_per_s": float(passes_np.sum()) / pr_s,
                            "full_scan_equivalent_candidates_per_s": total_evals / pr_s,
                            "same_result_as_full_scan": bool(torch.equal(pr_assign[K - 1], assigns[Wm + K - 1]))}

    # one large scenario (multi-workgroup path): reported on its own, not part of `value`
    if not args.no_large:
        c4 = W.config4()
        cost4 = torch.from_numpy(c4.cost).cuda()
        a4 = torch.from_numpy(c4.assign0).cuda()
        r4 = api.run_local_search(cost4, a4, c4.M, c4.cap, 64)   # warm-up, allocates outputs and workspace
        torch.cuda.synchronize()
        reps = 3
        starts = [a4.clone() for _ in range(reps)]
        t0 = time.perf_counter()
        for k in range(reps):
            api.mmbp_local_search(cost4, c4.M, c4.cap, 64, starts[k], r4["load"], r4["makespan"], r4["passes"],
                                  r4["status"], evals_out=r4["evals"], workspace=r4["workspace"])
        torch.cuda.synchronize()
        dt4 = (time.perf_counter() - t0) / reps
        ev4 = int(r4["evals"].cpu().numpy().view(np.uint64).sum())
        out["large_scenario"] = {"workload": "configs[3]: 1 scenario x N=65536 requests, M=64 instances, 64 passes "
                                             "(three kernels per pass in the caller's workspace)",
                                 "ms_per_call": dt4 * 1e3, "us_per_pass": dt4 * 1e6 / 64,
                                 "candidates_per_s": ev4 / dt4,
                                 "frac_issued": (ev4 - 64 * c4.N * (c4.M - 1)) * ISSUED_PER_SWAP / dt4 / ALU_PEAK_LANE_OPS}

    if not args.no_sim:
        w = W.config5()
        arr = torch.from_numpy(w.arrival_us).cuda()
        il = torch.from_numpy(w.in_len).cuda()
        ol = torch.from_numpy(w.out_len).cuda()
        r = api.run_online_sim(arr, il, ol, w.params)            # warm-up, allocates outputs
        torch.cuda.synchronize()
        reps = 3
        t0 = time.perf_counter()
        for _ in range(reps):
            api.online_iter_sim(arr, il, ol, w.params, r["finish_us"], r["total_us"], r["busy_slot_us"],
                                r["n_prefill_iter"], r["n_decode_iter"], r["trace_hash"], r["status"])
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps
        iters = int(r["n_prefill_iter"].sum().item() + r["n_decode_iter"].sum().item())

        def utilisation():
            busy = r["busy_slot_us"].double()
            return float((busy / (w.params["cap"] * r["total_us"].double())).mean().item())

        out["online_sim"] = {"metric": "online sim scenarios/sec", "value": w.S / dt, "unit": "scenarios/s",
                             "ms_per_call": dt * 1e3, "iterations_per_s": iters / dt,
                             "workload": "configs[4]: 8192 scenarios x 2048 requests, cap 64",
                             "slot_utilisation": {"rule": utilisation()}}
        # the paper's baseline (prefill first, with / without batched prefill) on the same scenarios
        for name, pol in (("prefill_first", api.POLICY_PREFILL_FIRST), ("prefill_first_single", api.POLICY_PREFILL_FIRST_SINGLE)):
            pp = dict(w.params, policy=pol)
            t0 = time.perf_counter()
            api.online_iter_sim(arr, il, ol, pp, r["finish_us"], r["total_us"], r["busy_slot_us"],
                                r["n_prefill_iter"], r["n_decode_iter"], r["trace_hash"], r["status"])
            torch.cuda.synchronize()
            out["online_sim"]["slot_utilisation"][name] = utilisation()
            out["online_sim"].setdefault("baseline_ms_per_call", {})[name] = (time.perf_counter() - t0) * 1e3

    if not args.no_sim:
        # the paper's offline + online combination on the same lengths, all requests known at t = 0:
        # local search over M = cap clients, then the simulator that runs the assignment as sorted
        # per-client queues with stealing; against it the FCFS simulator on the same requests
        Sh, cap = 2048, w.params["cap"]
        hin, hout = il[:Sh].contiguous(), ol[:Sh].contiguous()
        hcost = torch.from_numpy(W.job_cost(w.in_len[:Sh], w.out_len[:Sh], np.int32)).cuda()
        rr = torch.from_numpy(np.tile((np.arange(w.N) % cap).astype(np.int32), (Sh, 1))).cuda()
        t0 = time.perf_counter()
        hls = api.run_local_search(hcost, rr, cap, w.N, 1024, pruned=True)
        torch.cuda.synchronize()
        ls_dt = time.perf_counter() - t0
        ha = api.run_online_sim_assigned(hin, hout, hls["assign"], w.params)      # warm-up, allocates outputs
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            api.online_iter_sim_assigned(hin, hout, hls["assign"], w.params, ha["finish_us"], ha["total_us"],
                                         ha["busy_slot_us"], ha["n_prefill_iter"], ha["n_decode_iter"],
                                         ha["trace_hash"], ha["status"])
        torch.cuda.synchronize()
        sim_dt = (time.perf_counter() - t0) / 3
        hf = api.run_online_sim(torch.zeros((Sh, w.N), dtype=torch.int64, device=dev), hin, hout, w.params)
        torch.cuda.synchronize()
        util = lambda r: float((r["busy_slot_us"].double() / (cap * r["total_us"].double())).mean().item())
        out["hybrid_pipeline"] = {
            "workload": "first 2048 scenarios of configs[4] (2048 requests each), all requests at t = 0, M = cap = 64",
            "offline_search_ms": ls_dt * 1e3, "offline_search_entry": "mmbp_local_search_pruned",
            "assigned_sim_ms": sim_dt * 1e3, "assigned_sim_scenarios_per_s": Sh / sim_dt,
            "slot_utilisation": {"offline_assignment_then_queues_with_stealing": util(ha), "fcfs": util(hf)},
            "mean_total_s": {"offline_assignment_then_queues_with_stealing": float(ha["total_us"].double().mean().item()) / 1e6,
                             "fcfs": float(hf["total_us"].double().mean().item()) / 1e6}}

    if not args.no_cpu_baseline:
        from oracle import oracle as O
        t0 = time.perf_counter()
        o = O.local_search(c.cost, c.assign0, M, c.cap, c.max_passes)
        dt = time.perf_counter() - t0
        ok = (np.array_equal(assigns[Wm + K - 1].cpu().numpy(), o["assign"])
              and np.array_equal(ev_np, o["evals"]) and np.array_equal(mk.cpu().numpy(), o["makespan"]))
        out["cpu_baseline"] = {"value": float(o["evals"].sum()) / dt, "unit": "candidates/s",
                               "cores": O.num_threads(), "kind": "oracle",
                               "sample": "all 1024 scenarios of the same batch, local search only (OpenMP over scenarios)",
                               "seconds": dt}
        out["parity_with_oracle"] = bool(ok)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
