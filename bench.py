#!/usr/bin/env python3
"""Benchmark: one step = lower bound + full local search over the 4096 x 4096 (M = 16) batch.

Prints ONE JSON line.  `value` = candidate moves/swaps evaluated per second (sum of the library's
own evals_out counters / wall time of the timed steps, inputs resident in HBM).

`roofline` sets the local-search kernel against the chip's 32-bit vector-ALU issue rate.  The
kernel evaluates a swap candidate with 2 vector lane-operations (one subtract, half a three-way min,
half a three-way max) and a move candidate with 3; `achieved` counts exactly those, `peak` is
256 CUs x 64 lanes x 2.4 GHz, and `peak_calibrated` is what the library's register-only loop of the
same instruction mix sustains on this device in this run.  `priced_5_3` repeats the figure at the
price of a straightforward evaluation (5 per swap, 3 per move), which the kernel's formulation
undercuts, so that ratio can exceed 1 and is not a utilisation.  `traffic` and the instruction counts
come from the rocprofv3 counter summaries under profiles/ and are dropped (null) when the kernel
sources have changed since those were taken.

`cpu_baseline` times the CPU oracle on a bounded sample of the same batch on the host cores.
`secondary` repeats the measurement on the 1024 x 1024 (M = 8) batch, `online_sim` reports the second
metric (simulated scenarios per second on the 8192 x 2048 online configuration).
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

N_CU, LANES_PER_CU_CLK, CLOCK_HZ = 256, 64, 2.4e9
ALU_PEAK_LANE_OPS = N_CU * LANES_PER_CU_CLK * CLOCK_HZ       # 39.3e12 32-bit lane-ops/s
ISSUE_PEAK_WAVE_INSTS = N_CU * 2 * CLOCK_HZ                  # per CU and clock: one vector (4 SIMDs x 1/4) + one scalar
ISSUED_PER_SWAP, ISSUED_PER_MOVE = 2, 3
PRICED_PER_SWAP, PRICED_PER_MOVE = 5, 3
CSRC = os.path.join(ROOT, "paper_2502_15763_amd", "csrc")
KERNEL_SOURCES = {
    "ls_lds_kernel": ("ls_lds.hip", "ls_tile.hpp", "mmbp_dev.hpp"),
    "online_sim_kernel": ("online_sim.hip", "sim_trace.hpp", "mmbp_dev.hpp"),
}


def sources_sha256(kernel):
    h = hashlib.sha256()
    for f in KERNEL_SOURCES[kernel]:
        with open(os.path.join(CSRC, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def profile_facts():
    """Counter figures per (kernel, workload) from the `bench-facts:` lines of the summaries under
    profiles/; a figure is used only while the kernel's sources hash to what the summary records."""
    facts = {}
    pdir = os.path.join(ROOT, "profiles")
    for name in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not name.endswith((".md", ".txt")):
            continue
        for line in open(os.path.join(pdir, name), errors="ignore"):
            m = re.match(r"\s*bench-facts:\s*(\{.*\})\s*$", line)
            if m:
                try:
                    d = json.loads(m.group(1))
                except ValueError:
                    continue
                d["file"] = "profiles/" + name
                facts[(d.get("kernel"), d.get("workload"))] = d
    return facts


def current_facts(facts, kernel, workload):
    d = facts.get((kernel, workload))
    if not d or d.get("sources_sha256") != sources_sha256(kernel):
        return None
    return d


def hbm_traffic(d):
    if not d or "fetch_kib" not in d or "write_kib" not in d:
        return None
    return (d["fetch_kib"] * d.get("fetch_factor", 1.0) + d["write_kib"] * d.get("write_factor", 1.0)) * 1024.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true", help="skip the 1024 x 1024 batch")
    ap.add_argument("--no-sim", action="store_true", help="skip the simulator and hybrid-pipeline legs")
    ap.add_argument("--no-pruned", action="store_true", help="skip the pruned-scan leg")
    ap.add_argument("--no-large", action="store_true", help="skip the one-large-scenario (multi-workgroup path) leg")
    ap.add_argument("--only", choices=["headline", "secondary", "sim", "pipeline", "probe"], default=None,
                    help="run one leg only (for profiling a single kernel)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch one plain 256 MiB device copy (calibrates FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc)")
    ap.add_argument("--tail-study", action="store_true",
                    help="with the secondary leg: time its longest scenarios alone and in company (per-scan latency)")
    ap.add_argument("--kernel-hash", action="store_true", help="print the source hashes the profile summaries record, and exit")
    args = ap.parse_args()
    if args.kernel_hash:
        print(json.dumps({k: sources_sha256(k) for k in KERNEL_SOURCES}))
        return
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU (scenarios are independent: more GPUs would each take a share of "
              "the batch, with no exchange between them); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.only:
        args.no_cpu_baseline = True
        args.no_pruned = args.no_large = True
        args.no_secondary = args.only != "secondary"
        args.no_sim = args.only not in ("sim", "pipeline")

    import numpy as np
    import torch
    from paper_2502_15763_amd import api, workloads as W

    api.load_library()
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    K, Wm = args.steps, args.warmup
    facts = profile_facts()

    if args.copy_probe:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- calibration: what the vector ALUs sustain on the tile loop's instruction mix ----
    def calibrate():
        blocks, trips = 2048, 12000                      # 8 waves per SIMD resident, ~20 ms
        buf = torch.empty(blocks * 256, dtype=torch.int32, device=dev)
        api.mmbp_valu_probe(buf, blocks, 200)
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            ops = api.mmbp_valu_probe(buf, blocks, trips)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b)
            best = ms if best is None else min(best, ms)
        rate = ops / (best / 1e3)
        # the same loop with fewer resident waves: what one, two and four waves per SIMD sustain (a workgroup
        # of 256 threads is one wave per SIMD of its CU; 256 workgroups are one per CU)
        by_occ = {}
        for waves, nb in ((1, 256), (2, 512), (4, 1024)):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            o = api.mmbp_valu_probe(buf[:nb * 256], nb, trips)
            b.record()
            torch.cuda.synchronize()
            by_occ[str(waves)] = o / (a.elapsed_time(b) / 1e3) / ALU_PEAK_LANE_OPS
        by_occ["8"] = rate / ALU_PEAK_LANE_OPS
        return {"lane_ops_per_s": rate, "ms": best, "lane_ops": ops,
                "implied_clock_ghz": rate / (N_CU * LANES_PER_CU_CLK) / 1e9,
                "fraction_of_nominal_peak_by_waves_per_simd": by_occ,
                "kernel": "valu_probe_kernel (registers only: 32 v_sub_u32 + 16 v_min3_u32 + 16 v_max3_u32 + 8 v_add_u32 per trip)"}

    calib = calibrate()
    if args.only == "probe":
        print(json.dumps({"calibration": calib}))
        return

    # ---- one offline batch: lower bound + local search, K timed steps ----
    def offline_leg(c, label, steps, warm):
        cost = torch.from_numpy(c.cost).cuda()
        assign0 = torch.from_numpy(c.assign0).cuda()
        S, N, M = c.S, c.N, c.M
        assigns = [assign0.clone() for _ in range(steps + warm)]
        load = torch.empty((S, M), dtype=torch.int64, device=dev)
        mk = torch.empty(S, dtype=torch.int64, device=dev)
        passes = torch.empty(S, dtype=torch.int32, device=dev)
        evals = torch.empty(S, dtype=torch.int64, device=dev)
        status = torch.empty(S, dtype=torch.int32, device=dev)
        lb = torch.empty(S, dtype=torch.int64, device=dev)
        lbst = torch.empty(S, dtype=torch.int32, device=dev)
        ws_bytes = api.mmbp_workspace_bytes(S, N, M)
        ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=dev) if ws_bytes else None
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]

        def step(k, timed_idx=None):
            api.mmbp_lower_bound(cost, M, lb, lbst)
            if timed_idx is not None:
                ev[timed_idx][0].record()
            api.mmbp_local_search(cost, M, c.cap, c.max_passes, assigns[k], load, mk, passes, status,
                                  evals_out=evals, workspace=ws)
            if timed_idx is not None:
                ev[timed_idx][1].record()

        for k in range(warm):
            step(k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            step(warm + k, k)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ls_ms = [a.elapsed_time(b) for a, b in ev]
        ls_avg_s = sum(ls_ms) / len(ls_ms) / 1e3

        ev_np = evals.cpu().numpy().view(np.uint64)
        passes_np = passes.cpu().numpy()
        status_np = status.cpu().numpy()
        total_evals = int(ev_np.sum())
        scans = passes_np.astype(np.int64) + (status_np == 0)
        move_evals = int((scans * (N * (M - 1))).sum())
        swap_evals = total_evals - move_evals
        issued = swap_evals * ISSUED_PER_SWAP + move_evals * ISSUED_PER_MOVE
        priced = swap_evals * PRICED_PER_SWAP + move_evals * PRICED_PER_MOVE
        d = current_facts(facts, "ls_lds_kernel", label)
        roof = {"bound": "alu", "achieved": issued / ls_avg_s / 1e12, "peak": ALU_PEAK_LANE_OPS / 1e12,
                "unit": "T lane-ops/s (32-bit vector lane operations the evaluation issues: 2 per swap candidate, 3 per move "
                        "candidate; peak = 256 CUs x 64 lanes x 2.4 GHz)",
                "frac": issued / ls_avg_s / ALU_PEAK_LANE_OPS,
                "peak_calibrated": calib["lane_ops_per_s"] / 1e12,
                "frac_of_calibrated": issued / ls_avg_s / calib["lane_ops_per_s"],
                "traffic": hbm_traffic(d),
                "traffic_source": d["file"] if d else None,
                "kernel": "ls_lds_kernel (the mmbp_local_search launch)", "kernel_ms": ls_avg_s * 1e3,
                "lane_ops_per_launch": issued,
                "measured_valu_lane_ops_per_candidate": (d["valu_insts"] * 64.0 / total_evals) if d and "valu_insts" in d else None,
                "priced_5_3": {"achieved": priced / ls_avg_s / 1e12, "ratio_to_peak": priced / ls_avg_s / ALU_PEAK_LANE_OPS,
                               "note": "candidates priced at 5 lane-ops per swap and 3 per move (a direct evaluation); the "
                                       "kernel needs 2 per swap, so this ratio can exceed 1 and is not a utilisation"}}
        res = dict(S=S, N=N, M=M, cap=c.cap, max_passes=c.max_passes, wall=wall, ms_per_step=wall / steps * 1e3,
                   total_evals=total_evals, value=total_evals * steps / wall, roofline=roof,
                   mean_passes=float(passes_np.mean()), max_passes_seen=int(passes_np.max()),
                   converged=int((status_np == 0).sum()), evals=ev_np, passes=passes_np, makespan=mk.cpu().numpy(),
                   assign_last=assigns[warm + steps - 1], cost=cost, assign0=assign0, ws=ws,
                   bufs=(load, mk, passes, status, evals))
        return res

    out = {"calibration": calib}
    c3 = W.config3()
    head = offline_leg(c3, "c3", K, Wm) if args.only in (None, "headline") else None
    if head:
        out.update({
            "metric": "candidate moves evaluated/sec (MMBP local search)",
            "value": head["value"], "unit": "candidates/s", "n_gpus": 1, "steps": K, "warmup": Wm,
            "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "int64 costs and loads at the interface; int32 inside the kernel (exact narrowing)", "data": "synthetic",
            "config": {"workload": "configs[2]: 4096 scenarios x N=4096 requests, M=16 instances, batch cap 128 "
                                   "(capacity 256 per instance), bimodal lengths, int64 costs, max_passes 64; "
                                   "step = mmbp_lower_bound + mmbp_local_search (the largest configuration that is a batch on one GPU)",
                       "S": head["S"], "N": head["N"], "M": head["M"], "cap": head["cap"], "max_passes": head["max_passes"],
                       "mean_passes": head["mean_passes"], "max_passes_seen": head["max_passes_seen"],
                       "scenarios_converged": head["converged"], "candidates_per_step": head["total_evals"]},
            "roofline": head["roofline"],
        })

    c2 = W.config2()
    sec = None
    if not args.no_secondary:
        sec = offline_leg(c2, "c2", max(K, 10), Wm)
        out["secondary"] = {
            "workload": "configs[1]: 1024 scenarios x N=1024 requests, M=8 instances, capacity 128 per instance, lognormal "
                        "lengths, int32 costs, search to convergence (max_passes 1024)",
            "value": sec["value"], "unit": "candidates/s", "ms_per_step": sec["ms_per_step"],
            "mean_passes": sec["mean_passes"], "max_passes_seen": sec["max_passes_seen"],
            "candidates_per_step": sec["total_evals"], "roofline": sec["roofline"]}
        if args.tail_study:
            # where this batch loses time: its scenarios with the most passes, alone and in company (one launch each)
            import dataclasses
            order = np.argsort(-sec["passes"], kind="stable")
            study = []
            for kk in (1, 64, 256, 512, 1024):
                idx = np.sort(order[:kk])
                sub = dataclasses.replace(c2, S=kk, cost=c2.cost[idx], assign0=c2.assign0[idx], in_len=c2.in_len[idx],
                                          out_len=c2.out_len[idx])
                r = offline_leg(sub, "c2-subset", 5, 1)
                scans = int(r["passes"].max()) + 1
                study.append({"scenarios": kk, "kernel_ms": r["roofline"]["kernel_ms"], "scans_of_the_longest": scans,
                              "us_per_scan_of_the_longest": r["roofline"]["kernel_ms"] * 1e3 / scans,
                              "scans_total": int(r["passes"].sum()) + kk, "frac": r["roofline"]["frac"]})
            out["secondary"]["tail_study"] = {
                "what": "the K scenarios of configs[1] with the most passes, one launch per K (K = 1: the longest scenario "
                        "alone on the chip; 256: one workgroup per CU; 512: two per CU, all resident; 1024: the whole batch)",
                "runs": study}

    # the same search with the pruned scan (identical results): reported on its own, never mixed
    # into `value` or the roofline, which count evaluated candidates only
    if not args.no_pruned and sec:
        load, mk, passes, status, evals = sec["bufs"]
        reps = 10
        pr_assign = [sec["assign0"].clone() for _ in range(reps)]
        api.mmbp_local_search_pruned(sec["cost"], c2.M, c2.cap, c2.max_passes, sec["assign0"].clone(), load, mk, passes, status,
                                     evals_out=evals, workspace=sec["ws"])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(reps):
            api.mmbp_local_search_pruned(sec["cost"], c2.M, c2.cap, c2.max_passes, pr_assign[k], load, mk, passes, status,
                                         evals_out=evals, workspace=sec["ws"])
        torch.cuda.synchronize()
        pr_s = (time.perf_counter() - t0) / reps
        out["pruned_scan"] = {"entry": "mmbp_local_search_pruned", "workload": "configs[1]", "ms_per_call": pr_s * 1e3,
                              "passes_per_s": float(sec["passes"].sum()) / pr_s,
                              "full_scan_equivalent_candidates_per_s": sec["total_evals"] / pr_s,
                              "same_result_as_full_scan": bool(torch.equal(pr_assign[reps - 1], sec["assign_last"]))}

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
        mv4 = 64 * c4.N * (c4.M - 1)
        out["large_scenario"] = {"workload": "configs[3]: 1 scenario x N=65536 requests, M=64 instances, 64 passes "
                                             "(multi-workgroup path in the caller's workspace)",
                                 "ms_per_call": dt4 * 1e3, "us_per_pass": dt4 * 1e6 / 64,
                                 "candidates_per_s": ev4 / dt4,
                                 "frac_of_alu_peak": ((ev4 - mv4) * ISSUED_PER_SWAP + mv4 * ISSUED_PER_MOVE) / dt4 / ALU_PEAK_LANE_OPS}

    w = None
    if not args.no_sim:
        w = W.config5()
        arr = torch.from_numpy(w.arrival_us).cuda()
        il = torch.from_numpy(w.in_len).cuda()
        ol = torch.from_numpy(w.out_len).cuda()
        if args.only != "pipeline":
            r = api.run_online_sim(arr, il, ol, w.params)            # warm-up, allocates outputs
            torch.cuda.synchronize()
            reps = 5
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            t0 = time.perf_counter()
            for k in range(reps):
                evs[k][0].record()
                api.online_iter_sim(arr, il, ol, w.params, r["finish_us"], r["total_us"], r["busy_slot_us"],
                                    r["n_prefill_iter"], r["n_decode_iter"], r["trace_hash"], r["status"])
                evs[k][1].record()
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / reps
            k_s = sum(a.elapsed_time(b) for a, b in evs) / reps / 1e3
            iters = int(r["n_prefill_iter"].sum().item() + r["n_decode_iter"].sum().item())

            def utilisation():
                busy = r["busy_slot_us"].double()
                return float((busy / (w.params["cap"] * r["total_us"].double())).mean().item())

            d = current_facts(facts, "online_sim_kernel", "c5")
            insts = (d["valu_insts"] + d["salu_insts"]) if d and "valu_insts" in d and "salu_insts" in d else None
            out["online_sim"] = {"metric": "online sim scenarios/sec", "value": w.S / dt, "unit": "scenarios/s",
                                 "ms_per_call": dt * 1e3, "iterations_per_s": iters / dt,
                                 "workload": "configs[4]: 8192 scenarios x 2048 requests, cap 64",
                                 "dtype": "int64 times, int32 lengths",
                                 "roofline": {"bound": "alu",
                                              "unit": "T wave-instructions/s (vector + scalar issue; peak = 256 CUs x (1 vector + 1 scalar) "
                                                      "per clock x 2.4 GHz; one dependent chain per wave, so latency-bound below it)",
                                              "achieved": (insts / k_s / 1e12) if insts else None,
                                              "peak": ISSUE_PEAK_WAVE_INSTS / 1e12,
                                              "frac": (insts / k_s / ISSUE_PEAK_WAVE_INSTS) if insts else None,
                                              "wave_insts_per_launch": insts,
                                              "wave_insts_per_simulated_iteration": (insts / iters) if insts else None,
                                              "traffic": hbm_traffic(d), "traffic_source": d["file"] if d else None,
                                              "algorithmic_bytes": w.S * w.N * (16 + 8),
                                              "hbm_gb_per_s_algorithmic": w.S * w.N * 24 / k_s / 1e9,
                                              "kernel": "online_sim_kernel", "kernel_ms": k_s * 1e3},
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

        if args.only in (None, "pipeline"):
            # the paper's offline + online combination on the same lengths, all requests known at t = 0:
            # local search over M = cap clients, then the simulator that runs the assignment as sorted
            # per-client queues with stealing; against it the FCFS simulator on the same requests
            Sh, cap = 2048, w.params["cap"]
            hin, hout = il[:Sh].contiguous(), ol[:Sh].contiguous()
            hcost = torch.from_numpy(W.job_cost(w.in_len[:Sh], w.out_len[:Sh], np.int32)).cuda()
            rr = torch.from_numpy(np.tile((np.arange(w.N) % cap).astype(np.int32), (Sh, 1))).cuda()
            def second_call(f):                           # the first call loads the kernel and allocates: the second is timed
                f()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                r = f()
                torch.cuda.synchronize()
                return r, time.perf_counter() - t0
            hls, ls_dt = second_call(lambda: api.run_local_search(hcost, rr, cap, w.N, 1024, pruned=True))
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
            util = lambda q: float((q["busy_slot_us"].double() / (cap * q["total_us"].double())).mean().item())
            out["hybrid_pipeline"] = {
                "workload": "first 2048 scenarios of configs[4] (2048 requests each), all requests at t = 0, M = cap = 64",
                "offline_search_ms": ls_dt * 1e3, "offline_search_entry": "mmbp_local_search_pruned",
                "assigned_sim_ms": sim_dt * 1e3, "assigned_sim_scenarios_per_s": Sh / sim_dt,
                "slot_utilisation": {"offline_assignment_then_queues_with_stealing": util(ha), "fcfs": util(hf)},
                "mean_total_s": {"offline_assignment_then_queues_with_stealing": float(ha["total_us"].double().mean().item()) / 1e6,
                                 "fcfs": float(hf["total_us"].double().mean().item()) / 1e6}}

    if not args.no_sim and args.only in (None, "pipeline"):
        # the paper's own shape (Table "Experiment Settings": 1319 requests, 200 clients, its time model), lengths
        # drawn from the printed means and deviations: baseline policy against offline assignment + online rule
        Sp = 1024
        pin, pout = W.paper_shaped(S=Sp)
        Np, Mp = pin.shape[1], W.PAPER_PARAMS["cap"]
        capp = -(-Np // Mp)                               # a balanced number of requests per client
        din, dout = torch.from_numpy(pin).cuda(), torch.from_numpy(pout).cuda()
        pcost = torch.from_numpy(W.job_cost(pin, pout, np.int32)).cuda()
        zero_arr = torch.zeros((Sp, Np), dtype=torch.int64, device=dev)
        pp = dict(W.PAPER_PARAMS)
        def second_call(f):                               # the first call loads the kernel and allocates: the second is timed
            f()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            r = f()
            torch.cuda.synchronize()
            return r, time.perf_counter() - t0
        lpt, lpt_dt = second_call(lambda: api.run_lpt_start(pcost, Mp, capp))
        pls, pls_dt = second_call(lambda: api.run_local_search(pcost, lpt["assign"], Mp, capp, 1024, pruned=True))
        pa, pa_dt = second_call(lambda: api.run_online_sim_assigned(din, dout, pls["assign"], pp))
        pb = api.run_online_sim(zero_arr, din, dout, dict(pp, policy=api.POLICY_PREFILL_FIRST_SINGLE))
        pr_ = api.run_online_sim(zero_arr, din, dout, pp)
        plb = api.run_lower_bound_ex(pcost, Mp, cap=[capp] * Mp)
        torch.cuda.synchronize()
        utilp = lambda q: float((q["busy_slot_us"].double() / (Mp * q["total_us"].double())).mean().item())
        tot = lambda q: float(q["total_us"].double().mean().item()) / 1e6
        out["paper_shaped"] = {
            "workload": "1024 scenarios x 1319 requests on 200 clients, lengths ~ the paper's printed means / deviations, its time "
                        "model (0.13 ms/token + 25 ms prefill, 0.21 ms/token + 29 ms decode); synthetic stand-in, not its dataset",
            "lpt_start_ms": lpt_dt * 1e3, "pruned_local_search_ms": pls_dt * 1e3,
            "local_search_mean_passes": float(pls["passes"].double().mean().item()), "assigned_sim_ms": pa_dt * 1e3,
            "offline_makespan_over_lower_bound": float((pls["makespan"].double() / plb["lb"].double()).mean().item()),
            "slot_utilisation": {"baseline_fcfs_prefill_first_single": utilp(pb), "online_rule_only": utilp(pr_),
                                 "offline_assignment_plus_online_rule": utilp(pa)},
            "mean_total_s": {"baseline_fcfs_prefill_first_single": tot(pb), "online_rule_only": tot(pr_),
                             "offline_assignment_plus_online_rule": tot(pa)},
            "paper_context": "the paper reports 80.2 % -> 89.1 % utilisation and 201.00 s -> 190.58 s on its own hardware and data"}

    if not args.no_cpu_baseline and head:
        from oracle import oracle as O
        ns = 512                                          # bounded sample: the first 512 of the 4096 scenarios
        t0 = time.perf_counter()
        o = O.local_search(c3.cost[:ns], c3.assign0[:ns], c3.M, c3.cap, c3.max_passes)
        dt = time.perf_counter() - t0
        ok = (np.array_equal(head["assign_last"][:ns].cpu().numpy(), o["assign"])
              and np.array_equal(head["evals"][:ns], o["evals"]) and np.array_equal(head["makespan"][:ns], o["makespan"]))
        out["cpu_baseline"] = {"value": float(o["evals"].sum()) / dt, "unit": "candidates/s",
                               "cores": O.num_threads(), "kind": "oracle",
                               "sample": "the first 512 of the 4096 scenarios of the same batch, local search only "
                                         "(OpenMP over scenarios)",
                               "seconds": dt}
        out["parity_with_oracle"] = bool(ok)
        if w is not None:
            nso = w.S                                     # the literal oracle runs the whole batch in well under a minute
            t0 = time.perf_counter()
            os_ = O.online_iter_sim(w.arrival_us[:nso], w.in_len[:nso], w.out_len[:nso], w.params)
            dts = time.perf_counter() - t0
            api.online_iter_sim(arr, il, ol, w.params, r["finish_us"], r["total_us"], r["busy_slot_us"],
                                r["n_prefill_iter"], r["n_decode_iter"], r["trace_hash"], r["status"])
            torch.cuda.synchronize()
            oks = (np.array_equal(r["finish_us"][:nso].cpu().numpy(), os_["finish_us"])
                   and np.array_equal(r["trace_hash"][:nso].cpu().numpy().view(np.uint64), os_["trace_hash"]))
            out["online_sim"]["cpu_baseline"] = {"value": nso / dts, "unit": "scenarios/s", "cores": O.num_threads(),
                                                 "kind": "oracle", "sample": "all 8192 scenarios (OpenMP over scenarios)",
                                                 "seconds": dts}
            out["online_sim"]["parity_with_oracle"] = bool(oks)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
