"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit.

Integer work throughout (costs, loads, times are integer microseconds), so the bar is exact
equality of assignments, loads, makespans, pass counts, candidate counts, applied candidate ids,
finish times and canonical traces."""
import numpy as np
import pytest

from paper_2502_15763_amd import workloads as W
from gpu_util import (say, gpu_local_search, compare_ls, gpu_lower_bound, gpu_lower_bound_ex, gpu_lpt_start, gpu_online_sim, compare_sim,
                      gpu_online_sim_assigned)

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ local search
SMALL_SHAPES = [
    # N, M, cap, cost_hi
    (1, 1, 1, 10), (1, 3, 1, 10), (2, 2, 1, 10), (5, 5, 1, 50), (6, 2, 3, 30), (7, 3, 3, 1000),
    (16, 4, 4, 100), (16, 4, 7, 100), (33, 5, 9, 500), (64, 4, 16, 40000), (64, 4, 20, 40000),
    (65, 3, 30, 300), (100, 7, 15, 2000), (127, 2, 64, 100), (128, 8, 16, 5), (130, 8, 40, 3),
    (200, 16, 13, 100000), (257, 9, 33, 700), (300, 3, 300, 50), (96, 33, 3, 1000), (70, 70, 1, 99),
]


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_ls_small_random(oracle, dtype):
    rng = np.random.default_rng(2024)
    for (N, M, cap, hi) in SMALL_SHAPES:
        S = 5
        say(f"ls_small dtype={np.dtype(dtype).name} N={N} M={M} cap={cap} hi={hi}")
        cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=hi, dtype=dtype)
        o = oracle.local_search(cost, assign, M, cap, 200, want_log=True)
        g = gpu_local_search(cost, assign, M, cap, 200)
        compare_ls(g, o, label=f"N={N} M={M} cap={cap}")


def test_ls_shapes_between_64_and_156_kb_of_lds(oracle):
    """Layouts that need more than the default 64 KB of LDS per workgroup but still fit one CU."""
    rng = np.random.default_rng(31)
    for (S, N, M, cap, passes) in [(5, 2048, 64, 40, 400), (3, 8192, 16, 600, 40), (3, 10000, 8, 1300, 30)]:
        cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=50000, dtype=np.int32, start="rr")
        say(f"ls large-LDS shapes S={S} N={N} M={M}")
        o = oracle.local_search(cost, assign, M, cap, passes, want_log=True)
        g = gpu_local_search(cost, assign, M, cap, passes, use_workspace=False)       # one workgroup per scenario
        compare_ls(g, o, label=f"large LDS N={N} M={M}")
        g = gpu_local_search(cost, assign, M, cap, passes)                            # the library's choice of path
        compare_ls(g, o, label=f"large LDS N={N} M={M}, with workspace")


def test_ls_maximum_sizes(oracle):
    """The largest client count (256), a long request list (2^18 requests, two passes against the
    oracle) and the largest request count (2^20: loads only, max_passes = 0)."""
    rng = np.random.default_rng(8)
    cost, assign = W.random_offline(rng, 2, 3000, 256, 20, cost_hi=40000, dtype=np.int32)
    say("ls M=256 N=3000")
    compare_ls(gpu_local_search(cost, assign, 256, 20, 40), oracle.local_search(cost, assign, 256, 20, 40, want_log=True),
               label="M=256")
    cost, assign = W.random_offline(rng, 1, 1 << 18, 4, 1 << 17, cost_hi=3000, dtype=np.int32, start="rr")
    say("ls N=2^18 M=4, 2 passes")
    compare_ls(gpu_local_search(cost, assign, 4, 1 << 17, 2), oracle.local_search(cost, assign, 4, 1 << 17, 2, want_log=True),
               label="N=2^18")
    cost, assign = W.random_offline(rng, 1, 1 << 20, 3, 1 << 19, cost_hi=500, dtype=np.int32, start="rr")
    say("ls N=2^20 M=3, loads only")
    compare_ls(gpu_local_search(cost, assign, 3, 1 << 19, 0), oracle.local_search(cost, assign, 3, 1 << 19, 0, want_log=True),
               label="N=2^20")


def test_ls_pass_limits_and_resume(oracle):
    rng = np.random.default_rng(5)
    cost, assign = W.random_offline(rng, 6, 90, 5, 20, cost_hi=5000, dtype=np.int32)
    for mp in (0, 1, 2, 3):
        say(f"ls_pass_limit max_passes={mp}")
        o = oracle.local_search(cost, assign, 5, 20, mp, want_log=True)
        g = gpu_local_search(cost, assign, 5, 20, mp, want_log=mp > 0)
        compare_ls(g, o, label=f"max_passes={mp}")
    g1 = gpu_local_search(cost, assign, 5, 20, 2)
    g2 = gpu_local_search(cost, g1["assign"], 5, 20, 2)
    g12 = gpu_local_search(cost, assign, 5, 20, 4)
    assert np.array_equal(g2["assign"], g12["assign"]) and np.array_equal(g2["load"], g12["load"])


def test_ls_bad_scenarios_do_not_disturb_others(oracle):
    rng = np.random.default_rng(6)
    cost, assign = W.random_offline(rng, 6, 40, 4, 12, cost_hi=900, dtype=np.int64)
    cost[1, 7] = -5                 # BAD_COST
    assign[2, 3] = 4                # BAD_ASSIGN (out of range)
    assign[3, :] = 0                # BAD_ASSIGN (more than cap on client 0)
    cost[4, :2] = 1 << 61           # BAD_COST (sum >= 2^62)
    say("ls_bad_scenarios")
    o = oracle.local_search(cost, assign, 4, 12, 100, want_log=True)
    g = gpu_local_search(cost, assign, 4, 12, 100)
    assert o["status"].tolist()[1:5] == [3, 2, 2, 3]
    compare_ls(g, o, label="bad scenarios")


def test_ls_pruned_best_values_ending_in_sixteen_ones(oracle):
    """The pruned scan keeps 16 bits of every row's best value as a filter for the rows that may attain the best
    value of the pass; rows it never wrote hold 0xFFFF.  Loads are placed so that many passes have a best value
    whose low 16 bits are all ones: every such row then passes the filter and must fail the exact test."""
    rng = np.random.default_rng(5)
    for (S, M, n, target, slack) in [(600, 3, 9, 65535, 2), (300, 5, 70, 131071, 0), (300, 4, 40, 65535 + 65536 * 3, 1)]:
        N = M * n
        cost = rng.integers(0, 25, size=(S, N)).astype(np.int32)
        assign = np.tile((np.arange(N) % M).astype(np.int32), (S, 1))
        for j in range(M):                                # job j is on client j: one big job each puts the loads near the target
            cost[:, j] = target - rng.integers(12 * n - 50, 12 * n + 50, size=S)
        say(f"ls pruned, best values near {target}: S={S} M={M} n={n}")
        o = oracle.local_search(cost, assign, M, n + slack, 60, want_log=True)
        compare_ls(gpu_local_search(cost, assign, M, n + slack, 60, pruned=True), o, label=f"pruned, values near {target}")
        compare_ls(gpu_local_search(cost, assign, M, n + slack, 60), o, label=f"full scan, values near {target}")


def test_ls_large_costs_need_64_bit(oracle):
    """Loads far above 2^31: the exact 64-bit path."""
    rng = np.random.default_rng(8)
    cost, assign = W.random_offline(rng, 4, 60, 4, 18, cost_hi=(1 << 40), dtype=np.int64)
    say("ls_large_costs")
    o = oracle.local_search(cost, assign, 4, 18, 100, want_log=True)
    g = gpu_local_search(cost, assign, 4, 18, 100)
    compare_ls(g, o, label="large costs")
    # near the int32 narrowing boundary as well
    cost, assign = W.random_offline(rng, 4, 60, 4, 18, cost_hi=(1 << 27), dtype=np.int64)
    o = oracle.local_search(cost, assign, 4, 18, 100, want_log=True)
    g = gpu_local_search(cost, assign, 4, 18, 100)
    compare_ls(g, o, label="boundary costs")


def test_ls_config1(oracle):
    for slack in (0, 16):
        c = W.config1(slack=slack)
        say(f"ls_config1 slack={slack}")
        o = oracle.local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, want_log=True)
        g = gpu_local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes)
        compare_ls(g, o, label=f"c1 slack={slack}")


def test_ls_config2_full(oracle):
    c = W.config2()
    say("ls_config2 full 1024x1024 tight")
    o = oracle.local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, want_log=True)
    g = gpu_local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes)
    compare_ls(g, o, label="c2")
    assert (o["status"] == 0).all()


def test_ls_config2_slack(oracle):
    c = W.config2(S=48, slack=64)
    say("ls_config2 slack S=48")
    o = oracle.local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, want_log=True)
    g = gpu_local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes)
    compare_ls(g, o, label="c2 slack")
    applied = o["log"][o["log"] != np.iinfo(np.uint64).max]
    assert (applied < c.N * c.M).any(), "the slack case must apply at least one move"


_C3 = {}


def _config3_on_gpu():
    """The full batch (4096 x 4096, int64 costs, 64 passes) in ONE call, the launch configuration the
    benchmark times; computed once and shared by the tests below."""
    if not _C3:
        c = W.config3()
        say("ls_config3 full batch on GPU")
        _C3["c"] = c
        _C3["g"] = gpu_local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes)
    return _C3["c"], _C3["g"]


@pytest.mark.parametrize("part", range(8))
def test_ls_config3_full_batch(oracle, part):
    """Every scenario of the batch against the oracle (scenarios are independent, so the oracle takes
    them in eight slices of 512): all outputs and the applied ids."""
    c, g = _config3_on_gpu()
    lo, hi = part * c.S // 8, (part + 1) * c.S // 8
    say(f"ls_config3 oracle on scenarios {lo}..{hi - 1}")
    o = oracle.local_search(c.cost[lo:hi], c.assign0[lo:hi], c.M, c.cap, c.max_passes, want_log=True)
    gs = {k: (v[lo:hi] if isinstance(v, np.ndarray) else v) for k, v in g.items()}
    compare_ls(gs, o, label=f"c3 scenarios {lo}..{hi - 1}")


def test_ls_config3_properties():
    """What holds for every scenario of the batch without an oracle."""
    c, g = _config3_on_gpu()
    assert np.array_equal(g["load"].sum(axis=1), c.cost.sum(axis=1))
    assert np.array_equal(g["makespan"], g["load"].max(axis=1))
    cnt = np.stack([np.bincount(a, minlength=c.M) for a in g["assign"]])
    assert cnt.max() <= c.cap
    assert np.isin(g["status"], (0, 1)).all() and ((g["status"] == 1) == (g["passes"] == c.max_passes)).all()
    per_scan = c.N * (c.M - 1) + (c.N * c.N - c.M * (c.N // c.M) ** 2) // 2     # tight capacity: counts never change
    scans = g["passes"].astype(np.int64) + (g["status"] == 0)                    # a converged search ran one more scan
    assert np.array_equal(g["evals"], (scans * per_scan).astype(np.uint64))
    start = np.stack([np.bincount(a, weights=w.astype(np.float64), minlength=c.M) for a, w in zip(c.assign0, c.cost)]).max(axis=1)
    assert (g["makespan"] < start.astype(np.int64)).all()


def test_ls_config3_first_32_to_convergence(oracle):
    c = W.config3(S=32, max_passes=4000)
    say("ls_config3 scenarios 0..31 to convergence")
    g = gpu_local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes)
    say("ls_config3 oracle on the same 32 scenarios")
    o = oracle.local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, want_log=True)
    assert (o["status"] == 0).all()
    compare_ls(g, o, label="c3 0..31 converged")


def test_ls_repeatable(oracle):
    """Same input three times, through the LDS path and the multi-workgroup path: identical outputs
    (the argmin has a total order, so nothing may depend on scheduling)."""
    for c, passes in ((W.config2(S=64), 1024), (W.config4(slack=256), 5)):
        say(f"ls repeatable {c.name if hasattr(c, 'name') else ''} N={c.N}")
        runs = [gpu_local_search(c.cost, c.assign0, c.M, c.cap, passes) for _ in range(3)]
        for r in runs[1:]:
            for k in ("assign", "load", "makespan", "passes", "evals", "status", "log"):
                assert np.array_equal(r[k], runs[0][k]), k


def test_ls_config3_slack_converged(oracle):
    c = W.config3(S=4, slack=128, max_passes=4000)
    say("ls_config3 slack, to convergence, S=4")
    o = oracle.local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, want_log=True)
    g = gpu_local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes)
    compare_ls(g, o, label="c3 slack")
    g = gpu_local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, use_workspace=False)
    compare_ls(g, o, label="c3 slack, one workgroup per scenario")


@pytest.mark.parametrize("slack,passes", [(0, 256), (256, 256)])
def test_ls_config4(oracle, slack, passes):
    """One scenario of 65536 requests on the multi-workgroup path for the configuration's full 256
    passes, with the tight capacity (swaps only) and with slack (moves and swaps)."""
    c = W.config4(slack=slack)
    say(f"ls_config4 N=65536 M=64 slack={slack} passes={passes}")
    g = gpu_local_search(c.cost, c.assign0, c.M, c.cap, passes)
    o = oracle.local_search(c.cost, c.assign0, c.M, c.cap, passes, want_log=True)
    compare_ls(g, o, label=f"c4 slack={slack}")


def test_ls_multi_workgroup_path_batch(oracle):
    """Shapes too large for one workgroup's LDS, several scenarios per call, slack capacity so that
    moves and swaps are both applied; one scenario needs the 64-bit path."""
    rng = np.random.default_rng(77)
    S, N, M, cap = 3, 14000, 6, 2500
    cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=30000, dtype=np.int32, start="rr")
    cost = cost.astype(np.int64)
    cost[2] *= 1 << 16                      # loads above the 32-bit narrowing bound
    say(f"ls multi-workgroup batch S={S} N={N} M={M}")
    o = oracle.local_search(cost, assign, M, cap, 6, want_log=True)
    g = gpu_local_search(cost, assign, M, cap, 6)
    compare_ls(g, o, label="multi-workgroup batch")


def test_ls_multi_workgroup_resumed_calls_equal_one_search(oracle):
    """Multi-workgroup path: a call stops at its pass limit with TRUNCATED and `assign` in/out lets the
    caller go on; two calls of 4 passes must equal the oracle's single run of 8 (assignment, loads,
    applied ids in order, candidate counts summed).  This is how a caller gets past the per-call limit
    of that path (a larger max_passes is refused on the host, see tests/test_abi.py)."""
    rng = np.random.default_rng(80)
    S, N, M, cap = 2, 14000, 6, 2500
    cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=30000, dtype=np.int32)
    say(f"ls multi-workgroup resume S={S} N={N} M={M}")
    o = oracle.local_search(cost, assign, M, cap, 8, want_log=True)
    g1 = gpu_local_search(cost, assign, M, cap, 4)
    g2 = gpu_local_search(cost, g1["assign"], M, cap, 4)
    assert (g1["status"] == 1).all() and (g1["passes"] == 4).all()
    assert np.array_equal(g2["assign"], o["assign"]) and np.array_equal(g2["load"], o["load"])
    assert np.array_equal(g2["makespan"], o["makespan"]) and np.array_equal(g2["status"], o["status"])
    assert np.array_equal(g1["passes"] + g2["passes"], o["passes"])
    assert np.array_equal(g1["evals"] + g2["evals"], o["evals"])
    for s in range(S):
        ids = np.concatenate([g1["log"][s][:g1["passes"][s]], g2["log"][s][:g2["passes"][s]]])
        assert np.array_equal(ids, o["log"][s][:o["passes"][s]])


def test_ls_multi_workgroup_moves_in_place(oracle):
    """Multi-workgroup path, uneven client sizes and slack capacity: a run of moves (the layout is
    updated in place, rebuilt only when the target client's slots are full) mixed with swaps."""
    rng = np.random.default_rng(78)
    S, N, M, cap = 2, 14000, 6, 2600
    cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=30000, dtype=np.int32)
    say(f"ls multi-workgroup moves S={S} N={N} M={M}")
    o = oracle.local_search(cost, assign, M, cap, 30, want_log=True)
    g = gpu_local_search(cost, assign, M, cap, 30)
    compare_ls(g, o, label="multi-workgroup moves")
    moves = int((o["log"][o["log"] >= 0] < N * M).sum())
    assert moves >= 10, moves                      # the case must exercise the move path


def test_ls_multi_workgroup_heavy_ties(oracle):
    """Multi-workgroup path with costs from a tiny range: almost every candidate ties, so the
    lowest-id rule decides every pass (full scan and pruned scan)."""
    rng = np.random.default_rng(79)
    S, N, M, cap = 2, 14000, 7, 2100
    cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=4, dtype=np.int32)
    say(f"ls multi-workgroup ties S={S} N={N} M={M}")
    o = oracle.local_search(cost, assign, M, cap, 10, want_log=True)
    compare_ls(gpu_local_search(cost, assign, M, cap, 10), o, label="multi-workgroup ties")
    compare_ls(gpu_local_search(cost, assign, M, cap, 10, pruned=True), o, label="multi-workgroup ties, pruned")


@pytest.mark.parametrize("seed", [1000, 1008])
def test_ls_multi_workgroup_client_out_of_reach(oracle, seed):
    """Multi-workgroup path, few clients, costs 0..3: loads end up within a few units of each other,
    so for some client NO swap with the critical client can reach the best value (its load plus the
    makespan exceeds twice that value), while thousands of rows of the other clients tie.  The
    selection must give such a client no partners (regression: a wrapping difference once did)."""
    rng = np.random.default_rng(seed)
    S, N, M, cap = 3, 22000, 4, 5500
    cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=3, dtype=np.int32)
    say(f"ls multi-workgroup out-of-reach client seed={seed}")
    o = oracle.local_search(cost, assign, M, cap, 30, want_log=True)
    compare_ls(gpu_local_search(cost, assign, M, cap, 30), o, label=f"out of reach, seed {seed}")
    compare_ls(gpu_local_search(cost, assign, M, cap, 30, pruned=True), o, label=f"out of reach, pruned, seed {seed}")


def test_ls_few_large_scenarios_take_either_path(oracle):
    """Shapes that fit one workgroup's LDS but leave most of the chip idle: with the optional
    workspace the multi-workgroup path runs, without it the one-workgroup path; both must give the
    oracle's result, and a workspace that is too small or misaligned only selects the fallback."""
    import torch
    from paper_2502_15763_amd import api
    rng = np.random.default_rng(91)
    for (S, N, M, cap, passes) in [(1, 4096, 16, 256, 120), (3, 5000, 10, 520, 60), (12, 3500, 7, 500, 40)]:
        assert api.mmbp_workspace_bytes(S, N, M) > 0 and api.mmbp_workspace_bytes(1024, N, M) == 0
        cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=20000, dtype=np.int32)
        say(f"ls either path S={S} N={N} M={M}")
        o = oracle.local_search(cost, assign, M, cap, passes, want_log=True)
        for pruned in (False, True):
            compare_ls(gpu_local_search(cost, assign, M, cap, passes, pruned=pruned), o, label=f"multi-workgroup N={N} pruned={pruned}")
            compare_ls(gpu_local_search(cost, assign, M, cap, passes, pruned=pruned, use_workspace=False), o,
                       label=f"one workgroup N={N} pruned={pruned}")
    # too small / misaligned workspace: not an error here, the one-workgroup path runs
    S, N, M, cap = 1, 4096, 16, 256
    cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=20000, dtype=np.int32)
    o = oracle.local_search(cost, assign, M, cap, 20, want_log=True)
    need = api.mmbp_workspace_bytes(S, N, M)
    for ws in (torch.empty(need - 1, dtype=torch.uint8, device="cuda"), torch.empty(need + 256, dtype=torch.uint8, device="cuda")[16:]):
        out = dict(assign=torch.from_numpy(assign).cuda(), load=torch.empty((S, M), dtype=torch.int64, device="cuda"),
                   makespan=torch.empty(S, dtype=torch.int64, device="cuda"), passes=torch.empty(S, dtype=torch.int32, device="cuda"),
                   status=torch.empty(S, dtype=torch.int32, device="cuda"))
        rc = api.mmbp_local_search(torch.from_numpy(cost).cuda(), M, cap, 20, out["assign"], out["load"], out["makespan"],
                                   out["passes"], out["status"], workspace=ws)
        torch.cuda.synchronize()
        assert rc == 0
        assert np.array_equal(out["assign"].cpu().numpy(), o["assign"]) and np.array_equal(out["passes"].cpu().numpy(), o["passes"])


# ------------------------------------------------------------------ pruned scan (identical results)
def test_ls_pruned_small_random(oracle):
    """The pruned scan must return exactly what the full search returns (the oracle is the full
    search): assignments, loads, passes, applied ids, status and the full-scan candidate count."""
    rng = np.random.default_rng(2025)
    for (N, M, cap, hi) in SMALL_SHAPES:
        S = 5
        say(f"ls_pruned N={N} M={M} cap={cap} hi={hi}")
        cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=hi, dtype=np.int32)
        o = oracle.local_search(cost, assign, M, cap, 200, want_log=True)
        g = gpu_local_search(cost, assign, M, cap, 200, pruned=True)
        compare_ls(g, o, label=f"pruned N={N} M={M} cap={cap}")


def test_ls_pruned_configs(oracle):
    c = W.config2()
    say("ls_pruned config2 full")
    o = oracle.local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, want_log=True)
    compare_ls(gpu_local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, pruned=True), o, label="pruned c2")
    c = W.config2(S=16, slack=64)
    say("ls_pruned config2 slack (moves applied)")
    o = oracle.local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, want_log=True)
    compare_ls(gpu_local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, pruned=True), o, label="pruned c2 slack")
    c = W.config3(S=6, max_passes=4000)
    say("ls_pruned config3 S=6 int64 costs, to convergence")
    o = oracle.local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, want_log=True)
    compare_ls(gpu_local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, pruned=True), o, label="pruned c3")
    c = W.config4(slack=256)
    say("ls_pruned config4 (multi-workgroup path), 12 passes, slack")
    o = oracle.local_search(c.cost, c.assign0, c.M, c.cap, 12, want_log=True)
    compare_ls(gpu_local_search(c.cost, c.assign0, c.M, c.cap, 12, pruned=True), o, label="pruned c4")
    # a scenario that needs the 64-bit kernel next to narrow ones
    rng = np.random.default_rng(5)
    cost, assign = W.random_offline(rng, 3, 200, 5, 50, cost_hi=1000, dtype=np.int64)
    cost[1] *= 1 << 22
    say("ls_pruned with a 64-bit scenario")
    o = oracle.local_search(cost, assign, 5, 50, 300, want_log=True)
    compare_ls(gpu_local_search(cost, assign, 5, 50, 300, pruned=True), o, label="pruned 64-bit mix")


def test_ls_pruned_sorted_search_with_ties_and_uneven_clients(oracle):
    """The pruned scan keeps every client's positions sorted and finds partners by binary search:
    uneven client sizes (random start, ranges of several 64-position segments), costs from a small range
    (many equal keys, so equal neighbours above and below), swaps and moves mixed."""
    rng = np.random.default_rng(2026)
    for (S, N, M, cap, hi, passes) in [(4, 2000, 5, 600, 50, 300), (4, 700, 3, 400, 7, 200), (3, 3000, 11, 280, 100000, 150),
                                       (6, 130, 2, 129, 2, 100)]:
        say(f"ls_pruned sorted search N={N} M={M} cap={cap} hi={hi}")
        cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=hi, dtype=np.int32)
        o = oracle.local_search(cost, assign, M, cap, passes, want_log=True)
        compare_ls(gpu_local_search(cost, assign, M, cap, passes, pruned=True, use_workspace=False), o,
                   label=f"pruned sorted N={N} M={M}")
    # many small clients, no binding limit, round-robin start: nearly every pass is a move, applied in place in
    # the sorted layout until a client's range is full (then the jobs are regrouped)
    for (S, N, M, cap, hi, passes) in [(3, 2048, 64, 2048, 60000, 400), (3, 640, 10, 640, 900, 200)]:
        say(f"ls_pruned moves in place N={N} M={M}")
        cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=hi, dtype=np.int32, start="rr")
        o = oracle.local_search(cost, assign, M, cap, passes, want_log=True)
        assert (o["log"][:, :20] < N * M).any()
        compare_ls(gpu_local_search(cost, assign, M, cap, passes, pruned=True, use_workspace=False), o,
                   label=f"pruned moves in place N={N} M={M}")


# ------------------------------------------------------------------ lower bound
def test_lb_parity(oracle):
    rng = np.random.default_rng(31)
    for (N, M, hi, dtype) in [(1, 1, 10, np.int32), (3, 5, 10, np.int64), (5, 4, 100, np.int32), (9, 8, 3, np.int32),
                              (64, 4, 40000, np.int32), (1000, 7, 1 << 20, np.int64), (4097, 16, 1 << 40, np.int64),
                              (5000, 256, 1000, np.int32), (300, 255, 7, np.int32)]:
        say(f"lb N={N} M={M}")
        cost = rng.integers(0, hi + 1, size=(7, N)).astype(dtype)
        tok = rng.integers(1, 3000, size=(7, N)).astype(np.int32)
        for kw in (dict(), dict(prefill_tokens=tok, ncap_L=5000, tp_L=675000)):
            o = oracle.lower_bound(cost, M, **kw)
            g = gpu_lower_bound(cost, M, **kw)
            assert np.array_equal(g["status"], o["status"]) and np.array_equal(g["lb"], o["lb"]), (N, M, kw.keys())
    cost = np.array([[3, -1, 4], [1, 2, 3]], np.int64)
    o = oracle.lower_bound(cost, 2)
    g = gpu_lower_bound(cost, 2)
    assert g["status"].tolist() == o["status"].tolist() == [3, 0] and g["lb"].tolist() == o["lb"].tolist()
    # a negative token count invalidates the scenario (only when the prefill term is enabled)
    cost = np.array([[10, 10], [10, 10]], np.int64)
    tok = np.array([[100, -1], [100, 7000]], np.int32)
    for kw in (dict(ncap_L=5000, tp_L=675000), dict(ncap_L=0, tp_L=675000)):
        o = oracle.lower_bound(cost, 2, prefill_tokens=tok, **kw)
        g = gpu_lower_bound(cost, 2, prefill_tokens=tok, **kw)
        assert g["status"].tolist() == o["status"].tolist() and g["lb"].tolist() == o["lb"].tolist(), kw


def test_lb_configs(oracle):
    for c in (W.config1(), W.config2(), W.config3(S=256), W.config4()):
        say(f"lb config {c.name}")
        o = oracle.lower_bound(c.cost, c.M)
        g = gpu_lower_bound(c.cost, c.M)
        assert np.array_equal(g["lb"], o["lb"]) and (g["status"] == 0).all()


# ------------------------------------------------------------------ online simulator
def test_sim_small(oracle):
    rng = np.random.default_rng(41)
    for (N, cap, tok, rate) in [(1, 1, 0, 50), (5, 1, 0, 50), (40, 4, 0, 200), (300, 16, 0, 50), (300, 16, 600, 50),
                                (500, 64, 0, 20), (500, 64, 4000, 500), (200, 33, 0, 5), (64, 64, 0, 1e6)]:
        say(f"sim N={N} cap={cap} tok={tok} rate={rate}")
        S = 9
        w = W.config5(S=S, N=N, rate_per_s=rate, seed_offset=N + cap)
        p = dict(w.params, cap=cap, max_prefill_tokens=tok)
        o = oracle.online_iter_sim(w.arrival_us, w.in_len, w.out_len, p, trace_scenarios=S, trace_capacity=3 * N + 8)
        g = gpu_online_sim(w.arrival_us, w.in_len, w.out_len, p, trace_scenarios=S, trace_capacity=3 * N + 8)
        compare_sim(g, o, label=f"N={N} cap={cap} tok={tok}")


def test_sim_paper_constants(oracle):
    in_len, out_len = W.paper_shaped(S=8, N=1319)
    arr = np.zeros_like(in_len, dtype=np.int64)
    p = dict(W.PAPER_PARAMS, cap=64)
    say("sim paper-shaped lengths, all requests at t=0")
    o = oracle.online_iter_sim(arr, in_len, out_len, p, trace_scenarios=2, trace_capacity=5000)
    g = gpu_online_sim(arr, in_len, out_len, p, trace_scenarios=2, trace_capacity=5000)
    compare_sim(g, o, label="paper-shaped")


def test_sim_wide_fields_and_sparse_arrivals(oracle):
    """Records whose fields leave the small-number range of the fast hash (long decode runs, times
    beyond 2^40, prefills of 2^16 tokens and more), decode runs cut by an arrival that finds a free
    slot, and a time model whose decode iterations take no time."""
    rng = np.random.default_rng(77)
    S, N = 6, 40

    def both(arr, inl, outl, p, cap, label):
        say("sim " + label)
        compare_sim(gpu_online_sim(arr, inl, outl, p, S, cap), oracle.online_iter_sim(arr, inl, outl, p, S, cap),
                    label=label)

    # one slot, very long outputs: decode runs of more than 2^16 iterations
    arr = np.sort(rng.integers(0, 10_000, (S, N))).astype(np.int64)
    inl = rng.integers(1, 50, (S, N)).astype(np.int32)
    outl = rng.integers(60_000, 200_000, (S, N)).astype(np.int32)
    both(arr, inl, outl, dict(cap=1, a_prefill=3, b_decode=2, c_prefill=10, c_decode=1, max_prefill_tokens=0),
         4 * N, "long decode runs")
    # arrivals late on the clock (beyond 2^40 us) and far apart: idle jumps, runs cut by arrivals
    arr = ((1 << 41) + np.cumsum(rng.integers(0, 3_000_000, (S, N)), axis=1)).astype(np.int64)
    outl = rng.integers(1, 400, (S, N)).astype(np.int32)
    both(arr, inl, outl, dict(W.C5_PARAMS, cap=8), 6 * N, "late clock, sparse arrivals")
    # big prompts admitted together: P >= 2^16
    arr = np.zeros((S, N), np.int64)
    inl = rng.integers(30_000, 90_000, (S, N)).astype(np.int32)
    both(arr, inl, outl, dict(W.C5_PARAMS, cap=16), 6 * N, "large prefills")
    # decode iterations of zero duration while requests keep arriving
    arr = np.cumsum(rng.integers(0, 2000, (S, N)), axis=1).astype(np.int64)
    inl = rng.integers(1, 300, (S, N)).astype(np.int32)
    both(arr, inl, outl, dict(cap=4, a_prefill=7, b_decode=0, c_prefill=100, c_decode=0, max_prefill_tokens=500),
         6 * N, "zero-time decode")


@pytest.mark.parametrize("policy", [1, 2])
def test_sim_baseline_policies(oracle, policy):
    """The prefill-first baselines (with and without batched prefill) on online and on
    all-at-once workloads, with and without a prefill token cap."""
    for (S, N, cap, tok, rate) in [(9, 300, 16, 0, 50), (9, 300, 16, 600, 200), (6, 500, 64, 0, 20), (5, 64, 64, 0, 1e6)]:
        w = W.config5(S=S, N=N, rate_per_s=rate, seed_offset=policy + N)
        p = dict(w.params, cap=cap, max_prefill_tokens=tok, policy=policy)
        say(f"sim policy={policy} N={N} cap={cap} tok={tok} rate={rate}")
        o = oracle.online_iter_sim(w.arrival_us, w.in_len, w.out_len, p, trace_scenarios=S, trace_capacity=4 * N)
        g = gpu_online_sim(w.arrival_us, w.in_len, w.out_len, p, trace_scenarios=S, trace_capacity=4 * N)
        compare_sim(g, o, label=f"policy {policy} N={N}")
    in_len, out_len = W.paper_shaped(S=4, N=1319)
    arr = np.zeros_like(in_len, dtype=np.int64)
    p = dict(W.PAPER_PARAMS, cap=64, policy=policy)
    say(f"sim policy={policy} paper-shaped lengths")
    compare_sim(gpu_online_sim(arr, in_len, out_len, p, 2, 6000), oracle.online_iter_sim(arr, in_len, out_len, p, 2, 6000),
                label=f"policy {policy} paper-shaped")


def test_sim_bad_input(oracle):
    w = W.config5(S=5, N=50)
    w.arrival_us[1, 10] = w.arrival_us[1, 9] - 1
    w.in_len[2, 0] = 0
    w.out_len[3, 49] = 0
    say("sim bad input")
    o = oracle.online_iter_sim(w.arrival_us, w.in_len, w.out_len, w.params)
    g = gpu_online_sim(w.arrival_us, w.in_len, w.out_len, w.params)
    assert o["status"].tolist() == [0, 4, 4, 4, 0]
    compare_sim(g, o, label="bad input")


def test_sim_bad_input_found_late(oracle):
    """Inputs are checked as they enter the simulator's window, so a bad entry far down the list is
    found after hundreds of iterations have run and finish times have been written: every output of such
    a scenario must still come out zero, and the scenarios around it untouched.  Entries at window
    boundaries (multiples of 64 and 256) take the path that re-reads the previous arrival."""
    for cap in (8, 200):
        w = W.config5(S=9, N=1500, seed_offset=cap)
        w.out_len[1, 1400] = 0
        w.arrival_us[2, 1024] = w.arrival_us[2, 1023] - 1          # decreasing exactly at a window boundary
        w.arrival_us[3, 641:] -= 5 * 10 ** 6
        w.arrival_us[3, 641:] = np.maximum(w.arrival_us[3, 641:], 0)   # drops below its predecessor at 641
        w.in_len[4, 1499] = -3
        w.arrival_us[5, 768] = -1
        w.arrival_us[6, 1] = w.arrival_us[6, 0] - 1 if w.arrival_us[6, 0] > 0 else -1
        p = dict(w.params, cap=cap)
        say(f"sim bad input found late, cap={cap}")
        o = oracle.online_iter_sim(w.arrival_us, w.in_len, w.out_len, p, 9, 64)
        g = gpu_online_sim(w.arrival_us, w.in_len, w.out_len, p, 9, 64)
        assert o["status"].tolist() == [0, 4, 4, 4, 4, 4, 4, 0, 0]
        compare_sim(g, o, label=f"bad input late cap={cap}")
        assert not g["finish_us"][1:7].any()
    # the assigned simulator: lengths are checked in the pass that fills the queues
    w = W.config5(S=4, N=900)
    assign = (np.arange(4 * 900).reshape(4, 900) % 130).astype(np.int32)
    w.in_len[1, 899] = 0
    w.out_len[2, 450] = -1
    p = dict(w.params, cap=130)
    o = oracle.online_iter_sim_assigned(w.in_len, w.out_len, assign, p)
    g = gpu_online_sim_assigned(w.in_len, w.out_len, assign, p)
    assert o["status"].tolist() == [0, 4, 4, 0]
    compare_sim(g, o, label="assigned bad lengths")


def test_sim_trace_capacity_overflow(oracle):
    w = W.config5(S=3, N=100)
    say("sim trace capacity smaller than the trace")
    o = oracle.online_iter_sim(w.arrival_us, w.in_len, w.out_len, w.params, trace_scenarios=2, trace_capacity=10)
    g = gpu_online_sim(w.arrival_us, w.in_len, w.out_len, w.params, trace_scenarios=2, trace_capacity=10)
    compare_sim(g, o, label="trace overflow")
    assert (g["trace_len"] > 10).all()


def test_sim_config5_full(oracle):
    w = W.config5()
    say("sim config5 full 8192 x 2048 on GPU")
    g = gpu_online_sim(w.arrival_us, w.in_len, w.out_len, w.params, trace_scenarios=4, trace_capacity=8192)
    say("sim config5 oracle, all scenarios")
    o = oracle.online_iter_sim(w.arrival_us, w.in_len, w.out_len, w.params, trace_scenarios=4, trace_capacity=8192)
    compare_sim(g, o, label="c5")


def _same_lb_ex(g, o, label):
    assert g["rc"] == o["rc"], (label, g["rc"], o["rc"])
    if o["rc"] != 0:
        return
    for k in ("status", "lb", "parts"):
        assert np.array_equal(g[k], o[k]), f"{label}: {k} differs: gpu {g[k][:3]} oracle {o[k][:3]}"


def test_lb_ex_parity(oracle):
    """Extended bound: every term (L1, L2, L3 and its k, Lcap, t^p*) and the total, bit for bit."""
    rng = np.random.default_rng(53)
    levels = dict(ncap=[1000, 5000, 2048], tp=[155000, 675000, 300000])
    for (N, M, hi, dtype) in [(1, 1, 10, np.int32), (3, 5, 10, np.int64), (5, 4, 100, np.int32), (9, 8, 3, np.int32),
                              (13, 4, 50, np.int64), (64, 4, 40000, np.int32), (1000, 7, 1 << 20, np.int64),
                              (4097, 16, 1 << 40, np.int64), (5000, 256, 1000, np.int32), (300, 255, 7, np.int32),
                              (16385, 1, 1000, np.int32), (40000, 3, 100000, np.int32), (2000, 2, 0, np.int32)]:
        say(f"lb_ex N={N} M={M}")
        S = 5
        cost = rng.integers(0, hi + 1, size=(S, N)).astype(dtype)
        tok = rng.integers(0, 3000, size=(S, N)).astype(np.int32)
        caps = rng.integers(0, 2 * (N // M + 1) + 1, size=M)
        while caps.sum() < N:
            caps[rng.integers(M)] += N // M + 1
        for kw in (dict(), dict(kmax=1), dict(kmax=3, cap=caps.tolist()), dict(cap=caps.tolist(), prefill_tokens=tok, tp_form=0, **levels),
                   dict(prefill_tokens=tok, tp_form=1, **levels), dict(cap=[N] + [0] * (M - 1))):
            _same_lb_ex(gpu_lower_bound_ex(cost, M, **kw), oracle.lower_bound_ex(cost, M, **kw), f"N={N} M={M} {sorted(kw)}")
    # bad scenarios, bad arguments
    cost = np.array([[3, -1, 4, 2], [1, 2, 3, 4], [5, 5, 5, 5]], np.int64)
    tok = np.array([[1, 1, 1, 1], [1, -1, 1, 1], [2 ** 31 - 1] * 4], np.int32)
    for kw in (dict(), dict(prefill_tokens=tok, ncap=[4], tp=[10]), dict(prefill_tokens=tok, ncap=[1], tp=[2 ** 31 - 1], tp_form=1),
               dict(cap=[1, 2]), dict(cap=[-1, 9])):
        _same_lb_ex(gpu_lower_bound_ex(cost, 2, **kw), oracle.lower_bound_ex(cost, 2, **kw), f"bad inputs {sorted(kw)}")
    o = oracle.lower_bound_ex(cost, 2, prefill_tokens=tok, ncap=[4], tp=[10])
    assert o["status"].tolist() == [3, 3, 0]


def test_lb_ex_hand_worked_and_configs(oracle):
    from test_oracle_lb_sim import _lb_ex_cases
    for c in _lb_ex_cases():
        kw = {}
        if c["levels"]:
            kw = dict(prefill_tokens=np.array([c["tokens"]], np.int32), ncap=[l[0] for l in c["levels"]],
                      tp=[l[1] for l in c["levels"]], tp_form=c["tp_form"])
        g = gpu_lower_bound_ex(np.array([c["cost"]], np.int64), c["M"], cap=c["caps"], kmax=c["kmax"], **kw)
        assert g["rc"] == 0 and g["parts"][0].tolist() == c["parts"] and int(g["lb"][0]) == c["lb"], c["name"]
    for c in (W.config1(), W.config2(), W.config3(S=256), W.config4()):
        say(f"lb_ex config {c.name}")
        caps = [c.cap] * c.M
        o = oracle.lower_bound_ex(c.cost, c.M, cap=caps)
        _same_lb_ex(gpu_lower_bound_ex(c.cost, c.M, cap=caps), o, c.name)
        basic = oracle.lower_bound(c.cost, c.M)
        assert (o["lb"] >= basic["lb"]).all()


# ------------------------------------------------------------------ longest-processing-time start
def _same_lpt(g, o, label):
    assert g["rc"] == o["rc"], (label, g["rc"], o["rc"])
    if o["rc"] == 0:
        for k in ("status", "order", "assign", "load"):
            assert np.array_equal(g[k], o[k]), f"{label}: {k} differs"


def test_lpt_start_parity(oracle):
    from test_oracle_lpt import _cases
    for c in _cases():
        g = gpu_lpt_start(np.array([c["cost"]], np.int64), c["M"], c["cap"])
        assert g["rc"] == 0 and g["order"][0].tolist() == c["order"] and g["assign"][0].tolist() == c["assign"] \
            and g["load"][0].tolist() == c["load"], c["name"]
    rng = np.random.default_rng(71)
    for (N, M, cap, hi, dtype) in [(1, 1, 1, 10, np.int32), (2, 3, 1, 10, np.int64), (5, 5, 1, 50, np.int32), (64, 4, 16, 40000, np.int32),
                                   (65, 3, 30, 3, np.int32), (100, 7, 15, 2000, np.int64), (257, 9, 33, 700, np.int32),
                                   (1319, 200, 7, 60000, np.int32), (4096, 16, 256, 700000, np.int64), (3000, 256, 12, 40000, np.int32),
                                   (1000, 70, 1000, 0, np.int32), (16384, 64, 256, 1 << 20, np.int32), (9000, 5, 1800, 1 << 30, np.int64),
                                   (700, 6, 200, 1 << 50, np.int64), (513, 130, 4, 1 << 50, np.int64)]:
        say(f"lpt N={N} M={M} cap={cap} hi={hi}")
        S = 3
        cost = rng.integers(0, hi + 1, size=(S, N)).astype(dtype)
        if hi >= 1 << 50:
            # a few costs too large to pack beside an index (the ranking path), some of them equal: the index decides
            cost[:, 5:13] = (1 << 57) + rng.integers(0, 3, size=(S, 8))
            cost[:, 100:120] = cost[:, 300:320]
        _same_lpt(gpu_lpt_start(cost, M, cap), oracle.lpt_start(cost, M, cap), f"N={N} M={M}")
    cost = np.array([[5, 3, 2, 1], [5, -3, 2, 1], [1 << 61, 1 << 61, 1, 1]], np.int64)
    _same_lpt(gpu_lpt_start(cost, 2, 2), oracle.lpt_start(cost, 2, 2), "bad cost")
    assert gpu_lpt_start(cost, 2, 1)["rc"] == -2


def test_lpt_start_feeds_the_local_search(oracle):
    """The start is feasible for mmbp_local_search, and the search from it ends no worse than it started."""
    for c in (W.config2(S=32), W.config3(S=8)):
        say(f"lpt -> local search {c.name}")
        o = oracle.lpt_start(c.cost, c.M, c.cap)
        g = gpu_lpt_start(c.cost, c.M, c.cap)
        _same_lpt(g, o, c.name)
        ol = oracle.local_search(c.cost, o["assign"], c.M, c.cap, 50, want_log=True)
        gl = gpu_local_search(c.cost, g["assign"], c.M, c.cap, 50)
        compare_ls(gl, ol, label=f"search from the LPT start, {c.name}")
        assert (gl["makespan"] <= g["load"].max(axis=1)).all()
        rr = oracle.local_search(c.cost, c.assign0, c.M, c.cap, 0)
        assert (g["load"].max(axis=1) <= rr["makespan"]).all()      # on these inputs LPT starts below round-robin


# ------------------------------------------------------------------ simulator fed by an offline assignment
def test_sim_assigned_hand_worked_cases(oracle):
    for (cap, pol, inl, outl, asg) in [(2, 0, [10, 20, 5, 8], [3, 2, 4, 1], [0, 0, 0, 1]),
                                       (3, 1, [4, 6, 5, 3, 2, 2], [2, 3, 2, 3, 2, 1], [0, 1, 1, 2, 2, 2])]:
        p = dict(cap=cap, a_prefill=1, b_decode=10, c_prefill=5, c_decode=2, max_prefill_tokens=0, policy=pol)
        a, b, c = np.array([inl], np.int32), np.array([outl], np.int32), np.array([asg], np.int32)
        say(f"sim assigned hand-worked cap={cap}")
        compare_sim(gpu_online_sim_assigned(a, b, c, p, 1, 32), oracle.online_iter_sim_assigned(a, b, c, p, 1, 32),
                    label=f"assigned hand-worked cap={cap}")


@pytest.mark.parametrize("policy", [0, 1, 2])
def test_sim_assigned_random(oracle, policy):
    rng = np.random.default_rng(300 + policy)
    for (S, N, cap, tok) in [(7, 1, 1, 0), (7, 5, 3, 0), (6, 180, 7, 0), (6, 180, 7, 700), (5, 400, 64, 0), (4, 1000, 33, 3000),
                             (3, 64, 64, 0)]:
        w = W.config5(S=S, N=N, seed_offset=N + cap + policy)
        assign = rng.integers(0, cap, (S, N)).astype(np.int32)
        assign[0] = np.arange(N) % cap
        if S > 1:
            assign[1] = np.minimum(np.arange(N) // max(N // 3, 1), cap - 1)      # few loaded clients, the others steal
        if S > 2:
            assign[2] = 0                                                       # one queue, everybody else steals
        p = dict(w.params, cap=cap, max_prefill_tokens=tok, policy=policy)
        say(f"sim assigned policy={policy} N={N} cap={cap} tok={tok}")
        o = oracle.online_iter_sim_assigned(w.in_len, w.out_len, assign, p, S, 4 * N + 8)
        g = gpu_online_sim_assigned(w.in_len, w.out_len, assign, p, S, 4 * N + 8)
        compare_sim(g, o, label=f"assigned policy={policy} N={N} cap={cap}")


def test_sim_assigned_equal_lengths_and_bad_input(oracle):
    S, N, cap = 4, 200, 16
    inl = np.full((S, N), 50, np.int32)
    outl = np.full((S, N), 20, np.int32)            # all lengths equal: ties everywhere (index order, lowest client)
    assign = (np.arange(S * N).reshape(S, N) * 7 % cap).astype(np.int32)
    assign[3, :150] = 2
    p = dict(W.C5_PARAMS, cap=cap)
    say("sim assigned equal lengths")
    compare_sim(gpu_online_sim_assigned(inl, outl, assign, p, S, 900), oracle.online_iter_sim_assigned(inl, outl, assign, p, S, 900),
                label="assigned equal lengths")
    bad = assign.copy()
    bad[1, 7] = cap
    bad[2, 0] = -1
    inl2 = inl.copy(); inl2[3, 5] = 0
    say("sim assigned bad input")
    o = oracle.online_iter_sim_assigned(inl2, outl, bad, p)
    assert o["status"].tolist() == [0, 4, 4, 4]
    compare_sim(gpu_online_sim_assigned(inl2, outl, bad, p), o, label="assigned bad input")


def test_hybrid_pipeline_offline_search_then_assigned_sim(oracle):
    """The paper's offline + online combination on synthetic requests: the local search balances the
    estimated costs over cap clients, the assigned simulator runs the result."""
    S, N, cap = 64, 2048, 64
    w = W.config5(S=S, N=N)
    cost = W.job_cost(w.in_len, w.out_len, np.int32)
    assign0 = np.tile((np.arange(N) % cap).astype(np.int32), (S, 1))
    say("hybrid: local search M=64")
    ls = gpu_local_search(cost, assign0, cap, N, 300, want_log=False)
    assert (ls["status"] <= 1).all()
    say("hybrid: assigned simulator")
    p = dict(w.params, cap=cap)
    o = oracle.online_iter_sim_assigned(w.in_len, w.out_len, ls["assign"], p, 2, 8192)
    g = gpu_online_sim_assigned(w.in_len, w.out_len, ls["assign"], p, 2, 8192)
    compare_sim(g, o, label="hybrid")


_HYB = {}


def _hybrid_on_gpu():
    """The hybrid leg as the benchmark runs it, computed once: 2048 scenarios x 2048 requests on 64 clients, pruned
    search from round-robin (limit 1024 passes) in ONE call, then the assigned simulator on its result."""
    if not _HYB:
        w = W.config5()
        S, N, cap = 2048, w.N, w.params["cap"]
        in_len, out_len = w.in_len[:S], w.out_len[:S]
        cost = W.job_cost(in_len, out_len, np.int32)
        assign0 = np.tile((np.arange(N) % cap).astype(np.int32), (S, 1))
        say("hybrid at the benchmark size: pruned search and assigned simulator on GPU")
        g = gpu_local_search(cost, assign0, cap, N, 1024, pruned=True)
        p = dict(w.params, cap=cap)
        _HYB.update(in_len=in_len, out_len=out_len, cost=cost, assign0=assign0, cap=cap, N=N, p=p, g=g,
                    sim=gpu_online_sim_assigned(in_len, out_len, g["assign"], p))
    return _HYB


@pytest.mark.parametrize("part", range(4))
def test_hybrid_pipeline_at_the_benchmark_size(oracle, part):
    """Every output of both steps against the oracle (scenarios are independent: four slices of 512)."""
    h = _hybrid_on_gpu()
    sl = slice(512 * part, 512 * (part + 1))
    say(f"hybrid at the benchmark size: oracle on scenarios {sl.start}..{sl.stop - 1}")
    o = oracle.local_search(h["cost"][sl], h["assign0"][sl], h["cap"], h["N"], 1024, want_log=True)
    compare_ls({k: (v[sl] if isinstance(v, np.ndarray) else v) for k, v in h["g"].items()}, o, label=f"hybrid pruned search, slice {part}")
    osim = oracle.online_iter_sim_assigned(h["in_len"][sl], h["out_len"][sl], o["assign"], h["p"], 0, 0)
    compare_sim({k: (v[sl] if isinstance(v, np.ndarray) else v) for k, v in h["sim"].items()}, osim, label=f"hybrid assigned simulator, slice {part}")


def test_paper_shaped_pipeline_at_the_benchmark_size(oracle):
    """The paper-shaped leg as the benchmark runs it: 1024 scenarios x 1319 requests on 200 clients of at most 7,
    LPT start, pruned search, assigned simulator, and the FCFS simulator under the rule and the baseline."""
    in_len, out_len = W.paper_shaped(S=1024)
    S, N = in_len.shape
    p = dict(W.PAPER_PARAMS)
    M = p["cap"]
    cap = -(-N // M)
    cost = W.job_cost(in_len, out_len, np.int32)
    say("paper-shaped at the benchmark size: LPT start")
    lg, lo = gpu_lpt_start(cost, M, cap), oracle.lpt_start(cost, M, cap)
    _same_lpt(lg, lo, "paper-shaped LPT, benchmark size")
    say("paper-shaped at the benchmark size: pruned search")
    g = gpu_local_search(cost, lg["assign"], M, cap, 1024, pruned=True)
    o = oracle.local_search(cost, lo["assign"].astype(np.int32), M, cap, 1024, want_log=True)
    compare_ls(g, o, label="paper-shaped pruned search, benchmark size")
    say("paper-shaped at the benchmark size: simulators")
    compare_sim(gpu_online_sim_assigned(in_len, out_len, g["assign"], p), oracle.online_iter_sim_assigned(in_len, out_len, o["assign"], p, 0, 0),
                label="paper-shaped assigned simulator, benchmark size")
    arr = np.zeros((S, N), np.int64)
    for pol in (0, 2):
        pp = dict(p, policy=pol)
        compare_sim(gpu_online_sim(arr, in_len, out_len, pp), oracle.online_iter_sim(arr, in_len, out_len, pp, 0, 0),
                    label=f"paper-shaped FCFS policy {pol}, benchmark size")


# ------------------------------------------------------------------ more clients than one wave has lanes
@pytest.mark.parametrize("policy", [0, 1, 2])
def test_sim_many_clients(oracle, policy):
    """Batch sizes above 64 (up to the limit of 256): several client slots per lane."""
    rng = np.random.default_rng(400 + policy)
    for (S, N, cap, tok, rate) in [(5, 300, 65, 0, 400.0), (5, 700, 100, 0, 2000.0), (4, 900, 128, 5000, 3000.0),
                                   (4, 900, 129, 0, 50.0), (4, 1319, 200, 0, 1e9), (3, 2500, 256, 9000, 5000.0),
                                   (3, 600, 256, 300, 1e9)]:
        w = W.config5(S=S, N=N, rate_per_s=rate, seed_offset=N + cap + policy)
        p = dict(w.params, cap=cap, max_prefill_tokens=tok, policy=policy)
        say(f"sim many clients policy={policy} N={N} cap={cap} tok={tok} rate={rate}")
        o = oracle.online_iter_sim(w.arrival_us, w.in_len, w.out_len, p, S, 6 * N + 8)
        g = gpu_online_sim(w.arrival_us, w.in_len, w.out_len, p, S, 6 * N + 8)
        compare_sim(g, o, label=f"many clients policy={policy} N={N} cap={cap}")


def test_sim_paper_shaped_200_clients(oracle):
    """The paper's own shape (Table "Experiment Settings": 1319 requests, 200 clients, its time model),
    lengths drawn from its printed means and deviations: FCFS simulator with all requests at t = 0, and the
    offline assignment (local search over 200 clients) run through the sorted queues with stealing."""
    in_len, out_len = W.paper_shaped(S=12)
    S, N = in_len.shape
    p = dict(W.PAPER_PARAMS)
    arr = np.zeros((S, N), np.int64)
    say("paper-shaped FCFS, cap 200")
    for pol in (0, 1, 2):
        pp = dict(p, policy=pol)
        compare_sim(gpu_online_sim(arr, in_len, out_len, pp, 2, 4096), oracle.online_iter_sim(arr, in_len, out_len, pp, 2, 4096),
                    label=f"paper-shaped fcfs policy {pol}")
    cost = W.job_cost(in_len, out_len, np.int32)
    M = p["cap"]
    cap = -(-N // M)
    a0 = np.tile((np.arange(N) % M).astype(np.int32), (S, 1))
    say("paper-shaped: local search over 200 clients, then the assigned simulator")
    ls = gpu_local_search(cost, a0, M, cap + 2, 400, want_log=True)
    ols = oracle.local_search(cost, a0, M, cap + 2, 400, want_log=True)
    compare_ls(ls, ols, label="paper-shaped local search")
    # the pruned scan of this shape fits one workgroup (no tile tables), with or without a workspace
    compare_ls(gpu_local_search(cost, a0, M, cap + 2, 400, pruned=True), ols, label="paper-shaped pruned search")
    compare_ls(gpu_local_search(cost, a0, M, cap + 2, 400, pruned=True, use_workspace=False), ols,
               label="paper-shaped pruned search, no workspace")
    for pol in (0, 1):
        pp = dict(p, policy=pol)
        o = oracle.online_iter_sim_assigned(in_len, out_len, ls["assign"], pp, 2, 4096)
        g = gpu_online_sim_assigned(in_len, out_len, ls["assign"], pp, 2, 4096)
        compare_sim(g, o, label=f"paper-shaped assigned policy {pol}")


@pytest.mark.parametrize("policy", [0, 1, 2])
def test_sim_assigned_many_clients(oracle, policy):
    rng = np.random.default_rng(500 + policy)
    for (S, N, cap, tok) in [(6, 300, 65, 0), (6, 500, 130, 0), (5, 1319, 200, 0), (5, 1319, 200, 900), (4, 2000, 256, 0),
                             (4, 256, 256, 0), (4, 100, 200, 150)]:
        w = W.config5(S=S, N=N, seed_offset=N + cap + policy)
        assign = rng.integers(0, cap, (S, N)).astype(np.int32)
        assign[0] = np.arange(N) % cap
        assign[1] = np.minimum(np.arange(N) // max(N // 3, 1), cap - 1)      # few loaded clients, the others steal
        assign[2] = cap - 1                                                  # one queue on the last client
        assign[3] = (np.arange(N) * 7 % 3) * 64 % cap                       # queues on clients 0, 64, 128 (one per register block)
        p = dict(w.params, cap=cap, max_prefill_tokens=tok, policy=policy)
        say(f"sim assigned many clients policy={policy} N={N} cap={cap} tok={tok}")
        o = oracle.online_iter_sim_assigned(w.in_len, w.out_len, assign, p, S, 4 * N + 8)
        g = gpu_online_sim_assigned(w.in_len, w.out_len, assign, p, S, 4 * N + 8)
        compare_sim(g, o, label=f"assigned many clients policy={policy} N={N} cap={cap}")


@pytest.mark.parametrize("cap", [64, 130, 256])
def test_sim_assigned_maximum_size(oracle, cap):
    """The largest request count the assigned simulator takes (its queues need more LDS than the
    default limit of a launch there), for one, two and four clients per lane."""
    N, S = 8192, 2
    rng = np.random.default_rng(97 + cap)
    w = W.config5(S=S, N=N, seed_offset=cap)
    assign = rng.integers(0, cap, size=(S, N)).astype(np.int32)
    assign[1] = np.minimum(assign[1], cap // 3)                             # idle clients from the start: stealing
    in_len = w.in_len.copy()
    if cap != 64:
        in_len[1, ::1500] = 70000 + np.arange(len(in_len[1, ::1500]))       # input lengths beyond 16 bits in one scenario
    w.in_len = in_len
    p = dict(w.params, cap=cap, max_prefill_tokens=3000)
    say(f"sim assigned maximum size N={N} cap={cap}")
    o = oracle.online_iter_sim_assigned(w.in_len, w.out_len, assign, p, S, 4 * N + 8)
    g = gpu_online_sim_assigned(w.in_len, w.out_len, assign, p, S, 4 * N + 8)
    compare_sim(g, o, label=f"assigned maximum size cap={cap}")


@pytest.mark.parametrize("cap,N", [(6, 48), (70, 210)])
def test_sim_assigned_large_remain_token(oracle, cap, N):
    """Queues whose remain_token exceeds 24 bits: a steal then compares the 64-bit sums themselves (the
    kernel packs sum and client into one 32-bit key only while every sum is small), and the decode runs are
    longer than 16 bits of count, so their records take the byte-by-byte hash."""
    S = 3
    rng = np.random.default_rng(1234 + cap)
    in_len = rng.integers(1, 3000, size=(S, N)).astype(np.int32)
    out_len = rng.integers(1 << 20, 1 << 22, size=(S, N)).astype(np.int32)
    out_len[2, ::2] = rng.integers(1, 50, size=len(out_len[2, ::2]))       # a scenario that mixes short and long
    assign = rng.integers(0, max(cap // 3, 1), size=(S, N)).astype(np.int32)    # most clients start idle: stealing
    assign[1] = rng.integers(0, cap, size=N)
    p = dict(cap=cap, a_prefill=130, b_decode=210, c_prefill=25000, c_decode=29000, max_prefill_tokens=4096, policy=0)
    say(f"sim assigned large remain_token cap={cap} N={N}")
    o = oracle.online_iter_sim_assigned(in_len, out_len, assign, p, S, 6 * N + 8)
    g = gpu_online_sim_assigned(in_len, out_len, assign, p, S, 6 * N + 8)
    compare_sim(g, o, label=f"assigned large remain_token cap={cap}")


@pytest.mark.parametrize("b_decode", [0, 1, 7])
def test_sim_prefill_waits_many_iterations(oracle, b_decode):
    """A small decode slope against a large prefill constant: C_d needs hundreds of decode iterations
    to pass C_p (never, with slope 0: then the prefill waits until nothing runs).  The kernels apply such
    a wait in one step, bounded by the next finish and, in the FCFS simulator, by the next arrival that
    could join the prefill; finish times, counters and the run-length trace must not change."""
    S, N = 6, 400
    for cap, rate, tok in ((8, 20, 0), (64, 200, 500), (200, 2000, 0)):
        w = W.config5(S=S, N=N, rate_per_s=rate, seed_offset=cap + b_decode)
        p = dict(cap=cap, a_prefill=3, b_decode=b_decode, c_prefill=40000, c_decode=900, max_prefill_tokens=tok, policy=0)
        say(f"sim long waits b_decode={b_decode} cap={cap} rate={rate}")
        o = oracle.online_iter_sim(w.arrival_us, w.in_len, w.out_len, p, S, 6 * N + 8)
        g = gpu_online_sim(w.arrival_us, w.in_len, w.out_len, p, S, 6 * N + 8)
        compare_sim(g, o, label=f"long waits b={b_decode} cap={cap}")
        assign = (np.arange(N)[None, :] * 7 % max(cap // 2, 1)).astype(np.int32).repeat(S, axis=0)
        o = oracle.online_iter_sim_assigned(w.in_len, w.out_len, assign, p, S, 6 * N + 8)
        g = gpu_online_sim_assigned(w.in_len, w.out_len, assign, p, S, 6 * N + 8)
        compare_sim(g, o, label=f"assigned, long waits b={b_decode} cap={cap}")
