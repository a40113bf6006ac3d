"""Pins for the CPU oracle's local search (no GPU).

The C oracle is checked against things other than itself: hand-worked examples
(tests/golden/ls_hand_worked.txt), a definition-level recomputation of every candidate,
brute-force enumeration of all assignments, and invariants of the MMBP model
(paper section "Offline requests scheduling & theoretical lower bound").
"""
import os

import numpy as np
import pytest

from oracle import definition as D
from paper_2502_15763_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "ls_hand_worked.txt")


def _ints(s):
    s = s.strip()
    return [] if s in ("", "-") else [int(x) for x in s.split()]


def _golden_cases():
    cases = []
    with open(GOLD) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            p = [x.strip() for x in line.split("|")]
            cases.append(dict(name=p[0], M=int(p[1]), cap=int(p[2]), cost=_ints(p[3]), assign0=_ints(p[4]),
                              max_passes=int(p[5]), log=_ints(p[6]), assign=_ints(p[7]), load=_ints(p[8]),
                              passes=int(p[9]), evals=int(p[10]), status=int(p[11])))
    return cases


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c["name"])
def test_hand_worked_examples(oracle, case):
    cost = np.array([case["cost"]], np.int64)
    a0 = np.array([case["assign0"]], np.int32)
    r = oracle.local_search(cost, a0, case["M"], case["cap"], case["max_passes"], want_log=True)
    assert r["rc"] == 0
    assert r["assign"][0].tolist() == case["assign"]
    assert r["load"][0].tolist() == case["load"]
    assert int(r["makespan"][0]) == max(case["load"])
    assert int(r["passes"][0]) == case["passes"]
    assert int(r["evals"][0]) == case["evals"]
    assert int(r["status"][0]) == case["status"]
    assert r["log"][0][: case["passes"]].tolist() == case["log"]
    # the definition-level implementation must reproduce the same hand-worked numbers
    d = D.local_search(case["cost"], case["assign0"], case["M"], case["cap"], case["max_passes"])
    assert d["assign"] == case["assign"] and d["log"] == case["log"] and d["evals"] == case["evals"]


@pytest.mark.parametrize("mode", [0, 1], ids=["threads_over_scenarios", "threads_inside_scan"])
@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c["name"])
def test_hand_worked_examples_both_threadings(oracle, case, mode):
    """The oracle runs its swap scan either serially (threads over scenarios) or split over threads
    (one scenario at a time); each way is held to the hand-worked numbers, whatever the host's core
    count would have picked."""
    cost = np.array([case["cost"]], np.int64)
    a0 = np.array([case["assign0"]], np.int32)
    r = oracle.local_search(cost, a0, case["M"], case["cap"], case["max_passes"], want_log=True, mode=mode)
    assert r["rc"] == 0
    assert r["assign"][0].tolist() == case["assign"]
    assert r["load"][0].tolist() == case["load"]
    assert int(r["passes"][0]) == case["passes"]
    assert int(r["evals"][0]) == case["evals"]
    assert int(r["status"][0]) == case["status"]
    assert r["log"][0][: case["passes"]].tolist() == case["log"]


@pytest.mark.parametrize("mode", [0, 1], ids=["threads_over_scenarios", "threads_inside_scan"])
@pytest.mark.parametrize("N,M,cap", [(6, 2, 3), (7, 3, 3), (9, 3, 4), (8, 4, 2), (10, 4, 10), (5, 5, 1),
                                     (12, 3, 6), (16, 4, 5)])
def test_delta_formula_equals_recomputation(oracle, N, M, cap, mode):
    rng = np.random.default_rng(100 + N * 10 + M)
    for trial in range(12):
        cost, assign = W.random_offline(rng, 1, N, M, cap, cost_hi=[30, 1000, 3][trial % 3])
        r = oracle.local_search(cost, assign, M, cap, 50, want_log=True, mode=mode)
        d = D.local_search(cost[0], assign[0], M, cap, 50)
        p = int(r["passes"][0])
        assert p == d["passes"]
        assert r["log"][0][:p].tolist() == d["log"]
        assert r["assign"][0].tolist() == d["assign"]
        assert r["load"][0].tolist() == d["load"]
        assert int(r["evals"][0]) == d["evals"]
        assert int(r["status"][0]) == d["status"]


def test_brute_force_sandwich(oracle):
    """LB <= OPT <= LS <= start, OPT by enumeration of all M^N assignments."""
    rng = np.random.default_rng(7)
    for N, M, cap in [(6, 2, 3), (6, 2, 6), (7, 3, 3), (8, 3, 4), (9, 3, 3), (8, 4, 2), (10, 4, 3), (5, 4, 5)]:
        for trial in range(6):
            cost, assign = W.random_offline(rng, 1, N, M, cap, cost_hi=50)
            opt = oracle.brute_force_opt(cost[0], M, cap)
            if N <= 8:
                assert opt == D.brute_force_opt(cost[0].tolist(), M, cap)
            r = oracle.local_search(cost, assign, M, cap, 1000)
            lb = int(oracle.lower_bound(cost, M)["lb"][0])
            start = D.makespan_of(cost[0], assign[0], M)
            assert lb <= opt <= int(r["makespan"][0]) <= start


def test_lower_bound_can_be_strict_and_tight(oracle):
    # three equal jobs on two clients: LB = max(ceil(9/2)=5, 3, 3+3=6) = 6 = OPT
    cost = np.array([[3, 3, 3]], np.int64)
    assert int(oracle.lower_bound(cost, 2)["lb"][0]) == 6
    assert oracle.brute_force_opt(cost[0], 2, 3) == 6


def _check_invariants(oracle, cost, assign0, M, cap, r):
    S, N = cost.shape
    for s in range(S):
        a = r["assign"][s]
        assert a.min() >= 0 and a.max() < M
        cnt = np.bincount(a, minlength=M)
        assert cnt.max() <= cap
        load = np.bincount(a, weights=cost[s].astype(np.float64), minlength=M).astype(np.int64)
        assert load.tolist() == r["load"][s].tolist()
        assert int(load.sum()) == int(cost[s].sum())
        assert int(r["makespan"][s]) == int(load.max())
        assert int(r["makespan"][s]) <= D.makespan_of(cost[s], assign0[s], M)


def test_invariants_and_local_optimum(oracle):
    rng = np.random.default_rng(11)
    for N, M, cap in [(40, 4, 10), (40, 4, 13), (33, 5, 9), (64, 8, 8), (50, 3, 50), (20, 20, 1), (17, 1, 17)]:
        cost, assign = W.random_offline(rng, 3, N, M, cap, cost_hi=500)
        r = oracle.local_search(cost, assign, M, cap, 10000, want_log=True)
        assert (r["status"] == 0).all()
        _check_invariants(oracle, cost, assign, M, cap, r)
        for s in range(3):
            # converged => the definition-level scan finds nothing strictly better
            best, _, _ = D.scan(cost[s].tolist(), r["assign"][s].tolist(), M, cap)
            assert best is None or best[0] >= int(r["makespan"][s])


def test_strict_decrease_and_resumability(oracle):
    rng = np.random.default_rng(13)
    cost, assign = W.random_offline(rng, 4, 48, 4, 14, cost_hi=900)
    full = oracle.local_search(cost, assign, 4, 14, 10000, want_log=True)
    # makespan after k passes strictly decreases in k
    prev = None
    for k in range(0, int(full["passes"].max()) + 2):
        rk = oracle.local_search(cost, assign, 4, 14, k)
        if prev is not None:
            for s in range(4):
                if k <= int(full["passes"][s]):
                    assert rk["makespan"][s] < prev["makespan"][s]
                else:
                    assert rk["makespan"][s] == prev["makespan"][s]
        prev = rk
    # k passes then k more == 2k passes
    k = 2
    r1 = oracle.local_search(cost, assign, 4, 14, k)
    r2 = oracle.local_search(cost, r1["assign"], 4, 14, k)
    r12 = oracle.local_search(cost, assign, 4, 14, 2 * k)
    assert (r2["assign"] == r12["assign"]).all() and (r2["load"] == r12["load"]).all()
    assert ((r1["passes"] + r2["passes"]) == r12["passes"]).all()


def test_cost_scaling_metamorphic(oracle):
    rng = np.random.default_rng(17)
    cost, assign = W.random_offline(rng, 3, 36, 3, 13, cost_hi=200)
    r1 = oracle.local_search(cost, assign, 3, 13, 1000, want_log=True)
    r7 = oracle.local_search(cost * 7, assign, 3, 13, 1000, want_log=True)
    assert (r1["assign"] == r7["assign"]).all()
    assert (r1["load"] * 7 == r7["load"]).all()
    assert (r1["log"] == r7["log"]).all()


def test_degenerate_cases(oracle):
    # M = 1: no candidates at all
    r = oracle.local_search(np.array([[4, 5, 6]], np.int64), np.zeros((1, 3), np.int32), 1, 3, 10)
    assert int(r["passes"][0]) == 0 and int(r["evals"][0]) == 0 and int(r["makespan"][0]) == 15
    # N = 1: moving the only job never lowers the makespan
    r = oracle.local_search(np.array([[9]], np.int64), np.zeros((1, 1), np.int32), 3, 1, 10)
    assert int(r["passes"][0]) == 0 and int(r["evals"][0]) == 2 and int(r["makespan"][0]) == 9
    # all-equal costs, balanced: already optimal
    r = oracle.local_search(np.full((1, 8), 5, np.int64), (np.arange(8, dtype=np.int32) % 4)[None], 4, 2, 10)
    assert int(r["passes"][0]) == 0 and int(r["makespan"][0]) == 10
    # two clients tied for the maximum: a swap between exactly those two can still improve
    cost = np.array([[6, 1, 1, 6, 3]], np.int64)
    assign = np.array([[0, 0, 1, 1, 2]], np.int32)     # loads 7,7,3
    r = oracle.local_search(cost, assign, 3, 2, 10, want_log=True)
    d = D.local_search(cost[0], assign[0], 3, 2, 10)
    assert r["assign"][0].tolist() == d["assign"] and int(r["passes"][0]) == d["passes"]
    # zero costs
    r = oracle.local_search(np.zeros((1, 6), np.int64), (np.arange(6, dtype=np.int32) % 2)[None], 2, 3, 10)
    assert int(r["passes"][0]) == 0 and int(r["makespan"][0]) == 0


def test_status_and_return_codes(oracle):
    cost = np.array([[5, 3, 2, 1], [5, 3, 2, 1], [5, -3, 2, 1], [5, 3, 2, 1]], np.int64)
    assign = np.array([[0, 0, 1, 1], [0, 0, 2, 1], [0, 0, 1, 1], [0, 0, 0, 1]], np.int32)
    r = oracle.local_search(cost, assign, 2, 2, 10)
    assert r["rc"] == 0
    assert r["status"].tolist() == [0, 2, 3, 2]
    for s in (1, 2, 3):                      # bad scenarios are left untouched
        assert r["assign"][s].tolist() == assign[s].tolist()
        assert r["load"][s].tolist() == [0, 0] and int(r["makespan"][s]) == 0 and int(r["passes"][s]) == 0
    big = np.array([[1 << 61, 1 << 61, 1, 1]], np.int64)
    assert oracle.local_search(big, assign[:1], 2, 2, 10)["status"].tolist() == [3]
    assert oracle.local_search(cost[:1], assign[:1], 2, 1, 10)["rc"] == -2      # N > M*cap
    assert oracle.local_search(cost[:1], assign[:1], 2, 0, 10)["rc"] == -1
    assert oracle.local_search(cost[:1], assign[:1], 0, 2, 10)["rc"] == -1
    assert oracle.local_search(cost[:1], assign[:1], 2, 2, -1)["rc"] == -1


def test_config1_shape_and_tight_capacity(oracle):
    c = W.config1()
    assert (c.S, c.N, c.M, c.cap) == (1, 64, 4, 16)
    r = oracle.local_search(c.cost, c.assign0, c.M, c.cap, c.max_passes, want_log=True)
    assert int(r["status"][0]) == 0
    # tight capacity: every applied candidate is a swap, and evals per scan is constant
    p = int(r["passes"][0])
    assert (r["log"][0][:p] >= c.N * c.M).all()
    per_scan = c.N * (c.M - 1) + (c.N * c.N - c.M * 16 * 16) // 2
    assert int(r["evals"][0]) == per_scan * (p + 1)
    lb = int(oracle.lower_bound(c.cost, c.M)["lb"][0])
    assert lb <= int(r["makespan"][0])


@pytest.mark.parametrize("mode", [0, 1], ids=["threads_over_scenarios", "threads_inside_scan"])
def test_batch_of_scenarios_both_threadings(oracle, mode):
    """A batch larger than any host's thread count (so neither threading is chosen by accident),
    with rows long enough that the split scan really hands rows to several threads (its chunks are
    64 rows): every scenario against the definition-level search, pass by pass."""
    rng = np.random.default_rng(4242)
    S, N, M, cap = 40, 130, 4, 40
    cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=60)
    r = oracle.local_search(cost, assign, M, cap, 4, want_log=True, mode=mode)
    assert r["rc"] == 0
    for s in range(0, S, 8):
        d = D.local_search(cost[s], assign[s], M, cap, 4)
        p = int(r["passes"][s])
        assert p == d["passes"] and r["log"][s][:p].tolist() == d["log"]
        assert r["assign"][s].tolist() == d["assign"] and r["load"][s].tolist() == d["load"]
        assert int(r["evals"][s]) == d["evals"] and int(r["status"][s]) == d["status"]


def test_bad_mode_is_rejected(oracle):
    cost = np.array([[5, 3, 2, 1]], np.int64)
    assign = np.array([[0, 0, 1, 1]], np.int32)
    assert oracle.local_search(cost, assign, 2, 2, 10, mode=2)["rc"] == -1
