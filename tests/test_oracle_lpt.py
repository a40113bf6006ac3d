"""Pins for the CPU oracle's longest-processing-time start (no GPU): hand-worked runs, the
classical approximation guarantee against brute force, and feasibility under the cardinality limit."""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "lpt_hand_worked.txt")


def _cases():
    out = []
    ints = lambda t: [int(x) for x in t.split()]
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        p = [x.strip() for x in line.split("|")]
        out.append(dict(name=p[0], M=int(p[1]), cap=int(p[2]), cost=ints(p[3]), order=ints(p[4]), assign=ints(p[5]),
                        load=ints(p[6])))
    return out


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_lpt_hand_worked(oracle, case):
    r = oracle.lpt_start(np.array([case["cost"]], np.int64), case["M"], case["cap"])
    assert r["rc"] == 0 and int(r["status"][0]) == 0
    assert r["order"][0].tolist() == case["order"]
    assert r["assign"][0].tolist() == case["assign"]
    assert r["load"][0].tolist() == case["load"]


def test_lpt_guarantee_against_brute_force(oracle):
    """LB <= OPT <= LPT <= (4/3 - 1/(3M)) OPT when the cardinality limit does not bind."""
    rng = np.random.default_rng(61)
    for N, M in [(5, 2), (7, 2), (8, 3), (9, 3), (9, 4), (10, 4)]:
        for _ in range(12):
            c = rng.integers(1, 40, size=(1, N)).astype(np.int64)
            r = oracle.lpt_start(c, M, N)
            mk = int(r["load"][0].max())
            opt = oracle.brute_force_opt(c[0], M, N)
            lb = int(oracle.lower_bound_ex(c, M)["lb"][0])
            assert lb <= opt <= mk
            assert Fraction(mk) <= (Fraction(4, 3) - Fraction(1, 3 * M)) * opt, (c, mk, opt)


def test_lpt_feasible_and_consistent_under_tight_caps(oracle):
    rng = np.random.default_rng(67)
    for N, M, cap in [(12, 3, 4), (13, 4, 4), (40, 8, 5), (64, 4, 16), (100, 7, 15), (9, 9, 1)]:
        c = rng.integers(0, 1000, size=(4, N)).astype(np.int64)
        r = oracle.lpt_start(c, M, cap)
        assert r["rc"] == 0 and (r["status"] == 0).all()
        for s in range(4):
            a = r["assign"][s]
            assert a.min() >= 0 and a.max() < M and np.bincount(a, minlength=M).max() <= cap
            load = np.bincount(a, weights=c[s].astype(np.float64), minlength=M).astype(np.int64)
            assert load.tolist() == r["load"][s].tolist()
            o = r["order"][s]
            assert sorted(o.tolist()) == list(range(N))
            keys = [(-int(c[s][i]), int(i)) for i in o]
            assert keys == sorted(keys)                  # decreasing cost, equal costs by index
            if cap * M > N + M:                          # slack caps: the result is at least as good as any single-client pile
                assert load.max() <= c[s].sum()
        # with brute force on the small ones: LPT under caps is feasible, so it is at least the capped optimum
        if N <= 13 and M <= 4:
            for s in range(2):
                assert int(r["load"][s].max()) >= oracle.brute_force_opt(c[s], M, cap)


def test_lpt_status_and_return_codes(oracle):
    c = np.array([[5, 3, 2, 1], [5, -3, 2, 1]], np.int64)
    r = oracle.lpt_start(c, 2, 2)
    assert r["rc"] == 0 and r["status"].tolist() == [0, 3]
    assert r["assign"][1].tolist() == [-1] * 4 and r["load"][1].tolist() == [0, 0]
    assert oracle.lpt_start(c, 2, 1)["rc"] == -2
    assert oracle.lpt_start(c, 0, 2)["rc"] == -1
