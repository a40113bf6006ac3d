"""Pins for the CPU oracle's lower bound and online iteration simulator (no GPU).

Lower bound: paper section "Offline requests scheduling & theoretical lower bound"
(T^LB = t^p* + t^d*, t^p* = T^p_L floor(sum N^p_i / N^cap_L)).  Simulator: decision rule of
section "Online requests and iteration scheduling", time model of section "Experiment
settings and baseline".
"""
import os
import struct

import numpy as np
import pytest

from paper_2502_15763_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "time_model_examples.txt")
PAPER_US = dict(cap=200, a_prefill=130, b_decode=210, c_prefill=25000, c_decode=29000, max_prefill_tokens=0)


# ------------------------------------------------------------------ lower bound
def test_lb_closed_forms(oracle):
    rng = np.random.default_rng(3)
    # N <= M: LB = OPT = largest cost
    c = rng.integers(1, 100, size=(5, 4)).astype(np.int64)
    lb = oracle.lower_bound(c, 6)["lb"]
    assert lb.tolist() == c.max(axis=1).tolist()
    for s in range(5):
        assert oracle.brute_force_opt(c[s], 6, 1) == int(lb[s])
    # equal costs, M | N: LB = OPT = c*N/M
    c = np.full((1, 12), 7, np.int64)
    assert int(oracle.lower_bound(c, 4)["lb"][0]) == 21
    # N = M+1: OPT = max(c_(1), c_(M)+c_(M+1)) = LB
    for _ in range(10):
        c = rng.integers(1, 60, size=(1, 5)).astype(np.int64)
        s = np.sort(c[0])[::-1]
        expect = max(int(s[0]), int(s[3] + s[4]))
        assert int(oracle.lower_bound(c, 4)["lb"][0]) == expect == oracle.brute_force_opt(c[0], 4, 5)
    # ceil of the average: 3 jobs of 1 on 2 clients, plus a check where L1 dominates
    assert int(oracle.lower_bound(np.array([[5, 5, 5, 5, 1]], np.int64), 2)["lb"][0]) == 11


def test_lb_below_bruteforce_opt(oracle):
    rng = np.random.default_rng(5)
    for N, M in [(7, 2), (8, 3), (9, 4), (10, 3)]:
        for _ in range(8):
            c = rng.integers(0, 40, size=(1, N)).astype(np.int64)
            assert int(oracle.lower_bound(c, M)["lb"][0]) <= oracle.brute_force_opt(c[0], M, N)


def test_lb_prefill_term(oracle):
    # worked example of the paper's time model: a prefill bin of 5000 tokens takes 675 ms;
    # sum N^p = 5000..9999 with N^cap_L = 5000 -> floor = 1 -> t^p* = 675 ms
    c = np.array([[10, 10]], np.int64)
    base = int(oracle.lower_bound(c, 2)["lb"][0])
    for tok, k in [((2500, 2500), 1), ((4999, 5000), 1), ((5000, 5000), 2), ((2499, 2500), 0)]:
        r = oracle.lower_bound(c, 2, prefill_tokens=np.array([tok], np.int32), ncap_L=5000, tp_L=675000)
        assert int(r["lb"][0]) == base + 675000 * k
    # disabled when ncap_L == 0
    r = oracle.lower_bound(c, 2, prefill_tokens=np.array([[9000, 9000]], np.int32), ncap_L=0, tp_L=675000)
    assert int(r["lb"][0]) == base


def test_lb_bad_cost(oracle):
    r = oracle.lower_bound(np.array([[1, -1], [2, 2]], np.int64), 2)
    assert r["status"].tolist() == [3, 0] and r["lb"].tolist() == [0, 2]


def test_lb_negative_token_count_is_bad_input(oracle):
    # N^p_i is a token count; a negative entry invalidates the scenario when the prefill term is on,
    # and is not looked at when the term is off
    c = np.array([[10, 10], [10, 10]], np.int64)
    tok = np.array([[100, -1], [100, 7000]], np.int32)
    r = oracle.lower_bound(c, 2, prefill_tokens=tok, ncap_L=5000, tp_L=675000)
    assert r["status"].tolist() == [3, 0] and r["lb"].tolist() == [0, 10 + 675000]
    r = oracle.lower_bound(c, 2, prefill_tokens=tok, ncap_L=0, tp_L=675000)
    assert r["status"].tolist() == [0, 0] and r["lb"].tolist() == [10, 10]


# ------------------------------------------------------------------ extended lower bound
LB_EX_GOLD = os.path.join(os.path.dirname(__file__), "golden", "lb_ex_hand_worked.txt")


def _lb_ex_cases():
    cases = []
    ints = lambda t: None if t.strip() == "-" else [int(x) for x in t.split()]
    for line in open(LB_EX_GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        p = [x.strip() for x in line.split("|")]
        lv = None if p[6] == "-" else [tuple(int(v) for v in t.split(":")) for t in p[6].split()]
        cases.append(dict(name=p[0], M=int(p[1]), cost=ints(p[2]), caps=ints(p[3]), kmax=int(p[4]), tokens=ints(p[5]),
                          levels=lv, tp_form=int(p[7]), parts=[int(x) for x in p[8:14]], lb=int(p[14])))
    return cases


def _lb_ex(oracle, c):
    kw = {}
    if c["levels"]:
        kw = dict(prefill_tokens=np.array([c["tokens"]], np.int32), ncap=[l[0] for l in c["levels"]],
                  tp=[l[1] for l in c["levels"]], tp_form=c["tp_form"])
    return oracle.lower_bound_ex(np.array([c["cost"]], np.int64), c["M"], cap=c["caps"], kmax=c["kmax"], **kw)


@pytest.mark.parametrize("case", _lb_ex_cases(), ids=lambda c: c["name"])
def test_lb_ex_hand_worked(oracle, case):
    r = _lb_ex(oracle, case)
    assert r["rc"] == 0 and int(r["status"][0]) == 0
    assert r["parts"][0].tolist() == case["parts"]
    assert int(r["lb"][0]) == case["lb"]


def test_lb_ex_reduces_to_the_basic_bound(oracle):
    """With kmax = 1, no caps and a one-level table the extended bound is the basic one."""
    rng = np.random.default_rng(41)
    for N, M in [(1, 1), (3, 5), (9, 4), (64, 4), (200, 7), (33, 32)]:
        c = rng.integers(0, 1000, size=(6, N)).astype(np.int64)
        tok = rng.integers(1, 3000, size=(6, N)).astype(np.int32)
        a = oracle.lower_bound(c, M, prefill_tokens=tok, ncap_L=5000, tp_L=675000)
        b = oracle.lower_bound_ex(c, M, kmax=1, prefill_tokens=tok, ncap=[5000], tp=[675000], tp_form=0)
        assert a["lb"].tolist() == b["lb"].tolist()
        more = oracle.lower_bound_ex(c, M, prefill_tokens=tok, ncap=[5000], tp=[675000], tp_form=0)
        assert (more["lb"] >= a["lb"]).all()


def test_lb_ex_closed_forms(oracle):
    # N = kM + 1 equal costs c: some client holds k+1 of them; LB = OPT = (k+1) c, reached by L3(k) alone
    for k, M, cst in [(1, 3, 7), (2, 3, 7), (3, 2, 11), (2, 4, 5)]:
        N = k * M + 1
        c = np.full((1, N), cst, np.int64)
        r = oracle.lower_bound_ex(c, M)
        assert int(r["lb"][0]) == (k + 1) * cst and int(r["parts"][0][3]) == k
        if N <= 9:
            assert oracle.brute_force_opt(c[0], M, N) == (k + 1) * cst
    # N = kM + 1 with one small job and kM equal large ones: L3(k) = k large + the small one, the earlier
    # terms are (k'+1) large for k' < k, so the maximum is at k - 1 unless the small job is large enough
    c = np.array([[20] * 8 + [1]], np.int64)                             # M = 4, k = 2: L3(1) = 40, L3(2) = 41
    assert oracle.lower_bound_ex(c, 4)["parts"][0][2:4].tolist() == [41, 2]
    c = np.array([[20] * 8 + [0]], np.int64)                             # L3(2) = 40 = L3(1): the smaller k is reported
    assert oracle.lower_bound_ex(c, 4)["parts"][0][2:4].tolist() == [40, 1]
    rng = np.random.default_rng(43)
    # caps: uniform cap C -> every client holds at least N - (M-1)C jobs; tight caps (M*C == N) force C each
    c = rng.integers(1, 50, size=(1, 12)).astype(np.int64)
    r = oracle.lower_bound_ex(c, 3, cap=[4, 4, 4])
    assert int(r["parts"][0][4]) == int(np.sort(c[0])[:4].sum())
    r = oracle.lower_bound_ex(c, 3, cap=[12, 12, 12])
    assert int(r["parts"][0][4]) == 0
    # the rank limit only removes terms: a valid bound either way, never larger than with all ranks
    c = rng.integers(1, 50, size=(4, 40)).astype(np.int64)
    full = oracle.lower_bound_ex(c, 3)
    cut = oracle.lower_bound_ex(c, 3, rank_limit=10)                      # k <= 3
    lim = oracle.lower_bound_ex(c, 3, kmax=3)
    assert cut["parts"].tolist() == lim["parts"].tolist() and (cut["lb"] <= full["lb"]).all()


def test_lb_ex_below_bruteforce_opt_with_caps(oracle):
    """LB <= OPT by enumeration, per-client caps included; the brute force itself is checked
    against the definition-level enumeration."""
    from oracle import definition as D
    rng = np.random.default_rng(47)
    seen_cap_decides = seen_l3k_decides = False
    for N, M in [(6, 2), (7, 3), (8, 3), (9, 4), (7, 2), (9, 2)]:
        for trial in range(10):
            c = rng.integers(0, 30, size=(1, N)).astype(np.int64)
            if trial % 2 == 0:
                c[:] = rng.integers(10, 13)                # near-equal costs: the counting bounds decide
                c[0, : N // 3] += rng.integers(0, 3, size=N // 3)
            caps = rng.integers(1, N + 1, size=M)
            while caps.sum() < N:
                caps[rng.integers(M)] += 1
            r = oracle.lower_bound_ex(c, M, cap=caps)
            opt = oracle.brute_force_opt_caps(c[0], M, caps)
            if N <= 7:
                assert opt == D.brute_force_opt_caps(c[0].tolist(), M, caps.tolist())
            assert int(r["lb"][0]) <= opt, (c, caps, r["parts"])
            L1, L2, L3, k3, Lcap, _ = r["parts"][0].tolist()
            seen_cap_decides |= Lcap > max(L1, L2, L3)
            seen_l3k_decides |= L3 > max(L1, L2) and k3 >= 2
            free = oracle.lower_bound_ex(c, M)
            assert int(free["lb"][0]) <= oracle.brute_force_opt(c[0], M, N)
    assert seen_cap_decides and seen_l3k_decides        # the cases must exercise the new terms


def test_lb_ex_status_and_return_codes(oracle):
    c = np.array([[5, 3, 2, 1], [5, -3, 2, 1]], np.int64)
    r = oracle.lower_bound_ex(c, 2)
    assert r["rc"] == 0 and r["status"].tolist() == [0, 3] and int(r["lb"][1]) == 0
    assert oracle.lower_bound_ex(c, 2, cap=[1, 2])["rc"] == -2                 # caps cannot hold the requests
    assert oracle.lower_bound_ex(c, 2, cap=[-1, 9])["rc"] == -1
    tok = np.array([[1, 2, 3, 4], [1, 2, -3, 4]], np.int32)
    r = oracle.lower_bound_ex(c[:1].repeat(2, 0), 2, prefill_tokens=tok, ncap=[4], tp=[10])
    assert r["status"].tolist() == [0, 3] and int(r["lb"][0]) == 6 + 10 * 2
    assert oracle.lower_bound_ex(c, 2, prefill_tokens=tok, ncap=[0], tp=[10])["rc"] == -1
    assert oracle.lower_bound_ex(c, 2, prefill_tokens=tok, ncap=[4], tp=[10], tp_form=2)["rc"] == -1


# ------------------------------------------------------------------ simulator
def test_time_model_worked_examples(oracle):
    with open(GOLD) as f:
        rows = [l.split("|") for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for kind, units, expect in rows:
        fn = oracle.decode_time if kind.strip() == "decode" else oracle.prefill_time
        assert fn(PAPER_US, int(units)) == int(expect)
    # and through the simulator itself: 200 requests of 25 input tokens (5000 tokens), 1 output token each
    arr = np.zeros((1, 200), np.int64)
    r = oracle.online_iter_sim(arr, np.full((1, 200), 25, np.int32), np.ones((1, 200), np.int32), PAPER_US)
    assert int(r["total_us"][0]) == 675000 + 71000
    assert (r["finish_us"][0] == 746000).all()


def _params(cap, a=35, b=900, cp=5000, cd=5000, tok=0):
    return dict(cap=cap, a_prefill=a, b_decode=b, c_prefill=cp, c_decode=cd, max_prefill_tokens=tok)


def test_sim_single_request(oracle):
    p = _params(4)
    r = oracle.online_iter_sim(np.array([[1234]], np.int64), np.array([[100]], np.int32), np.array([[7]], np.int32), p,
                               trace_scenarios=1, trace_capacity=8)
    expect = 1234 + (35 * 100 + 5000) + 7 * (900 + 5000)
    assert int(r["total_us"][0]) == expect == int(r["finish_us"][0, 0])
    assert int(r["busy_slot_us"][0]) == expect - 1234
    assert int(r["n_prefill_iter"][0]) == 1 and int(r["n_decode_iter"][0]) == 7
    tr = r["trace"][0][: int(r["trace_len"][0])]
    assert [tuple(x) for x in tr.tolist()] == [(2, 1, 0, 0), (1, 1, 1234, 100), (0, 7, 1234 + 8500, 1)]


def test_sim_batch_at_time_zero(oracle):
    rng = np.random.default_rng(2)
    n, L = 6, 9
    in_len = rng.integers(1, 300, size=(1, n)).astype(np.int32)
    p = _params(8)
    r = oracle.online_iter_sim(np.zeros((1, n), np.int64), in_len, np.full((1, n), L, np.int32), p)
    expect = 35 * int(in_len.sum()) + 5000 + L * (900 * n + 5000)
    assert int(r["total_us"][0]) == expect
    assert (r["finish_us"][0] == expect).all()


def test_sim_cap_one_is_serial_fcfs(oracle):
    rng = np.random.default_rng(4)
    N = 40
    arr = np.cumsum(rng.integers(0, 30000, size=(1, N)), axis=1).astype(np.int64)
    in_len = rng.integers(1, 200, size=(1, N)).astype(np.int32)
    out_len = rng.integers(1, 20, size=(1, N)).astype(np.int32)
    p = _params(1)
    r = oracle.online_iter_sim(arr, in_len, out_len, p)
    t = 0
    for i in range(N):
        t = max(t, int(arr[0, i])) + 35 * int(in_len[0, i]) + 5000 + int(out_len[0, i]) * (900 + 5000)
        assert int(r["finish_us"][0, i]) == t
    assert int(r["total_us"][0]) == t


def _fnv(data):
    h = 0xcbf29ce484222325
    for b in data:
        h = ((h ^ b) * 0x100000001b3) & 0xFFFFFFFFFFFFFFFF
    return h


def test_fnv_published_vectors(oracle):
    assert oracle.fnv1a64(b"") == 0xcbf29ce484222325
    assert oracle.fnv1a64(b"a") == 0xaf63dc4c8601ec8c
    assert oracle.fnv1a64(b"foobar") == 0x85944171f73967e8


@pytest.mark.parametrize("tok_cap", [0, 600])
def test_sim_conservation_and_trace(oracle, tok_cap):
    c5 = W.config5(S=6, N=300)
    p = dict(c5.params)
    p["cap"] = 16
    p["max_prefill_tokens"] = tok_cap
    r = oracle.online_iter_sim(c5.arrival_us, c5.in_len, c5.out_len, p, trace_scenarios=6, trace_capacity=4000)
    assert (r["status"] == 0).all()
    a, b, cp, cd = p["a_prefill"], p["b_decode"], p["c_prefill"], p["c_decode"]
    for s in range(6):
        n = int(r["trace_len"][s])
        assert n <= 4000
        tr = r["trace"][s][:n]
        dec = tr[tr["kind"] == 0]
        pre = tr[tr["kind"] == 1]
        # conservation: every output token decoded once, every request prefilled once
        assert int((dec["count"].astype(np.int64) * dec["x"]).sum()) == int(c5.out_len[s].sum())
        assert int(pre["count"].sum()) == 300
        assert int(pre["x"].sum()) == int(c5.in_len[s].sum())
        assert int(dec["x"].max()) <= 16 and int(pre["count"].max()) <= 16
        assert int(dec["count"].sum()) == int(r["n_decode_iter"][s]) and len(pre) == int(r["n_prefill_iter"][s])
        if tok_cap:
            multi = pre[pre["count"] > 1]
            assert (multi["x"] <= tok_cap).all()
        # a prefill is always followed by a decode; merged decode runs are maximal
        kinds = tr["kind"].tolist()
        for q in range(n - 1):
            if kinds[q] == 1:
                assert kinds[q + 1] == 0
            if kinds[q] == 0 and kinds[q + 1] == 0:
                assert tr["x"][q] != tr["x"][q + 1]
        # time is the sum of the iteration times (+ idle gaps), busy slot time likewise
        t, busy = 0, 0
        for k, cnt, ts, x in tr.tolist():
            if k == 2:
                assert ts == t
                nxt = c5.arrival_us[s][c5.arrival_us[s] > t].min()
                t = int(nxt)
                continue
            assert ts == t
            if k == 1:
                dt = a * x + cp
                t += dt
                busy += cnt * dt
            else:
                dt = b * x + cd
                t += cnt * dt
                busy += cnt * x * dt
        assert t == int(r["total_us"][s]) == int(r["finish_us"][s].max())
        assert busy == int(r["busy_slot_us"][s])
        # no request finishes faster than running alone
        lo = c5.arrival_us[s] + a * c5.in_len[s] + cp + c5.out_len[s].astype(np.int64) * (b + cd)
        assert (r["finish_us"][s] >= lo).all()
        # hash of the canonical records, recomputed independently
        data = b"".join(struct.pack("<IIqq", *rec) for rec in tr.tolist())
        assert _fnv(data) == int(r["trace_hash"][s])


def test_sim_decision_rule_direction(oracle):
    """C_p >= C_d keeps decoding (ties included); the first strictly larger C_d triggers the prefill.
    One long request runs alone (D = 1, C_d grows by b per iteration); a second one waits."""
    b = 1000
    for cp_tokens, cfix in [(10, 0), (3, 2000)]:
        p = _params(2, a=500, b=b, cp=cfix, cd=0)
        Cp = 500 * cp_tokens + cfix          # 5000 / 3500
        arr = np.array([[0, 1]], np.int64)
        r = oracle.online_iter_sim(arr, np.array([[1, cp_tokens]], np.int32), np.array([[50, 1]], np.int32), p,
                                   trace_scenarios=1, trace_capacity=16)
        tr = [tuple(x) for x in r["trace"][0][: int(r["trace_len"][0])].tolist()]
        # decode iterations with D=1 before the second prefill: smallest m with m*b > Cp
        m = Cp // b + 1
        assert tr[0] == (1, 1, 0, 1)
        assert tr[1][0] == 0 and tr[1][1] == m and tr[1][3] == 1
        assert tr[2][0] == 1 and tr[2][3] == cp_tokens


def test_sim_oversized_head_request_still_admitted(oracle):
    p = _params(4, tok=100)
    r = oracle.online_iter_sim(np.zeros((1, 3), np.int64), np.array([[500, 60, 60]], np.int32),
                               np.array([[2, 2, 2]], np.int32), p, trace_scenarios=1, trace_capacity=16)
    tr = [tuple(x) for x in r["trace"][0][: int(r["trace_len"][0])].tolist()]
    assert tr[0] == (1, 1, 0, 500)           # alone, although above the token cap
    assert int(r["status"][0]) == 0


def test_sim_bad_input(oracle):
    arr = np.array([[0, 5, 3], [0, 1, 2], [0, 1, 2], [0, 1, 2]], np.int64)
    inl = np.array([[1, 1, 1], [1, 0, 1], [1, 1, 1], [1, 1, 1]], np.int32)
    outl = np.array([[1, 1, 1], [1, 1, 1], [1, 1, 0], [1, 1, 1]], np.int32)
    r = oracle.online_iter_sim(arr, inl, outl, _params(2))
    assert r["status"].tolist() == [4, 4, 4, 0]
    assert (r["finish_us"][:3] == 0).all() and (r["total_us"][:3] == 0).all()


# ------------------------------------------------------------------ baseline policies of the simulator
GOLD_POLICIES = os.path.join(os.path.dirname(__file__), "golden", "sim_policies_hand_worked.txt")


def test_sim_policies_hand_worked(oracle):
    """Traces worked by hand for the paper's rule and for the two readings of its baseline
    (prefill first, with and without batched prefill)."""
    arr = np.array([[0, 0, 30]], np.int64)
    inl = np.array([[10, 20, 100]], np.int32)
    outl = np.array([[3, 2, 2]], np.int32)
    seen = 0
    for line in open(GOLD_POLICIES):
        if line.startswith("#") or not line.strip():
            continue
        pol, total, busy, npre, ndec, fin, recs = [f.strip() for f in line.split("|")]
        p = dict(cap=2, a_prefill=1, b_decode=10, c_prefill=5, c_decode=2, max_prefill_tokens=0, policy=int(pol))
        r = oracle.online_iter_sim(arr, inl, outl, p, trace_scenarios=1, trace_capacity=16)
        assert r["rc"] == 0 and int(r["status"][0]) == 0
        assert int(r["total_us"][0]) == int(total) and int(r["busy_slot_us"][0]) == int(busy)
        assert int(r["n_prefill_iter"][0]) == int(npre) and int(r["n_decode_iter"][0]) == int(ndec)
        assert r["finish_us"][0].tolist() == [int(x) for x in fin.split(",")]
        want = [tuple(int(x) for x in rec.split(":")) for rec in recs.split()]
        got = [tuple(int(x) for x in rec) for rec in r["trace"][0][: int(r["trace_len"][0])]]
        assert got == want
        # the hash is FNV-1a over the little-endian bytes of exactly these records
        raw = b"".join(np.array([w], dtype=oracle.TRACE_DTYPE).tobytes() for w in want)
        assert int(r["trace_hash"][0]) == oracle.fnv1a64(raw)
        seen += 1
    assert seen == 3


@pytest.mark.parametrize("policy", [1, 2])
def test_sim_prefill_first_never_decodes_past_a_waiting_request(oracle, policy):
    """Property that defines the baseline: a decode iteration starts only if no arrived request
    could take a free slot.  Checked from the trace and the arrivals alone."""
    c5 = W.config5(S=5, N=200, rate_per_s=30)
    p = dict(c5.params, cap=8, policy=policy)
    r = oracle.online_iter_sim(c5.arrival_us, c5.in_len, c5.out_len, p, trace_scenarios=5, trace_capacity=3000)
    assert (r["status"] == 0).all()
    b, cd = p["b_decode"], p["c_decode"]
    for s in range(5):
        tr = r["trace"][s][: int(r["trace_len"][s])]
        admitted = 0
        n_pre_single = 0
        for kind, count, t0, x in tr.tolist():
            if kind == 1:
                admitted += count
                n_pre_single += count == 1
                if policy == 2:
                    assert count == 1
            elif kind == 0 and x < p["cap"] and admitted < 200:
                last_boundary = t0 + (count - 1) * (b * x + cd)      # start of the run's last iteration
                assert c5.arrival_us[s][admitted] > last_boundary
        assert admitted == 200
        # conservation as for the rule
        dec = tr[tr["kind"] == 0]
        assert int((dec["count"].astype(np.int64) * dec["x"]).sum()) == int(c5.out_len[s].sum())


def test_sim_policies_agree_where_they_must(oracle):
    """cap = 1 leaves no choice (serial FCFS), and requests that all fit at t = 0 are prefilled at
    once by the rule (forced) and by the batched baseline alike."""
    c5 = W.config5(S=4, N=40)
    base = dict(c5.params, cap=1)
    ref = oracle.online_iter_sim(c5.arrival_us, c5.in_len, c5.out_len, base)
    for pol in (1, 2):
        r = oracle.online_iter_sim(c5.arrival_us, c5.in_len, c5.out_len, dict(base, policy=pol))
        assert np.array_equal(r["finish_us"], ref["finish_us"]) and np.array_equal(r["trace_hash"], ref["trace_hash"])
    arr = np.zeros((4, 40), np.int64)
    wide = dict(c5.params, cap=64)
    ref = oracle.online_iter_sim(arr, c5.in_len, c5.out_len, wide)
    r = oracle.online_iter_sim(arr, c5.in_len, c5.out_len, dict(wide, policy=1))
    assert np.array_equal(r["finish_us"], ref["finish_us"]) and np.array_equal(r["trace_hash"], ref["trace_hash"])
    assert oracle.online_iter_sim(arr, c5.in_len, c5.out_len, dict(wide, policy=3))["rc"] != 0


# ------------------------------------------------------------------ simulator fed by an offline assignment
GOLD_ASSIGNED = os.path.join(os.path.dirname(__file__), "golden", "sim_assigned_hand_worked.txt")


def test_sim_assigned_hand_worked(oracle):
    seen = 0
    for line in open(GOLD_ASSIGNED):
        if line.startswith("#") or not line.strip():
            continue
        f = [x.strip() for x in line.split("|")]
        ints = lambda k: [int(x) for x in f[k].split(",")]
        p = dict(cap=int(f[1]), a_prefill=1, b_decode=10, c_prefill=5, c_decode=2, max_prefill_tokens=0, policy=int(f[2]))
        r = oracle.online_iter_sim_assigned(np.array([ints(3)]), np.array([ints(4)]), np.array([ints(5)]), p, 1, 32)
        assert r["rc"] == 0 and int(r["status"][0]) == 0
        assert [int(r[k][0]) for k in ("total_us", "busy_slot_us", "n_prefill_iter", "n_decode_iter")] == [int(f[k]) for k in (6, 7, 8, 9)]
        assert r["finish_us"][0].tolist() == ints(10) and r["served_by"][0].tolist() == ints(11)
        assert r["start_us"][0].tolist() == ints(12)
        want = [tuple(int(x) for x in rec.split(":")) for rec in f[13].split()]
        assert [tuple(int(x) for x in rec) for rec in r["trace"][0][: int(r["trace_len"][0])]] == want
        raw = b"".join(np.array([w], dtype=oracle.TRACE_DTYPE).tobytes() for w in want)
        assert int(r["trace_hash"][0]) == oracle.fnv1a64(raw)
        seen += 1
    assert seen == 2


@pytest.mark.parametrize("policy,tok_cap", [(0, 0), (1, 0), (1, 700), (2, 0)])
def test_sim_assigned_properties(oracle, policy, tok_cap):
    """What the method fixes, checked from the outputs alone: every request runs once on one client,
    a client runs one request at a time, own-queue requests start longest first, a client steals
    only when its own queue is used up, and what it steals is the longest request left in the
    victim's queue."""
    rng = np.random.default_rng(100 + policy)
    S, N, cap = 6, 180, 7
    c5 = W.config5(S=S, N=N)
    inl, outl = c5.in_len, c5.out_len
    assign = rng.integers(0, cap, (S, N)).astype(np.int32)
    assign[0] = np.arange(N) % cap                     # balanced
    assign[1] = np.minimum(np.arange(N) // 60, cap - 1)  # three loaded clients, four that only steal
    p = dict(c5.params, cap=cap, max_prefill_tokens=tok_cap, policy=policy)
    r = oracle.online_iter_sim_assigned(inl, outl, assign, p, S, 2000)
    assert (r["status"] == 0).all()
    for s in range(S):
        ln = inl[s].astype(np.int64) + outl[s]
        st, fi, by = r["start_us"][s], r["finish_us"][s], r["served_by"][s]
        assert ((by >= 0) & (by < cap)).all() and (fi > st).all()
        for j in range(cap):
            mine = np.where(by == j)[0]
            o = mine[np.argsort(st[mine], kind="stable")]
            assert (st[o][1:] >= fi[o][:-1]).all()                      # one at a time
            own = np.where((assign[s] == j))[0]
            own_sorted = own[np.lexsort((own, -ln[own]))]              # I_j: longest first, then index
            assert (np.diff(st[own_sorted]) >= 0).all()                 # whoever runs them, they leave I_j in order
            stolen = mine[assign[s][mine] != j]
            if len(stolen) and len(own):
                assert st[stolen].min() >= st[own].max()                # steals only after the own queue is used up
        tr = r["trace"][s][: int(r["trace_len"][s])]
        dec, pre = tr[tr["kind"] == 0], tr[tr["kind"] == 1]
        assert int((dec["count"].astype(np.int64) * dec["x"]).sum()) == int(outl[s].sum())
        assert int(pre["count"].sum()) == N and int(pre["x"].sum()) == int(inl[s].sum())
        assert (tr["kind"] != 2).all()
        if policy == 2:
            assert (pre["count"] == 1).all()
        if tok_cap:
            assert (pre[pre["count"] > 1]["x"] <= tok_cap).all()
    assert (r["served_by"][1] >= 3).any()                              # the idle clients did steal


def test_sim_assigned_reduces_to_known_cases(oracle):
    c5 = W.config5(S=3, N=30)
    inl, outl = c5.in_len, c5.out_len
    # one client: the requests run one after the other, longest first; the total has a closed form
    p = dict(c5.params, cap=1)
    r = oracle.online_iter_sim_assigned(inl, outl, np.zeros_like(inl), p)
    a, b, cp, cd = p["a_prefill"], p["b_decode"], p["c_prefill"], p["c_decode"]
    expect = (a * inl.astype(np.int64) + cp + outl.astype(np.int64) * (b + cd)).sum(axis=1)
    assert r["total_us"].tolist() == expect.tolist()
    ln = inl.astype(np.int64) + outl
    for s in range(3):
        order = np.argsort(r["start_us"][s], kind="stable")
        assert (np.diff(ln[s][order]) <= 0).all()
    # one request per client: everything is prefilled at t = 0, as in the FCFS simulator
    p = dict(c5.params, cap=30)
    r = oracle.online_iter_sim_assigned(inl, outl, np.tile(np.arange(30, dtype=np.int32), (3, 1)), p)
    f = oracle.online_iter_sim(np.zeros_like(inl, dtype=np.int64), inl, outl, p)
    assert np.array_equal(r["finish_us"], f["finish_us"]) and np.array_equal(r["trace_hash"], f["trace_hash"])
    # bad input: a client index outside [0, cap)
    bad = np.zeros_like(inl); bad[1, 5] = 30
    assert oracle.online_iter_sim_assigned(inl, outl, bad, p)["status"].tolist() == [0, 4, 0]
