"""Definition-level reference for the MMBP local search (pure Python, tiny inputs only).

TEST INFRASTRUCTURE ONLY.  Where the C oracle evaluates a candidate with the two-load delta
formula, this file applies the candidate to a copy of the assignment, recomputes EVERY client
load from scratch (t_j = sum of the T_i assigned to j, MMBP model constraint) and takes
max_j t_j (MMBP objective).  Agreement of the two, candidate by candidate and pass by pass,
pins the delta formula, the id layout and the tie-break of the C oracle.
"""
from __future__ import annotations

import itertools


def loads_of(cost, assign, M):
    load = [0] * M
    for c, a in zip(cost, assign):
        load[a] += int(c)
    return load


def makespan_of(cost, assign, M):
    return max(loads_of(cost, assign, M))


def scan(cost, assign, M, cap):
    """Enumerate the whole move + swap neighbourhood.  Returns (best, evals, candidates) where
    best = (value, id, new_assign) with the smallest (value, id), or None."""
    N = len(cost)
    cnt = [0] * M
    for a in assign:
        cnt[a] += 1
    evals = 0
    best = None
    cands = []
    for i in range(N):
        for b in range(M):
            if b == assign[i]:
                continue
            evals += 1
            if cnt[b] + 1 > cap:
                continue
            new = list(assign)
            new[i] = b
            v = makespan_of(cost, new, M)
            cid = i * M + b
            cands.append((v, cid))
            if best is None or (v, cid) < (best[0], best[1]):
                best = (v, cid, new)
    for i in range(N):
        for k in range(i + 1, N):
            if assign[i] == assign[k]:
                continue
            evals += 1
            new = list(assign)
            new[i], new[k] = assign[k], assign[i]
            v = makespan_of(cost, new, M)
            cid = N * M + i * N + k
            cands.append((v, cid))
            if best is None or (v, cid) < (best[0], best[1]):
                best = (v, cid, new)
    return best, evals, cands


def local_search(cost, assign0, M, cap, max_passes):
    assign = [int(a) for a in assign0]
    cost = [int(c) for c in cost]
    passes, evals, log = 0, 0, []
    status = 0
    while True:
        if passes == max_passes:
            status = 1
            break
        T = makespan_of(cost, assign, M)
        best, e, _ = scan(cost, assign, M, cap)
        evals += e
        if best is None or best[0] >= T:
            break
        assign = best[2]
        log.append(best[1])
        passes += 1
    return dict(assign=assign, load=loads_of(cost, assign, M), makespan=makespan_of(cost, assign, M),
                passes=passes, evals=evals, log=log, status=status)


def brute_force_opt(cost, M, cap):
    """Optimum of the MMBP model with the per-client cardinality limit, by enumeration."""
    N = len(cost)
    best = None
    for asg in itertools.product(range(M), repeat=N):
        cnt = [0] * M
        for a in asg:
            cnt[a] += 1
        if max(cnt) > cap:
            continue
        v = makespan_of(cost, asg, M)
        if best is None or v < best:
            best = v
    return best


def brute_force_opt_caps(cost, M, caps):
    """Optimum of the MMBP model with a cardinality limit per client, by enumeration."""
    N = len(cost)
    best = None
    for asg in itertools.product(range(M), repeat=N):
        cnt = [0] * M
        for a in asg:
            cnt[a] += 1
        if any(cnt[j] > caps[j] for j in range(M)):
            continue
        v = makespan_of(cost, asg, M)
        if best is None or v < best:
            best = v
    return best
