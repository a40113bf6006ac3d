"""GPU parity on randomly drawn shapes and parameters (fixed seeds): local search through both scan
modes, the FCFS simulator and the assigned-queue simulator, each against the CPU oracle bit for bit."""
import numpy as np
import pytest

from paper_2502_15763_amd import api, workloads as W
from gpu_util import (say, gpu_local_search, compare_ls, gpu_online_sim, gpu_online_sim_assigned, compare_sim)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [11, 12])
def test_ls_random_shapes(oracle, seed):
    rng = np.random.default_rng(seed)
    for t in range(150):
        N = int(rng.integers(1, 900))
        M = int(rng.integers(1, min(48, N) + 1))
        base = -(-N // M)
        cap = base if rng.random() < 0.5 else int(base + rng.integers(1, 6))
        hi = int(rng.choice([2, 3, 7, 30, 1000, 100000, 3000000]))
        S = int(rng.integers(1, 5))
        dtype = np.int64 if rng.random() < 0.3 else np.int32
        cost, asg = W.random_offline(rng, S, N, M, cap, cost_hi=hi, dtype=dtype,
                                     start="rr" if rng.random() < 0.5 else "random")
        mp = int(rng.choice([0, 1, 3, 50, 400]))
        pruned = bool(rng.random() < 0.4)
        if t % 25 == 0:
            say(f"ls random seed={seed} case {t}")
        o = oracle.local_search(cost, asg, M, cap, mp, want_log=True)
        g = gpu_local_search(cost, asg, M, cap, mp, pruned=pruned)
        compare_ls(g, o, label=f"seed {seed} case {t}: N={N} M={M} cap={cap} hi={hi} S={S} passes={mp} pruned={pruned}")


def test_ls_random_large_shapes(oracle):
    """Layouts from 20 KB of LDS up to the multi-workgroup path."""
    rng = np.random.default_rng(13)
    for t in range(12):
        N = int(rng.choice([1500, 3000, 5000, 9000, 14000, 22000]))
        M = int(rng.integers(2, 65))
        base = -(-N // M)
        cap = base if rng.random() < 0.5 else int(base + rng.integers(1, 40))
        cost, asg = W.random_offline(rng, int(rng.integers(1, 4)), N, M, cap, cost_hi=int(rng.choice([3, 50, 5000, 200000])),
                                     dtype=np.int32, start="rr" if rng.random() < 0.6 else "random")
        mp = int(rng.choice([1, 4, 12]))
        pruned = bool(rng.random() < 0.4)
        say(f"ls random large case {t}: N={N} M={M} cap={cap} passes={mp} pruned={pruned}")
        o = oracle.local_search(cost, asg, M, cap, mp, want_log=True)
        compare_ls(gpu_local_search(cost, asg, M, cap, mp, pruned=pruned), o, label=f"large case {t}")
        if api.mmbp_workspace_bytes(1024, N, M) == 0:          # fits one workgroup's LDS: that path too
            compare_ls(gpu_local_search(cost, asg, M, cap, mp, pruned=pruned, use_workspace=False), o,
                       label=f"large case {t}, one workgroup per scenario")


def test_ls_random_multi_workgroup_shapes(oracle):
    """Shapes of the multi-workgroup path only: many passes, slack and tight capacity, tiny cost
    ranges (heavy ties, clients within a few units of each other), uneven client sizes."""
    rng = np.random.default_rng(15)
    for t in range(24):
        N = int(rng.choice([13000, 14000, 17001, 22000, 30000]))
        M = int(rng.integers(2, 65))
        base = -(-N // M)
        cap = base if rng.random() < 0.3 else int(base + rng.integers(1, 200))
        hi = int(rng.choice([2, 3, 50, 5000, 200000]))
        S = int(rng.integers(1, 4))
        cost, asg = W.random_offline(rng, S, N, M, cap, cost_hi=hi, dtype=np.int64 if rng.random() < 0.3 else np.int32,
                                     start="rr" if rng.random() < 0.4 else "random")
        mp = int(rng.choice([3, 12, 40]))
        pruned = bool(rng.random() < 0.4)
        assert api.mmbp_workspace_bytes(S, N, M) > 0           # not an LDS-resident shape
        say(f"ls random multi-workgroup case {t}: N={N} M={M} cap={cap} hi={hi} S={S} passes={mp} pruned={pruned}")
        o = oracle.local_search(cost, asg, M, cap, mp, want_log=True)
        compare_ls(gpu_local_search(cost, asg, M, cap, mp, pruned=pruned), o, label=f"multi-workgroup case {t}")


def test_sim_random_parameters(oracle):
    rng = np.random.default_rng(14)
    for t in range(120):
        N = int(rng.integers(1, 700))
        cap = int(rng.integers(1, 65))
        S = int(rng.integers(1, 5))
        w = W.config5(S=S, N=N, rate_per_s=float(rng.choice([2, 20, 50, 500, 1e5])), seed_offset=int(rng.integers(0, 10 ** 6)))
        p = dict(cap=cap, a_prefill=int(rng.integers(0, 200)), b_decode=int(rng.integers(0, 2000)),
                 c_prefill=int(rng.integers(0, 30000)), c_decode=int(rng.integers(0, 30000)),
                 max_prefill_tokens=int(rng.choice([0, 0, 300, 2000, 100000])), policy=int(rng.integers(0, 3)))
        tc = 4 * N + 8
        if t % 30 == 0:
            say(f"sim random case {t}")
        compare_sim(gpu_online_sim(w.arrival_us, w.in_len, w.out_len, p, S, tc),
                    oracle.online_iter_sim(w.arrival_us, w.in_len, w.out_len, p, S, tc), label=f"sim case {t} {p}")
        asg = rng.integers(0, cap, (S, N)).astype(np.int32)
        if rng.random() < 0.3:
            asg[:] = rng.integers(0, cap)
        if rng.random() < 0.3:
            asg = np.minimum(asg, cap // 4).astype(np.int32)
        compare_sim(gpu_online_sim_assigned(w.in_len, w.out_len, asg, p, S, tc),
                    oracle.online_iter_sim_assigned(w.in_len, w.out_len, asg, p, S, tc), label=f"assigned case {t} {p}")
