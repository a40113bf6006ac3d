"""Seeded synthetic inputs for the five workload configurations.

This module only draws random request lengths / arrival times and turns them into the
integer job costs handed to the schedulers.  It contains none of the scheduling
arithmetic and is the only module shared by the GPU path's tests and the CPU oracle.

All draws come from ``numpy.random.Generator(PCG64(SEED_BASE + config_id))``; one draw of
shape [S, N] per array, in the order documented per configuration.  Floating point is
used inside the generator only; everything returned is an integer array.

Request lengths follow the paper's notation: ``in_len`` = N^p_i (input tokens),
``out_len`` = N^d_i (output tokens); ``cost`` = T_i of the offline MMBP model.
"""
from __future__ import annotations

from dataclasses import dataclass, field
import numpy as np

SEED_BASE = 250215763

# integer time model used for the offline job cost (microseconds)
COST_PER_IN_TOKEN = 40
COST_FIXED = 2000
COST_PER_OUT_TOKEN = 120


@dataclass
class OfflineWorkload:
    name: str
    S: int
    N: int
    M: int
    batch_cap: int          # B of the configuration
    cap: int                # C handed to the library: whole waves of B per instance
    cost: np.ndarray        # [S, N] int32 or int64, microseconds
    assign0: np.ndarray     # [S, N] int32 round-robin start
    in_len: np.ndarray      # [S, N] int32
    out_len: np.ndarray     # [S, N] int32
    max_passes: int


@dataclass
class OnlineWorkload:
    name: str
    S: int
    N: int
    arrival_us: np.ndarray  # [S, N] int64, nondecreasing along N
    in_len: np.ndarray      # [S, N] int32
    out_len: np.ndarray     # [S, N] int32
    params: dict = field(default_factory=dict)


def job_cost(in_len: np.ndarray, out_len: np.ndarray, dtype) -> np.ndarray:
    c = (COST_PER_IN_TOKEN * in_len.astype(np.int64) + COST_FIXED
         + COST_PER_OUT_TOKEN * out_len.astype(np.int64))
    return np.ascontiguousarray(c.astype(dtype))


def tight_capacity(N: int, M: int, B: int) -> int:
    """Cardinality limit per instance: whole waves of the batch cap B, C = B*ceil(N/(M*B))."""
    return B * (-(-N // (M * B)))


def round_robin(S: int, N: int, M: int) -> np.ndarray:
    return np.ascontiguousarray(np.broadcast_to((np.arange(N, dtype=np.int32) % M), (S, N)).copy())


def _rng(config_id: int, seed_offset: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(SEED_BASE + config_id + 1000 * seed_offset))


def _uniform_int(rng, lo, hi, shape):
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int32)


def _lognormal_int(rng, mu, sigma, lo, hi, shape):
    z = rng.normal(mu, sigma, size=shape)
    return np.clip(np.rint(np.exp(z)), lo, hi).astype(np.int32)


def _bounded_zipf(rng, s, kmax, shape):
    """Zipf(s) restricted to {1..kmax} by inverse CDF over the finite support."""
    k = np.arange(1, kmax + 1, dtype=np.float64)
    cdf = np.cumsum(k ** (-s))
    cdf /= cdf[-1]
    u = rng.random(size=shape)
    return (np.searchsorted(cdf, u, side="left") + 1).clip(1, kmax).astype(np.int32)


def _offline(name, cfg, S, N, M, B, in_len, out_len, dtype, max_passes, slack=0):
    cap = tight_capacity(N, M, B) + slack
    return OfflineWorkload(name=name, S=S, N=N, M=M, batch_cap=B, cap=cap,
                           cost=job_cost(in_len, out_len, dtype), assign0=round_robin(S, N, M),
                           in_len=in_len, out_len=out_len, max_passes=max_passes)


def config1(S=1, N=64, M=4, B=16, slack=0, seed_offset=0) -> OfflineWorkload:
    """Draw order: in_len ~ U{32..512}, out_len ~ U{16..256}."""
    rng = _rng(1, seed_offset)
    in_len = _uniform_int(rng, 32, 512, (S, N))
    out_len = _uniform_int(rng, 16, 256, (S, N))
    return _offline("c1", 1, S, N, M, B, in_len, out_len, np.int32, 10000, slack)


def config2(S=1024, N=1024, M=8, B=64, slack=0, seed_offset=0, max_passes=1024) -> OfflineWorkload:
    """Draw order: in_len ~ LN(5.0,0.6) clip [16,2048], out_len ~ LN(5.3,0.7) clip [8,1024]."""
    rng = _rng(2, seed_offset)
    in_len = _lognormal_int(rng, 5.0, 0.6, 16, 2048, (S, N))
    out_len = _lognormal_int(rng, 5.3, 0.7, 8, 1024, (S, N))
    return _offline("c2", 2, S, N, M, B, in_len, out_len, np.int32, max_passes, slack)


def config3(S=4096, N=4096, M=16, B=128, slack=0, seed_offset=0, max_passes=64) -> OfflineWorkload:
    """Draw order: u_in, u_out uniform [0,1), then the long-mode mask (p = 0.3).
    short: in U{32..256}, out U{16..128}; long: in U{1024..4096}, out U{256..1024}."""
    rng = _rng(3, seed_offset)
    u_in = rng.random(size=(S, N))
    u_out = rng.random(size=(S, N))
    long_mode = rng.random(size=(S, N)) < 0.3

    def pick(u, lo_s, hi_s, lo_l, hi_l):
        short = lo_s + np.floor(u * (hi_s - lo_s + 1)).astype(np.int64)
        long_ = lo_l + np.floor(u * (hi_l - lo_l + 1)).astype(np.int64)
        return np.where(long_mode, np.minimum(long_, hi_l), np.minimum(short, hi_s)).astype(np.int32)

    in_len = pick(u_in, 32, 256, 1024, 4096)
    out_len = pick(u_out, 16, 128, 256, 1024)
    return _offline("c3", 3, S, N, M, B, in_len, out_len, np.int64, max_passes, slack)


def config4(S=1, N=65536, M=64, B=256, slack=0, seed_offset=0, max_passes=256) -> OfflineWorkload:
    """Draw order: in_len ~ U{16..4096}, out_len ~ bounded Zipf(1.2) on {1..2048}."""
    rng = _rng(4, seed_offset)
    in_len = _uniform_int(rng, 16, 4096, (S, N))
    out_len = _bounded_zipf(rng, 1.2, 2048, (S, N))
    return _offline("c4", 4, S, N, M, B, in_len, out_len, np.int64, max_passes, slack)


C5_PARAMS = dict(cap=64, a_prefill=35, b_decode=900, c_prefill=5000, c_decode=5000,
                 max_prefill_tokens=0)


def config5(S=8192, N=2048, rate_per_s=50.0, seed_offset=0) -> OnlineWorkload:
    """Draw order: in_len, out_len as configuration 2, then exponential inter-arrival times
    (mean 1e6/rate microseconds); arrival_us = floor(cumsum)."""
    rng = _rng(5, seed_offset)
    in_len = _lognormal_int(rng, 5.0, 0.6, 16, 2048, (S, N))
    out_len = _lognormal_int(rng, 5.3, 0.7, 8, 1024, (S, N))
    gaps = rng.exponential(1e6 / rate_per_s, size=(S, N))
    arrival = np.floor(np.cumsum(gaps, axis=1)).astype(np.int64)
    return OnlineWorkload(name="c5", S=S, N=N, arrival_us=np.ascontiguousarray(arrival),
                          in_len=in_len, out_len=out_len, params=dict(C5_PARAMS))


# Paper-shaped context workload: Table "Experiment Settings" statistics only (no dataset items).
PAPER_PARAMS = dict(cap=200, a_prefill=130, b_decode=210, c_prefill=25000, c_decode=29000,
                    max_prefill_tokens=0)


def paper_shaped(S=100, N=1319, seed_offset=0):
    """Lengths ~ normal with the means / standard deviations the paper prints for its
    benchmark (input 68.43 +- 25.04, output 344.83 +- 187.99, output capped at 512)."""
    rng = _rng(9, seed_offset)
    in_len = np.clip(np.rint(rng.normal(68.43, 25.04, size=(S, N))), 1, None).astype(np.int32)
    out_len = np.clip(np.rint(rng.normal(344.83, 187.99, size=(S, N))), 1, 512).astype(np.int32)
    return in_len, out_len


def random_offline(rng: np.random.Generator, S, N, M, cap, cost_hi=1000, dtype=np.int64,
                   start="random"):
    """Small random instances for tests: feasible random (or round-robin) start."""
    cost = rng.integers(0, cost_hi + 1, size=(S, N)).astype(dtype)
    assign = np.empty((S, N), dtype=np.int32)
    for s in range(S):
        if start == "rr":
            assign[s] = np.arange(N) % M
            continue
        slots = np.repeat(np.arange(M, dtype=np.int32), cap)
        assign[s] = rng.permutation(slots)[:N]
    return np.ascontiguousarray(cost), np.ascontiguousarray(assign)
