"""Counter-based random numbers of the simulation (oracle side).

The paper only says that execution times are random (Section V-A) and that
minibatches are drawn independently across workers, local steps and rounds
(Section II-A, below Eq. 2).  Both are realised here as pure functions of a
counter (seed, stream, worker, job, index) hashed with the SplitMix64
output function (Steele, Lea, Flood 2014; Vigna's public-domain splitmix64),
so the order in which draws are requested never matters.
"""
from __future__ import annotations

import math

MASK64 = (1 << 64) - 1
GOLDEN_GAMMA = 0x9E3779B97F4A7C15

STREAM_TIME = 0    # execution time of job j of worker n
STREAM_BATCH = 1   # minibatch index b of job j of worker n


def mix64(z: int) -> int:
    """SplitMix64 output (finalisation) function."""
    z &= MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def splitmix64_stream(seed: int, count: int):
    """The plain SplitMix64 generator (state += gamma, output = mix64(state));
    only used to pin mix64 against the published test vector."""
    out, s = [], seed & MASK64
    for _ in range(count):
        s = (s + GOLDEN_GAMMA) & MASK64
        out.append(mix64(s))
    return out


def counter_hash(seed: int, stream: int, n: int, j: int, i: int) -> int:
    """64 random bits for the counter (seed, stream, worker n, job j, index i)."""
    a = mix64(seed + GOLDEN_GAMMA * (stream + 1))
    b = mix64(a ^ (((n & 0xFFFFFFFF) << 32) | (j & 0xFFFFFFFF)))
    return mix64(b + GOLDEN_GAMMA * (i + 1))


def uniform01(hbits: int) -> float:
    """Top 53 bits as a double in [0, 1)."""
    return (hbits >> 11) * (1.0 / 9007199254740992.0)


TICKS_PER_UNIT = 1 << 20


def compute_time_ticks(cfg: dict, n: int, j: int) -> int:
    """Execution time of job j of worker n in integer ticks (2^-20 time units).

    time_dist 0: 1 + Exp(1); 1: Pareto(x_m = 1, alpha = time_param); 2: constant 1.
    Workers 0 .. n_slow-1 are slowed by slow_factor.  Scalar libm log / pow in
    double precision; the tick value is floor(c * 2^20).
    """
    u = uniform01(counter_hash(cfg["seed_sim"], STREAM_TIME, n, j, 0))
    dist = cfg["time_dist"]
    if dist == 0:
        c = 1.0 - math.log(1.0 - u)
    elif dist == 1:
        c = math.pow(1.0 - u, -1.0 / cfg["time_param"])
    elif dist == 2:
        c = 1.0
    else:
        raise ValueError("time_dist")
    if n < cfg.get("n_slow", 0):
        c = c * cfg["slow_factor"]
    return int(math.floor(c * TICKS_PER_UNIT))


def shard_rows(cfg: dict) -> int:
    """Rows per worker shard: the dataset is split into N disjoint contiguous
    shards (Section II-A); left-over rows are unused."""
    return cfg["M"] // cfg["N"]


def batch_indices(cfg: dict, n: int, j: int, u: int = 0):
    """Dataset rows of the minibatch of local step u of job j of worker n: B draws, iid
    uniform (with replacement) from the worker's own shard; draw b of step u has counter
    index u * B + b, so minibatches are independent across workers, local steps and rounds."""
    S = shard_rows(cfg)
    base = n * S
    B = cfg["B"]
    return [base + counter_hash(cfg["seed_sim"], STREAM_BATCH, n, j, u * B + b) % S
            for b in range(B)]
