"""Pins for the oracle's random numbers and bf16 rounding (CPU only)."""
import math

import numpy as np
import torch

from oracle import counter_rng as crng
from oracle.bf16 import round_bf16, bits_to_f64
from parity_util import golden_lines


def test_splitmix64_published_vector():
    # Test vector of the public-domain splitmix64 generator for seed 1234567
    # (the values its reference implementation prints; also used by several
    # language runtimes' test suites).
    want = [int(row[0]) for row in golden_lines("splitmix64_seed_1234567.txt")]
    assert len(want) == 5 and want[0] == 6457827717110365317
    assert crng.splitmix64_stream(1234567, 5) == want


def test_counter_hash_depends_on_every_field():
    base = (7, 0, 3, 5, 2)
    vals = {crng.counter_hash(*base)}
    for pos in range(5):
        for delta in (1, 2, 1 << 20):
            c = list(base); c[pos] += delta
            vals.add(crng.counter_hash(*c))
    assert len(vals) == 16
    # worker and job do not alias each other
    assert crng.counter_hash(1, 0, 1, 0, 0) != crng.counter_hash(1, 0, 0, 1, 0)


def test_uniform_range_and_moments():
    us = [crng.uniform01(crng.counter_hash(11, 0, n, j, 0)) for n in range(40) for j in range(500)]
    assert 0.0 <= min(us) and max(us) < 1.0
    assert abs(np.mean(us) - 0.5) < 0.01
    assert abs(np.var(us) - 1 / 12) < 0.005


def test_shifted_exponential_times():
    cfg = dict(seed_sim=5, time_dist=0, time_param=0.0, n_slow=2, slow_factor=5.0)
    t = np.array([[crng.compute_time_ticks(cfg, n, j) for j in range(4000)] for n in range(4)],
                 dtype=np.float64) / crng.TICKS_PER_UNIT
    assert t[2:].min() >= 1.0
    assert abs(t[2:].mean() - 2.0) < 0.05          # E[1 + Exp(1)] = 2
    assert abs(np.median(t[2:]) - (1 + math.log(2))) < 0.05
    assert abs(t[:2].mean() - 10.0) < 0.25         # slowed five-fold
    assert t[:2].min() >= 5.0


def test_pareto_times():
    cfg = dict(seed_sim=9, time_dist=1, time_param=1.5, n_slow=0, slow_factor=1.0)
    t = np.array([crng.compute_time_ticks(cfg, n, j) for n in range(8) for j in range(3000)],
                 dtype=np.float64) / crng.TICKS_PER_UNIT
    assert t.min() >= 1.0
    assert abs(np.median(t) - 2 ** (1 / 1.5)) < 0.03      # median of Pareto(1, alpha) = 2^(1/alpha)
    assert abs(np.mean(t > 4.0) - 4.0 ** -1.5) < 0.01     # survival function x^-alpha


def test_constant_times():
    cfg = dict(seed_sim=9, time_dist=2, time_param=0.0, n_slow=0, slow_factor=1.0)
    assert crng.compute_time_ticks(cfg, 3, 17) == crng.TICKS_PER_UNIT


def test_batch_indices_stay_in_own_shard_and_cover_it():
    cfg = dict(seed_sim=3, M=1003, N=4, B=64)
    S = crng.shard_rows(cfg)
    assert S == 250
    seen = set()
    for n in range(4):
        for j in range(60):
            idx = crng.batch_indices(cfg, n, j)
            assert len(idx) == 64
            assert all(n * S <= i < (n + 1) * S for i in idx)
            if n == 1:
                seen.update(idx)
    assert len(seen) == S              # 3840 draws cover a 250-row shard
    assert crng.batch_indices(cfg, 1, 0) != crng.batch_indices(cfg, 1, 1)


def test_bf16_roundtrip_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    vals = bits_to_f64(bits)
    finite = np.isfinite(vals)
    again = round_bf16(vals[finite])
    assert np.array_equal(again.astype(np.float32).view(np.uint32) >> 16, bits[finite].astype(np.uint32))


def test_bf16_halfway_cases_by_hand():
    # 1 + 2^-8 lies half-way between 1 (even mantissa) and 1 + 2^-7: goes to 1
    assert round_bf16(1.0 + 2.0 ** -8) == 1.0
    # 1 + 3*2^-8 lies half-way between 1+2^-7 (odd) and 1+2^-6 (even): goes up
    assert round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert round_bf16(-(1.0 + 2.0 ** -8)) == -1.0
    assert round_bf16(0.0) == 0.0 and round_bf16(3.0e-9) > 0.0


def test_bf16_matches_library_conversion():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-30, 30, 200000))).astype(np.float32)
    ours = round_bf16(x).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours, lib)
