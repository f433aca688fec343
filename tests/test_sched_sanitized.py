"""The host scheduler under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): csrc/sched.cpp is
compiled with g++ -fsanitize=address,undefined into a small driver (tests/sched_sanitized_main.cpp) and fed
seeded random configurations - worker counts up to the maximum, every wait-count and threshold mode, all
three time models - together with the oracle's per-upload losses; its integer trace must equal the
oracle's bit for bit, and the sanitizers must stay silent."""
import os
import subprocess

import numpy as np
import pytest

import workloads
from oracle.abs_sim import AbsOracle, trace_words

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2301_08895_amd", "csrc")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("sched_san") / "sched_sanitized")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           os.path.join(ROOT, "tests", "sched_sanitized_main.cpp"), os.path.join(CSRC, "sched.cpp"), "-o", exe]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    return exe


def _random_setting(rng):
    N = int(rng.choice([1, 2, 3, 5, 8, 16, 31, 64, 128]))
    k_mode = int(rng.integers(0, 4))
    tau_mode = int(rng.integers(0, 3))
    K0 = int(rng.integers(1, N + 1))
    tau_cap = int(rng.integers(0, 9)) if tau_mode != 2 else 1024     # no threshold: the cap only sizes the ring
    p = workloads.scaled_preset(1, M=5 * N + int(rng.integers(0, 4)), dims=[3, 1], N=N, B=2, K0=K0, k_mode=k_mode,
                                tau_mode=tau_mode, tau_cap=tau_cap, a=int(rng.integers(-4, 7)),
                                sa_penalty=int(rng.integers(0, 2)), time_dist=int(rng.integers(0, 3)),
                                time_param=float(rng.choice([1.1, 1.5, 3.0])), n_slow=int(rng.integers(0, N + 1)),
                                slow_factor=float(rng.choice([1.0, 2.5, 5.0])), lr=0.05,
                                seed_sim=int(rng.integers(1, 2**62)))
    return p, int(rng.integers(3, 50))


def _run_driver(exe, p, T, ks, losses):
    head = " ".join(str(v) for v in (p["N"], p["M"], p["B"], p["K0"], p["k_mode"], p["tau_mode"], p["tau_cap"], p["a"],
                                      p["sa_penalty"], p["time_dist"], p["n_slow"], repr(p["time_param"]),
                                      repr(p["slow_factor"]), p["seed_sim"], T))
    lines = [head]
    for t in range(T):
        ls = losses[t]
        lines.append(" ".join([str(ks[t]), str(len(ls))] + [repr(float(np.float32(v))) for v in ls]))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], input="\n".join(lines) + "\n", stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True,
                       env=env, timeout=60)
    assert r.returncode == 0 and not r.stderr.strip(), f"sanitizer report or crash:\n{r.stderr[-3000:]}"
    return r.stdout


def test_seeded_fuzz_of_the_scheduler_under_sanitizers(driver):
    rng = np.random.default_rng(20250131)
    compared = 0
    for case in range(48):
        p, T = _random_setting(rng)
        d = workloads.make_inputs(p)
        if p["k_mode"] == 2:
            p["k_replay"] = [int(v) for v in rng.integers(1, p["N"] + 1, T)]
        o = AbsOracle(p, d["X"], d["y"], d["w0"], keep_models=False).run(T)
        ks = [r["K"] for r in o.trace]
        out = _run_driver(driver, p, T, ks, [r["worker_losses"] for r in o.trace])
        assert not out.startswith("error"), (case, p, out)
        got = np.array([[int(v) for v in ln.split()] for ln in out.strip().splitlines()], dtype=np.int64)
        want = np.stack([trace_words(r, p["N"]) for r in o.trace]).astype(np.int64)
        keep = np.ones(want.shape[1], bool)
        keep[10] = False                   # the loss word is a float (compared by the GPU parity tests)
        if p["k_mode"] == 2:
            keep[11] = False               # replay: the last record's K^{t+1} has no entry to take
        assert got.shape == want.shape, (case, got.shape, want.shape)
        assert np.array_equal(got[:, keep], want[:, keep]), (case, p)
        compared += 1
    assert compared == 48


def test_the_driver_reports_errors_cleanly_under_sanitizers(driver):
    """Error paths run under the sanitizers too: a replay array that ends early, and a worker staler than
    the ring when there is no threshold."""
    p = workloads.scaled_preset(1, M=40, dims=[3, 1], N=8, B=2, K0=2, k_mode=1, tau_mode=2, tau_cap=0, seed_sim=5,
                                n_slow=1, slow_factor=50.0)
    out = _run_driver(driver, p, 40, [2] * 40, [[] for _ in range(40)])
    assert out.startswith("error -4"), out
