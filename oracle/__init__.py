"""CPU oracle for the ABS parameter-server round (TEST INFRASTRUCTURE ONLY).

A plain, slow NumPy implementation of the paper's Algorithm 1 at U = 1,
written from the paper (Section II-A, Eq. 2-3; Section III, Eq. 4-6 and
Algorithm 1).  It shares no code with the HIP library and must never be
imported by the product path: only tests, the smoke check and the
benchmark's CPU-baseline leg call it.

Pins (see tests/test_oracle_*.py): finite differences and closed-form
least-squares gradients, the reductions to synchronous SGD / ASGD / K-async
SGD stated in Section II-B, the invariants of Eq. 4-6, a brute-force
re-derivation of the schedule from the job history, SplitMix64's published
test vector, closed-form threshold / wait-count values.
Parity unpinned: the actual trajectories of the classification workloads
(the paper prints no numbers for them).
"""
