// Test driver for the host scheduler (csrc/sched.cpp) built with -fsanitize=address,undefined:
// reads one configuration and, per round, the uploads' losses from stdin, runs Algorithm 1's server
// loop without any device and prints the integer trace.  tests/test_sched_sanitized.py compiles it,
// feeds it seeded random configurations and compares the trace with the oracle's.
//
// stdin:  N M B K0 k_mode tau_mode tau_cap a sa_penalty time_dist n_slow time_param slow_factor seed T
//         then T lines: K_replay n_losses loss_0 ... (losses in arrival order; n_losses = 0: none)
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "../paper_2301_08895_amd/csrc/sched.h"

using namespace abs_impl;

int main() {
  abs_config c{};
  long long M, T; unsigned long long seed;
  if (std::scanf("%d %lld %d %d %d %d %d %d %d %d %d %lf %lf %llu %lld", &c.N, &M, &c.B, &c.K0, &c.k_mode, &c.tau_mode,
                 &c.tau_cap, &c.a, &c.sa_penalty, &c.time_dist, &c.n_slow, &c.time_param, &c.slow_factor, &seed, &T) != 15)
    return 2;
  c.M = M; c.seed = seed; c.model = ABS_MODEL_LINEAR; c.n_layers = 1; c.dims[0] = 3; c.dims[1] = 1; c.lr = 0.01f; c.U = 1;
  std::vector<int32_t> replay((size_t)T);
  std::vector<std::vector<float>> losses((size_t)T);
  for (long long t = 0; t < T; ++t) {
    int k, n;
    if (std::scanf("%d %d", &k, &n) != 2) return 2;
    replay[(size_t)t] = k;
    losses[(size_t)t].resize((size_t)n);
    for (int i = 0; i < n; ++i) if (std::scanf("%f", &losses[(size_t)t][(size_t)i]) != 1) return 2;
  }
  if (c.k_mode == ABS_K_REPLAY) { c.k_replay = replay.data(); c.k_replay_len = T; }
  Scheduler s(c);
  std::vector<Upload> sel;
  std::string err;
  for (long long t = 0; t < T; ++t) {
    int rc = s.select(sel, err);
    if (rc != ABS_OK) { std::printf("error %d %s\n", rc, err.c_str()); return 0; }
    const std::vector<float>& l = losses[(size_t)t];
    if (!l.empty() && l.size() != sel.size()) { std::printf("error -1 loss count\n"); return 0; }
    rc = s.complete(sel, l.empty() ? nullptr : l.data(), !l.empty(), err);
    if (rc != ABS_OK) { std::printf("error %d %s\n", rc, err.c_str()); return 0; }
  }
  const std::vector<int32_t>& tr = s.trace();
  const int stride = s.stride();
  for (size_t i = 0; i < tr.size(); ++i) std::printf("%d%c", tr[i], (i + 1) % (size_t)stride ? ' ' : '\n');
  return 0;
}
