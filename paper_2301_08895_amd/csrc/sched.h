// Host event-queue scheduler of the ABS parameter server (Section III, Algorithm 1).
// Pure host code: execution-time draws, selection of the K^t fastest uploads, the wait
// count rule (Eq. 5), the staleness threshold (Eq. 4), the staleness / restart rule
// (Eq. 6), communication counters (Section V-B) and the integer event trace.
#pragma once
#include <cstdint>
#include <string>
#include <vector>
#include "abs_common.h"

namespace abs_impl {

struct Upload {       // one aggregated upload of the current round
  int32_t  id;
  int64_t  ver;       // model version the worker computed at
  int32_t  tau;       // staleness t - ver
  uint32_t job;       // job counter (selects the minibatch)
};

class Scheduler {
 public:
  explicit Scheduler(const abs_config& cfg);

  int64_t round() const { return t_; }
  int     wait_count() const { return K_; }
  int     stride() const { return ABS_TRACE_HEADER + 3 * N_; }

  // Step 1 of a round: K^t for this round and the K^t earliest finishers in arrival
  // order (ties: lower id).  Returns ABS_OK, ABS_E_REPLAY or ABS_E_VERSION.
  int select(std::vector<Upload>& out, std::string& err);

  // Remaining steps once the uploads' minibatch losses are known (NaN in schedule-only
  // mode): loss estimate, Eq. 5, Eq. 4 / Eq. 6, re-arming, counters, trace record.
  int complete(const std::vector<Upload>& sel, const float* worker_loss, bool have_loss,
               std::string& err);

  const std::vector<int32_t>& trace() const { return trace_; }

  static uint64_t time_ticks(const abs_config& cfg, int32_t n, int64_t j);

 private:
  bool over_stale(int tau, int K) const;
  int  threshold_floor(int K) const;
  int  next_wait_count(int K_now, double loss_t) const;

  abs_config cfg_;
  std::vector<int32_t> replay_;
  int N_;
  int64_t t_ = 0;
  int K_;
  double loss0_ = 0.0;
  uint64_t now_ = 0;
  uint64_t uploads_ = 0, restarts_ = 0;
  std::vector<int32_t> tau_;
  std::vector<int64_t> ver_;
  std::vector<uint32_t> job_;
  std::vector<uint64_t> fin_;
  std::vector<int32_t> order_;
  std::vector<char> in_sel_;          // scratch of complete(): aggregated or restarted this round
  std::vector<int32_t> restart_;      // scratch of complete(): the restart set, ascending
  std::vector<int32_t> trace_;
};

}  // namespace abs_impl
