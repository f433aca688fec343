#include "sched.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>

namespace abs_impl {

uint64_t Scheduler::time_ticks(const abs_config& cfg, int32_t n, int64_t j) {
  const uint64_t h = draw(job_key(stream_key(cfg.seed, kStreamTime), (uint32_t)n, (uint32_t)j), 0);
  const double u = (double)(h >> 11) * (1.0 / 9007199254740992.0);   // [0, 1)
  double c;
  switch (cfg.time_dist) {
    case ABS_TIME_EXP:    c = 1.0 - std::log(1.0 - u); break;
    case ABS_TIME_PARETO: c = std::pow(1.0 - u, -1.0 / cfg.time_param); break;
    default:              c = 1.0; break;
  }
  if (n < cfg.n_slow) c = c * cfg.slow_factor;
  return (uint64_t)std::floor(c * 1048576.0);
}

Scheduler::Scheduler(const abs_config& cfg) : cfg_(cfg), N_(cfg.N), K_(cfg.K0) {
  if (cfg.k_mode == ABS_K_REPLAY && cfg.k_replay && cfg.k_replay_len > 0)
    replay_.assign(cfg.k_replay, cfg.k_replay + cfg.k_replay_len);
  cfg_.k_replay = nullptr;
  tau_.assign(N_, 0);
  ver_.assign(N_, 0);
  job_.assign(N_, 0);
  fin_.resize(N_);
  order_.resize(N_);
  // Algorithm 1, initialisation: every worker starts its first job on w^0 at time 0.
  for (int n = 0; n < N_; ++n) fin_[n] = time_ticks(cfg_, n, 0);
}

int Scheduler::select(std::vector<Upload>& out, std::string& err) {
  int K = K_;
  if (cfg_.k_mode == ABS_K_REPLAY) {
    if (t_ >= (int64_t)replay_.size()) { err = "k_replay has no entry for this round"; return ABS_E_REPLAY; }
    K = replay_[(size_t)t_];
    if (K < 1 || K > N_) { err = "k_replay entry outside [1, N]"; return ABS_E_ARG; }
    K_ = K;
  }
  for (int n = 0; n < N_; ++n) order_[n] = n;
  std::partial_sort(order_.begin(), order_.begin() + K, order_.end(), [&](int32_t x, int32_t y) {
    return fin_[x] != fin_[y] ? fin_[x] < fin_[y] : x < y;
  });
  out.clear();
  for (int a = 0; a < K; ++a) {
    const int n = order_[a];
    Upload u{n, ver_[n], (int32_t)(t_ - ver_[n]), job_[n]};
    if (u.tau > cfg_.tau_cap + 1) {
      err = "a selected worker is staler than tau_cap + 1: its model left the ring "
            "(tau_mode 2 needs a larger tau_cap)";
      return ABS_E_VERSION;
    }
    out.push_back(u);
  }
  now_ = fin_[order_[K - 1]];
  return ABS_OK;
}

// tau > tau_max^t with tau_max^t = max{1, N / K^t + a} (Eq. 4), in exact integers.
bool Scheduler::over_stale(int tau, int K) const {
  if (cfg_.tau_mode == ABS_TAU_INF) return false;
  if (cfg_.tau_mode == ABS_TAU_FIXED) return tau > cfg_.tau_cap;
  if (tau > cfg_.tau_cap) return true;
  return tau > 1 && (int64_t)tau * K > (int64_t)N_ + (int64_t)cfg_.a * K;
}

int Scheduler::threshold_floor(int K) const {
  if (cfg_.tau_mode == ABS_TAU_INF) return std::numeric_limits<int32_t>::max();
  if (cfg_.tau_mode == ABS_TAU_FIXED) return cfg_.tau_cap;
  const int64_t num = (int64_t)N_ + (int64_t)cfg_.a * K;
  int64_t fl = num >= 0 ? num / K : -((-num + K - 1) / K);
  if (fl < 1) fl = 1;
  return (int)std::min<int64_t>(fl, cfg_.tau_cap);
}

// Eq. 5 without the square root: the largest j <= N with j^2 f(w^t) <= (K^0)^2 f(w^0).
int Scheduler::next_wait_count(int K_now, double loss_t) const {
  if (cfg_.k_mode == ABS_K_FIXED) return cfg_.K0;
  int cand = 0;
  if (loss_t <= 0.0) {
    cand = N_;
  } else {
    const double rhs = (double)((int64_t)cfg_.K0 * cfg_.K0) * loss0_;
    for (int j = 1; j <= N_; ++j)
      if ((double)((int64_t)j * j) * loss_t <= rhs) cand = j;
  }
  if (cfg_.k_mode == ABS_K_ADAPTIVE) cand = std::max(K_now, cand);
  return std::min(N_, std::max(1, cand));
}

int Scheduler::complete(const std::vector<Upload>& sel, const float* worker_loss, bool have_loss,
                        std::string& err) {
  const int K = (int)sel.size();
  double loss_t = std::numeric_limits<double>::quiet_NaN();
  if (have_loss) {
    double s = 0.0;
    for (int a = 0; a < K; ++a) s += (double)worker_loss[a];
    loss_t = s / (double)K;
    if (!std::isfinite(loss_t)) { err = "non-finite minibatch loss"; return ABS_E_NONFINITE; }
    if (t_ == 0) loss0_ = loss_t;
  }
  std::vector<char>& in_sel = in_sel_;
  in_sel.assign((size_t)N_, 0);
  for (const Upload& u : sel) in_sel[(size_t)u.id] = 1;
  std::vector<int32_t>& restart = restart_;
  restart.clear();
  for (int n = 0; n < N_; ++n)
    if (!in_sel[(size_t)n] && over_stale(tau_[(size_t)n], K)) restart.push_back(n);

  int K_next = K;
  if (cfg_.k_mode == ABS_K_REPLAY) {
    if (t_ + 1 < (int64_t)replay_.size()) K_next = replay_[(size_t)(t_ + 1)];
  } else if (have_loss) {
    K_next = next_wait_count(K, loss_t);
  } else {
    K_next = cfg_.K0;
  }

  for (int32_t n : restart) in_sel[(size_t)n] = 1;
  for (int n = 0; n < N_; ++n) {
    if (in_sel[(size_t)n]) {
      ver_[(size_t)n] = t_ + 1;
      tau_[(size_t)n] = 0;
      job_[(size_t)n] += 1;
      fin_[(size_t)n] = now_ + time_ticks(cfg_, n, job_[(size_t)n]);
    } else {
      tau_[(size_t)n] += 1;
    }
  }
  uploads_ += (uint64_t)K;
  restarts_ += (uint64_t)restart.size();

  const size_t base = trace_.size();
  trace_.resize(base + (size_t)stride(), -1);
  int32_t* w = trace_.data() + base;
  const float lf = (float)loss_t;
  int32_t lbits;
  std::memcpy(&lbits, &lf, 4);
  w[0] = (int32_t)t_;
  w[1] = K;
  w[2] = threshold_floor(K);
  w[3] = (int32_t)(uint32_t)(now_ & 0xFFFFFFFFull);
  w[4] = (int32_t)(uint32_t)(now_ >> 32);
  w[5] = (int32_t)restart.size();
  w[6] = (int32_t)(uint32_t)(uploads_ & 0xFFFFFFFFull);
  w[7] = (int32_t)(uint32_t)(uploads_ >> 32);
  w[8] = (int32_t)(uint32_t)(restarts_ & 0xFFFFFFFFull);
  w[9] = (int32_t)(uint32_t)(restarts_ >> 32);
  w[10] = lbits;
  w[11] = K_next;
  int o = ABS_TRACE_HEADER;
  for (int a = 0; a < K; ++a) w[o + a] = sel[(size_t)a].id;
  o += K;
  for (int a = 0; a < K; ++a) w[o + a] = (int32_t)sel[(size_t)a].ver;
  o += K;
  for (int a = 0; a < K; ++a) w[o + a] = sel[(size_t)a].tau;
  o += K;
  for (size_t i = 0; i < restart.size(); ++i) w[o + (int)i] = restart[i];

  K_ = K_next;
  t_ += 1;
  return ABS_OK;
}

}  // namespace abs_impl
