// C-ABI of libabs: handle, configuration checks, workspace carving, the per-round
// host loop (select -> launch -> losses -> adapt), trace and model read-out.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "kernels.h"
#include "sched.h"

using namespace abs_impl;

namespace {

thread_local std::string g_create_error;

size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

// How long the host waits for a round's losses before it gives the call up with ABS_E_HIP: a round
// of the largest workload lasts a few milliseconds, so minutes mean the stream is stuck behind
// something that will not end.  ABS_MAILBOX_TIMEOUT_MS overrides the two minutes.
double mailbox_timeout_s() {
  static const double t = [] {
    const char* e = std::getenv("ABS_MAILBOX_TIMEOUT_MS");
    const double ms = e ? std::atof(e) : 0.0;
    return ms > 0.0 ? ms * 1e-3 : 120.0;
  }();
  return t;
}
double seconds_since(std::chrono::steady_clock::time_point t0) {
  return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
}

size_t param_count(const abs_config& c) {
  if (c.model == ABS_MODEL_LINEAR) return (size_t)c.dims[0];
  if (c.model == ABS_MODEL_CNN) {
    CnnPlan cp; const char* w = nullptr;
    return cnn_plan(c, cp, &w) ? cp.P : 0;
  }
  size_t p = 0;
  for (int l = 0; l < c.n_layers; ++l) p += (size_t)c.dims[l] * c.dims[l + 1] + c.dims[l + 1];
  return p;
}

// Workspace of the two regression models.
struct RegPlan {
  size_t slot_stride;   // floats
  size_t off_ring, off_dz, off_rowloss, off_rowidx, off_delta, off_lossbuf, off_eval, total;
};

bool validate(const abs_config& c, std::string& why) {
  auto bad = [&](const char* m) { why = m; return false; };
  if (c.N < 1 || c.N > ABS_MAX_WORKERS) return bad("N must be in [1, 128]");
  if (c.B < 1 || c.B > 4096) return bad("B must be in [1, 4096]");
  if (c.K0 < 1 || c.K0 > c.N) return bad("K0 must be in [1, N]");
  if (c.M < c.N) return bad("M must be at least N (every worker needs a non-empty shard)");
  if (c.M / c.N > 0xFFFFFFFFll || c.M > 0xFFFFFFFFll) return bad("M too large");
  if (c.k_mode < 0 || c.k_mode > 3) return bad("k_mode must be 0..3");
  if (c.tau_mode < 0 || c.tau_mode > 2) return bad("tau_mode must be 0..2");
  if (c.tau_cap < 0 || c.tau_cap > 1024) return bad("tau_cap must be in [0, 1024]");
  if (c.k_mode == ABS_K_REPLAY && (!c.k_replay || c.k_replay_len < 1)) return bad("k_mode 2 needs k_replay");
  if (!(c.lr > 0.f) || !std::isfinite(c.lr)) return bad("lr must be positive and finite");
  if (c.time_dist < 0 || c.time_dist > 2) return bad("time_dist must be 0..2");
  if (c.time_dist == ABS_TIME_PARETO && !(c.time_param > 0.0)) return bad("Pareto needs time_param > 0");
  if (c.n_slow < 0 || c.n_slow > c.N) return bad("n_slow must be in [0, N]");
  if (c.n_slow > 0 && !(c.slow_factor > 0.0)) return bad("slow_factor must be positive");
  if (c.U < 0 || c.U > 64) return bad("U must be in [1, 64] (0 is read as 1)");
  if (c.reserved != 0) return bad("reserved must be 0");
  if (c.profile < 0) return bad("profile must be 0, 1 or a sampling period n > 1");
  if (c.device_mode == 0 && !(c.k_mode == ABS_K_FIXED || c.k_mode == ABS_K_REPLAY))
    return bad("schedule-only mode needs k_mode 1 or 2 (there are no losses to adapt K with)");
  switch (c.model) {
    case ABS_MODEL_LINEAR:
      if (c.n_layers != 1 || c.dims[1] != 1) return bad("linear model: n_layers 1, dims {d, 1}");
      if (c.dims[0] < 1 || c.dims[0] > 512) return bad("linear model: d must be in [1, 512]");
      if (c.x_dtype != ABS_X_FP32) return bad("linear model: X must be fp32");
      break;
    case ABS_MODEL_SOFTMAX:
      if (c.n_layers != 1) return bad("softmax model: n_layers 1");
      if (c.dims[0] < 4 || c.dims[0] > 1024 || c.dims[0] % 4) return bad("softmax model: d % 4 == 0, 4 <= d <= 1024");
      if (c.dims[1] < 2 || c.dims[1] > 16) return bad("softmax model: 2 <= C <= 16");
      if (c.x_dtype != ABS_X_FP32) return bad("softmax model: X must be fp32");
      break;
    case ABS_MODEL_MLP: {
      if (c.n_layers < 2 || c.n_layers > ABS_MAX_LAYERS) return bad("MLP: 2 <= n_layers <= 7");
      if (c.x_dtype != ABS_X_BF16) return bad("MLP: X must be bf16");
      MlpPlan p;
      const char* w = nullptr;
      if (!mlp_plan(c, p, &w)) return bad(w ? w : "unsupported MLP configuration");
      break;
    }
    case ABS_MODEL_CNN: {
      CnnPlan p;
      const char* w = nullptr;
      if (!cnn_plan(c, p, &w)) return bad(w ? w : "unsupported CNN configuration");
      break;
    }
    default: return bad("model must be 0, 1, 2 or 3");
  }
  return true;
}

void reg_plan(const abs_config& c, RegPlan& p) {
  const size_t R = (size_t)c.tau_cap + 3, rows = (size_t)c.N * c.B;
  p.slot_stride = round_up(param_count(c), 64);
  size_t o = 0;
  p.off_ring = o;    o = round_up(o + R * p.slot_stride * 4, 256);
  p.off_dz = o;      o = round_up(o + rows * 16 * 4, 256);
  p.off_rowloss = o; o = round_up(o + rows * 4, 256);
  p.off_rowidx = o;  o = round_up(o + rows * 4, 256);
  p.off_delta = o;   if (c.U > 1) o = round_up(o + (size_t)c.N * p.slot_stride * 4, 256);
  p.off_lossbuf = o; if (c.U > 1) o = round_up(o + (size_t)c.N * 4, 256);
  p.off_eval = o;    o = round_up(o + eval_scratch_bytes(kEvalChunk), 256);
  p.total = o;
}

// Scratch of abs_evaluate_static: the two fp64 sums, then per-row losses and hit flags of one pass
// (laid out as eval_scratch_bytes() says).  One copy per GPU, held from the library's load to the
// process's end; the name is a host-side stand-in, device code gets the address that
// hipGetSymbolAddress reports on the device in question.
constexpr int kStaticEvalRows = ABS_STATIC_EVAL_ROWS;
constexpr size_t kStaticScratchBytes = 256 + 2 * ((size_t)kStaticEvalRows * 4);
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void* g_static_ptr[kMaxDevices] = {};

// The device's own address of g_static_scratch, resolved once per device (with that device
// current: abs_create calls this for the device the handle is created on).
hipError_t static_scratch_of_current_device(int* dev_out, void** ptr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess) return e;
    g_static_ptr[dev] = p;
  }
  *dev_out = dev;
  *ptr_out = g_static_ptr[dev];
  return hipSuccess;
}

struct NoHook : LaunchHook {
  void begin(int, double, double) override {}
  void end(int) override {}
};

struct Stat {
  int64_t launches = 0; double ms = 0, flops = 0, bytes = 0;
  int64_t timed_launches = 0; double timed_flops = 0, timed_bytes = 0;   // the launches bracketed by events
};

}  // namespace

const char* abs_impl::kernel_kind_name(int kind) {
  static const char* names[KK_COUNT] = {
      "linreg_round", "softmax_rows", "softmax_update", "mlp_index", "mlp_gather_t", "mlp_fwd_l1",
      "mlp_fwd_hidden", "mlp_fwd_logits", "mlp_logits_ce", "mlp_loss", "mlp_dgrad_out", "mlp_dgrad", "mlp_wgrad_l1", "mlp_wgrad",
      "mlp_update", "mlp_bias_loss", "local_steps", "delta_update", "evaluate", "mlp_wgrad_out",
      "cnn_conv_fwd", "cnn_dense", "cnn_dense_wgrad", "cnn_conv_bwd", "cnn_conv_wgrad", "cnn_combine"};
  return kind >= 0 && kind < KK_COUNT ? names[kind] : "?";
}

struct abs_ctx : public LaunchHook {
  abs_config cfg;
  std::unique_ptr<Scheduler> sched;
  hipStream_t stream = nullptr;
  char* ws = nullptr;
  const void* dX = nullptr;
  const void* dy = nullptr;
  size_t P = 0, slot_stride = 0, off_ring = 0;
  int R = 0;
  RegPlan rplan{};
  MlpArgs margs{};
  CnnArgs cargs{};
  LossMailbox* h_box = nullptr;   // pinned, device-visible
  LossMailbox* d_box = nullptr;   // the device's address of h_box
  int device = -1;                // the GPU the handle was created on
  void* static_scratch = nullptr; // that GPU's copy of the evaluation scratch (abs_evaluate_static)
  std::string err;
  Stat stats[KK_COUNT];
  // profile mode: one event pair per launch of the current round
  std::vector<hipEvent_t> ev;
  std::vector<int> ev_kind;
  size_t ev_used = 0;
  bool timing = false;                 // this round's launches are bracketed (profile: every round or every n-th)

  void begin(int kind, double flops, double bytes) override {
    stats[kind].launches += 1;
    stats[kind].flops += flops;
    stats[kind].bytes += bytes;
    if (timing) {
      stats[kind].timed_launches += 1;
      stats[kind].timed_flops += flops;
      stats[kind].timed_bytes += bytes;
      if (ev_used + 2 > ev.size()) {
        for (int i = 0; i < 2; ++i) { hipEvent_t e; (void)hipEventCreate(&e); ev.push_back(e); }
      }
      (void)hipEventRecord(ev[ev_used], stream);
    }
  }
  void end(int kind) override {
    if (timing) {
      (void)hipEventRecord(ev[ev_used + 1], stream);
      ev_kind.push_back(kind);
      ev_used += 2;
    }
  }
  void begin_kernel(int kind, double flops, double bytes, hipEvent_t* e0, hipEvent_t* e1) override {
    stats[kind].launches += 1;
    stats[kind].flops += flops;
    stats[kind].bytes += bytes;
    *e0 = nullptr; *e1 = nullptr;
    if (timing) {
      stats[kind].timed_launches += 1;
      stats[kind].timed_flops += flops;
      stats[kind].timed_bytes += bytes;
      if (ev_used + 2 > ev.size()) {
        for (int i = 0; i < 2; ++i) { hipEvent_t e; (void)hipEventCreate(&e); ev.push_back(e); }
      }
      *e0 = ev[ev_used]; *e1 = ev[ev_used + 1];
    }
  }
  void end_kernel(int kind) override {
    if (timing) { ev_kind.push_back(kind); ev_used += 2; }
  }
  // Spin until the device has stamped the mailbox; every so often ask the runtime whether the
  // stream has failed or drained without the stamp, and give up after mailbox_timeout_s(), so
  // neither a broken launch nor a stream that never gets to run can hang the host.
  int wait_mailbox(uint32_t stamp) {
    const auto t0 = std::chrono::steady_clock::now();
    for (uint64_t spin = 1;; ++spin) {
      if (h_box->stamp == stamp) { std::atomic_thread_fence(std::memory_order_acquire); return ABS_OK; }
      if ((spin & 0x3FFF) == 0) {
        const hipError_t q = hipStreamQuery(stream);
        if (q == hipSuccess) {
          if (h_box->stamp == stamp) return ABS_OK;
          err = "stream drained but the loss mailbox was not written";
          return ABS_E_HIP;
        }
        if (q != hipErrorNotReady) { err = std::string("hipStreamQuery: ") + hipGetErrorString(q); return ABS_E_HIP; }
        if (seconds_since(t0) > mailbox_timeout_s()) {
          err = "timed out waiting for the round's losses (the stream has not completed the round)";
          return ABS_E_HIP;
        }
      }
#if defined(__x86_64__)
      __builtin_ia32_pause();
#endif
    }
  }
  void harvest() {   // after the stream has been synchronised
    for (size_t i = 0; i < ev_kind.size(); ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) == hipSuccess) stats[ev_kind[i]].ms += ms;
    }
    ev_kind.clear();
    ev_used = 0;
  }
};

#define ABS_HIP(ctx, call)                                                        \
  do {                                                                            \
    hipError_t e_ = (call);                                                       \
    if (e_ != hipSuccess) {                                                       \
      (ctx)->err = std::string(#call) + ": " + hipGetErrorString(e_);             \
      return ABS_E_HIP;                                                           \
    }                                                                             \
  } while (0)

extern "C" {

int32_t abs_config_bytes(void) { return (int32_t)sizeof(abs_config); }

size_t abs_workspace_size(const abs_config* cfg) {
  if (!cfg) { g_create_error = "cfg is NULL"; return 0; }
  std::string why;
  if (!validate(*cfg, why)) { g_create_error = why; return 0; }
  if (cfg->model == ABS_MODEL_MLP) {
    MlpPlan p; const char* w = nullptr;
    mlp_plan(*cfg, p, &w);
    return p.total;
  }
  if (cfg->model == ABS_MODEL_CNN) {
    CnnPlan p; const char* w = nullptr;
    cnn_plan(*cfg, p, &w);
    return p.total;
  }
  RegPlan p; reg_plan(*cfg, p);
  return p.total;
}

int abs_create(const abs_config* cfg, const void* d_X, const void* d_y, const float* d_w0,
               void* d_workspace, size_t workspace_bytes, void* hip_stream, abs_ctx** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) { g_create_error = "cfg / out is NULL"; return ABS_E_ARG; }
  std::string why;
  if (!validate(*cfg, why)) { g_create_error = why; return ABS_E_ARG; }
  std::unique_ptr<abs_ctx> c(new abs_ctx());
  c->cfg = *cfg;
  if (c->cfg.U == 0) c->cfg.U = 1;
  c->sched.reset(new Scheduler(*cfg));
  c->cfg.k_replay = nullptr;
  c->P = param_count(*cfg);
  c->R = cfg->tau_cap + 3;
  c->stream = (hipStream_t)hip_stream;
  if (!cfg->device_mode) { *out = c.release(); return ABS_OK; }

  if (!d_X || !d_y || !d_w0 || !d_workspace) { g_create_error = "a device pointer is NULL"; return ABS_E_ARG; }
  if (((uintptr_t)d_workspace & 255) || ((uintptr_t)d_X & 15)) {
    g_create_error = "d_workspace must be 256-byte aligned and d_X 16-byte aligned"; return ABS_E_ARG;
  }
  const size_t need = abs_workspace_size(cfg);
  if (workspace_bytes < need) { g_create_error = "workspace too small"; return ABS_E_WORKSPACE; }
  c->ws = (char*)d_workspace;
  c->dX = d_X; c->dy = d_y;
  auto fail = [&](const char* what, hipError_t e) {
    g_create_error = std::string(what) + ": " + hipGetErrorString(e);
    if (c->h_box) (void)hipHostFree(c->h_box);
    return ABS_E_HIP;
  };
  hipError_t e = hipHostMalloc((void**)&c->h_box, sizeof(LossMailbox), hipHostMallocMapped);
  if (e != hipSuccess) { c->h_box = nullptr; return fail("hipHostMalloc", e); }
  std::memset(c->h_box, 0, sizeof(LossMailbox));
  e = hipHostGetDevicePointer((void**)&c->d_box, c->h_box, 0);
  if (e != hipSuccess) return fail("hipHostGetDevicePointer", e);

  e = static_scratch_of_current_device(&c->device, &c->static_scratch);
  if (e != hipSuccess) return fail("hipGetSymbolAddress", e);

  const uint64_t shard = (uint64_t)(cfg->M / cfg->N);
  const uint64_t bkey = stream_key(cfg->seed, kStreamBatch);
  if (cfg->model == ABS_MODEL_MLP) {
    const char* w = nullptr;
    mlp_plan(*cfg, c->margs.plan, &w);
    c->margs.ws = c->ws;
    c->margs.X = (const uint16_t*)d_X;
    c->margs.y = (const int32_t*)d_y;
    c->margs.shard_rows = shard;
    c->margs.batch_key = bkey;
    c->margs.mailbox = c->d_box;
    c->slot_stride = c->margs.plan.slot_stride;
    c->off_ring = c->margs.plan.off_ring;
  } else if (cfg->model == ABS_MODEL_CNN) {
    const char* w = nullptr;
    cnn_plan(*cfg, c->cargs.plan, &w);
    c->cargs.ws = c->ws;
    c->cargs.X = (const float*)d_X;
    c->cargs.y = (const int32_t*)d_y;
    c->cargs.shard_rows = shard;
    c->cargs.batch_key = bkey;
    c->cargs.mailbox = c->d_box;
    c->slot_stride = c->cargs.plan.slot_stride;
    c->off_ring = c->cargs.plan.off_ring;
    e = cnn_prepare();
    if (e != hipSuccess) return fail("hipFuncSetAttribute", e);
  } else {
    reg_plan(*cfg, c->rplan);
    c->slot_stride = c->rplan.slot_stride;
    c->off_ring = c->rplan.off_ring;
  }
  // w^0 into ring slot 0 (Algorithm 1, initialisation)
  e = hipMemcpyAsync(c->ws + c->off_ring, d_w0, c->P * sizeof(float), hipMemcpyDeviceToDevice, c->stream);
  if (e != hipSuccess) return fail("hipMemcpyAsync(w0)", e);
  if (cfg->model == ABS_MODEL_MLP) {
    e = mlp_prepare(c->margs, c->stream);
    if (e != hipSuccess) return fail("mlp_prepare", e);
  }
  e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return fail("hipStreamSynchronize", e);
  *out = c.release();
  return ABS_OK;
}

// The device's view of round t of one simulation: the K^t uploads with the ring slot of their model
// version and their coefficient in Eq. 3.  Regression models: in arrival order.  MLP: grouped by
// model version (oldest first, arrival order inside a version), so that the stacked rows of the
// uploads that computed at the same w^{t - tau} are contiguous - neighbouring tiles of the forward
// and input-gradient products then share their weight operand (Eq. 2 evaluated per version) - and
// Eq. 3's sum runs in that order; pos_of[a] = position of the a-th arrival (the trace and the
// scheduler keep arrival order).
static void fill_round_desc(const abs_ctx* ctx, const std::vector<Upload>& sel, int64_t t, RoundDesc& rd,
                            int* pos_of = nullptr) {
  const abs_config& cfg = ctx->cfg;
  const int K = (int)sel.size();
  rd.K = K;
  rd.slot_cur = (uint32_t)(t % ctx->R);
  rd.slot_next = (uint32_t)((t + 1) % ctx->R);
  rd.stamp = (uint32_t)(t + 1);
  int order[ABS_MAX_WORKERS];
  for (int a = 0; a < K; ++a) order[a] = a;
  if (cfg.model == ABS_MODEL_MLP)
    std::stable_sort(order, order + K, [&](int x, int y) { return sel[(size_t)x].ver < sel[(size_t)y].ver; });
  for (int pos = 0; pos < K; ++pos) {
    const Upload& u = sel[(size_t)order[pos]];
    if (pos_of) pos_of[order[pos]] = pos;
    // coefficient of this upload in Eq. 3: eta_k / (K^t B), eta_k = eta / max(1, tau_k) under
    // the staleness-aware penalty
    double eta = (double)cfg.lr;
    if (cfg.sa_penalty && u.tau > 1) eta /= (double)u.tau;
    rd.w[pos].id = (uint32_t)u.id;
    rd.w[pos].job = u.job;
    rd.w[pos].slot = (uint32_t)(u.ver % ctx->R);
    // (with U > 1 the 1/K^t of Eq. 3 is applied when the uploads' changes are averaged)
    rd.w[pos].c = cfg.U > 1 ? (float)(eta / (double)cfg.B) : (float)(eta / ((double)K * (double)cfg.B));
  }
}

static void fill_regression_args(const abs_ctx* ctx, RegressionArgs& ra) {
  const abs_config& cfg = ctx->cfg;
  ra.X = (const float*)ctx->dX;
  ra.y = ctx->dy;
  ra.ring = (float*)(ctx->ws + ctx->rplan.off_ring);
  ra.slot_stride = ctx->slot_stride;
  ra.d = cfg.dims[0];
  ra.C = cfg.dims[1];
  ra.B = cfg.B;
  ra.shard_rows = (uint64_t)(cfg.M / cfg.N);
  ra.batch_key = stream_key(cfg.seed, kStreamBatch);
  ra.mailbox = ctx->d_box;
  ra.dz = (float*)(ctx->ws + ctx->rplan.off_dz);
  ra.rowloss = (float*)(ctx->ws + ctx->rplan.off_rowloss);
  ra.rowidx = (uint32_t*)(ctx->ws + ctx->rplan.off_rowidx);
  ra.U = cfg.U;
  ra.delta = (float*)(ctx->ws + ctx->rplan.off_delta);
  ra.lossbuf = (float*)(ctx->ws + ctx->rplan.off_lossbuf);
}

int abs_round(abs_ctx* ctx, int32_t n_rounds) {
  if (!ctx || n_rounds < 0) return ABS_E_ARG;
  const abs_config& cfg = ctx->cfg;
  std::vector<Upload> sel;
  RoundDesc rd;
  std::memset(&rd, 0, sizeof(rd));
  for (int32_t it = 0; it < n_rounds; ++it) {
    int rc = ctx->sched->select(sel, ctx->err);
    if (rc != ABS_OK) return rc;
    const int64_t t = ctx->sched->round();
    const int K = (int)sel.size();
    if (!cfg.device_mode) {
      rc = ctx->sched->complete(sel, nullptr, false, ctx->err);
      if (rc != ABS_OK) return rc;
      continue;
    }
    int pos_of[ABS_MAX_WORKERS];
    fill_round_desc(ctx, sel, t, rd, pos_of);
    ctx->timing = cfg.profile == 1 || (cfg.profile > 1 && t % cfg.profile == 0);
    hipError_t e;
    if (cfg.model == ABS_MODEL_MLP) {
      e = launch_mlp_round(ctx->margs, rd, ctx->stream, ctx);
    } else if (cfg.model == ABS_MODEL_CNN) {
      e = launch_cnn_round(ctx->cargs, rd, ctx->stream, ctx);
    } else {
      RegressionArgs ra;
      fill_regression_args(ctx, ra);
      if (cfg.U > 1)
        e = launch_regression_local_round(ra, rd, cfg.model == ABS_MODEL_SOFTMAX, ctx->stream, ctx);
      else
        e = cfg.model == ABS_MODEL_LINEAR ? launch_linreg_round(ra, rd, ctx->stream, ctx)
                                          : launch_softmax_round(ra, rd, ctx->stream, ctx);
    }
    if (e != hipSuccess) { ctx->err = std::string("kernel launch: ") + hipGetErrorString(e); return ABS_E_HIP; }
    // Eq. 5 needs this round's losses before the next round can be selected.  They arrive in
    // the mailbox as soon as the forward pass is through (the stamp is written last), so the
    // host prepares and enqueues round t+1 while the device still works on round t; stream
    // order keeps the rounds apart on the device.
    rc = ctx->wait_mailbox(rd.stamp);
    if (rc != ABS_OK) return rc;
    // profile mode: the rounds' events are read back in batches, after draining the stream
    if (cfg.profile && (ctx->ev_kind.size() >= 512 || it + 1 == n_rounds)) {
      ABS_HIP(ctx, hipStreamSynchronize(ctx->stream));
      ctx->harvest();
    }
    float losses[ABS_MAX_WORKERS];
    for (int a = 0; a < K; ++a) losses[a] = ctx->h_box->loss[pos_of[a]];
    rc = ctx->sched->complete(sel, losses, true, ctx->err);
    if (rc != ABS_OK) return rc;
  }
  return ABS_OK;
}

// ---- batched simulations: S handles of one shape advance together, one set of launches per round
constexpr int kBatchGroups = 4;            // a large batch advances as up to this many groups
struct abs_batch {
  std::vector<abs_ctx*> ctx;
  hipStream_t stream = nullptr;            // the handles' stream
  hipStream_t own[kBatchGroups - 1] = {};  // the library's own, for the further groups of a large batch
  hipEvent_t ev_in = nullptr, ev_out[kBatchGroups - 1] = {};   // order them after / before the handles' stream
  RegressionArgs* d_args = nullptr;        // device [S]
  char* h_rds[2] = {nullptr, nullptr};     // pinned host, S descriptors, alternating by round
  char* d_rds[2] = {nullptr, nullptr};     // device copies
  size_t rd_stride = 0;
  LossMailbox* h_box = nullptr;            // pinned, device-visible [S]
  LossMailbox* d_box = nullptr;
  char* d_slots = nullptr;                 // softmax: per-upload gradient slots and losses of all simulations
  uint64_t rounds = 0;
  std::string err;
};
namespace { thread_local std::string g_batch_error; }

void abs_batch_destroy(abs_batch* b) {
  if (!b) return;
  if (b->stream || !b->ctx.empty()) (void)hipStreamSynchronize(b->stream);
  for (hipStream_t s : b->own) if (s) { (void)hipStreamSynchronize(s); (void)hipStreamDestroy(s); }
  if (b->ev_in) (void)hipEventDestroy(b->ev_in);
  for (hipEvent_t e : b->ev_out) if (e) (void)hipEventDestroy(e);
  for (int i = 0; i < 2; ++i)
    if (b->h_rds[i]) (void)hipHostFree(b->h_rds[i]);
  if (b->h_box) (void)hipHostFree(b->h_box);
  delete b;          // (the device memory is the caller's workspace)
}

namespace {
// Checks that the handles can form a batch; the message of the first problem otherwise.
// models whose round is a chain of launches of their own (batches run them side by side on streams)
bool chain_model(int model) { return model == ABS_MODEL_MLP || model == ABS_MODEL_CNN; }
const char* batch_problem(abs_ctx** ctxs, int32_t n) {
  if (!ctxs) return "NULL argument";
  if (n < 1 || n > 4096) return "a batch holds 1..4096 simulations";
  const abs_ctx* c0 = ctxs[0];
  for (int32_t i = 0; i < n; ++i) {
    const abs_ctx* c = ctxs[i];
    if (!c) return "NULL handle in the batch";
    for (int32_t j = 0; j < i; ++j) if (ctxs[j] == c) return "a handle appears twice in the batch";
    if (!c->cfg.device_mode) return "schedule-only handles cannot be batched";
    if (c->cfg.profile) return "batched rounds are not profiled per kernel (profile must be 0)";
    if (c->cfg.model != c0->cfg.model || c->cfg.dims[0] != c0->cfg.dims[0] || c->cfg.dims[1] != c0->cfg.dims[1] ||
        c->cfg.B != c0->cfg.B || c->cfg.N != c0->cfg.N || c->cfg.U != c0->cfg.U || c->stream != c0->stream)
      return "all simulations of a batch need the same model, dims, N, B, U and stream";
  }
  return nullptr;
}
// Device memory of a batch of n handles shaped like c0, carved from the caller's workspace: the
// per-simulation kernel arguments, two copies of the round descriptors (alternating by round) and,
// for softmax rounds that keep one gradient per upload, N slots and N losses per simulation.
struct BatchPlan { size_t rd_stride, off_args, off_rds[2], off_slots, slot_floats, sim_floats, total; bool slots; };
BatchPlan batch_plan(const abs_ctx* c0, int32_t n) {
  BatchPlan p{};
  p.rd_stride = 16 + (size_t)c0->cfg.N * sizeof(WorkerDesc);
  if (chain_model(c0->cfg.model)) return p;      // MLP / CNN simulations keep their own launches and workspaces
  size_t o = 0;
  p.off_args = o; o = round_up(o + (size_t)n * sizeof(RegressionArgs), 256);
  for (int i = 0; i < 2; ++i) { p.off_rds[i] = o; o = round_up(o + (size_t)n * p.rd_stride, 256); }
  p.slot_floats = (size_t)c0->cfg.N * c0->slot_stride;
  p.sim_floats = p.slot_floats + round_up((size_t)c0->cfg.N, 64);
  p.slots = c0->cfg.U == 1 && regression_batch_uses_slots(c0->cfg.model == ABS_MODEL_SOFTMAX, c0->cfg.B);
  p.off_slots = o; if (p.slots) o = round_up(o + (size_t)n * p.sim_floats * sizeof(float), 256);
  p.total = o;
  return p;
}
}  // namespace

size_t abs_batch_workspace_size(abs_ctx** ctxs, int32_t n) {
  if (const char* why = batch_problem(ctxs, n)) { g_batch_error = why; return 0; }
  return batch_plan(ctxs[0], n).total;
}

int abs_batch_create(abs_ctx** ctxs, int32_t n, void* d_workspace, size_t workspace_bytes, abs_batch** out) {
  if (out) *out = nullptr;
  auto bad = [&](const char* m) { g_batch_error = m; return ABS_E_ARG; };
  if (!out) return bad("NULL argument");
  if (const char* why = batch_problem(ctxs, n)) return bad(why);
  const abs_ctx* c0 = ctxs[0];
  const BatchPlan plan = batch_plan(c0, n);
  if (plan.total) {
    if (!d_workspace || ((uintptr_t)d_workspace & 255)) return bad("d_workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < plan.total) { g_batch_error = "workspace smaller than abs_batch_workspace_size()"; return ABS_E_WORKSPACE; }
  }
  std::unique_ptr<abs_batch, void (*)(abs_batch*)> b(new abs_batch, abs_batch_destroy);
  b->ctx.assign(ctxs, ctxs + n);
  b->stream = c0->stream;
  b->rd_stride = plan.rd_stride;
  auto hip = [&](hipError_t e, const char* what) {
    if (e == hipSuccess) return true;
    g_batch_error = std::string(what) + ": " + hipGetErrorString(e);
    return false;
  };
  if (!hip(hipEventCreateWithFlags(&b->ev_in, hipEventDisableTiming), "hipEventCreateWithFlags")) return ABS_E_HIP;
  for (int i = 0; i < kBatchGroups - 1; ++i) {
    if (!hip(hipStreamCreateWithFlags(&b->own[i], hipStreamNonBlocking), "hipStreamCreateWithFlags")) return ABS_E_HIP;
    if (!hip(hipEventCreateWithFlags(&b->ev_out[i], hipEventDisableTiming), "hipEventCreateWithFlags")) return ABS_E_HIP;
  }
  // MLP simulations keep their own launches, workspaces and mailboxes: the batch only runs them
  // side by side (abs_batch_round)
  if (chain_model(c0->cfg.model)) { *out = b.release(); return ABS_OK; }
  char* ws = (char*)d_workspace;
  b->d_args = (RegressionArgs*)(ws + plan.off_args);
  for (int i = 0; i < 2; ++i) {
    if (!hip(hipHostMalloc((void**)&b->h_rds[i], (size_t)n * b->rd_stride, hipHostMallocDefault), "hipHostMalloc")) return ABS_E_HIP;
    b->d_rds[i] = ws + plan.off_rds[i];
  }
  if (!hip(hipHostMalloc((void**)&b->h_box, (size_t)n * sizeof(LossMailbox), hipHostMallocMapped), "hipHostMalloc")) return ABS_E_HIP;
  std::memset(b->h_box, 0, (size_t)n * sizeof(LossMailbox));
  if (!hip(hipHostGetDevicePointer((void**)&b->d_box, b->h_box, 0), "hipHostGetDevicePointer")) return ABS_E_HIP;
  if (plan.slots) b->d_slots = ws + plan.off_slots;
  std::vector<RegressionArgs> args((size_t)n);
  for (int32_t i = 0; i < n; ++i) {
    fill_regression_args(ctxs[i], args[(size_t)i]);
    args[(size_t)i].mailbox = b->d_box + i;          // the batch's own mailboxes
    if (b->d_slots) {
      args[(size_t)i].delta = (float*)b->d_slots + (size_t)i * plan.sim_floats;
      args[(size_t)i].lossbuf = args[(size_t)i].delta + plan.slot_floats;
    }
  }
  if (!hip(hipMemcpyAsync(b->d_args, args.data(), (size_t)n * sizeof(RegressionArgs), hipMemcpyHostToDevice, b->stream), "hipMemcpyAsync")) return ABS_E_HIP;
  if (!hip(hipStreamSynchronize(b->stream), "hipStreamSynchronize")) return ABS_E_HIP;
  *out = b.release();
  return ABS_OK;
}

// The host part of a batched round (select, descriptor, mailbox, Eq. 4-6 per simulation) is
// independent per simulation, so large batches spread it over a few threads that live for the
// duration of the call: thread k owns simulations lo + k, lo + k + T, ... of the group [lo, hi) in
// hand.  A round of a group has two parallel phases around the launch; workers spin on a phase
// counter (a round lasts tens of microseconds).
namespace {
struct BatchRoundState {
  abs_batch* b;
  int S, T;
  std::vector<std::vector<Upload>> sel;
  std::vector<uint32_t> stamp;
  std::vector<int> kmax, rc, bad_sim;          // per thread
  std::atomic<int> phase{0};                   // bumped for every parallel phase; `kind` says which
  int kind = 0;                                // 0: prepare, 1: finish, -1: exit (written before the bump)
  int lo = 0, hi = 0;                          // the group of simulations this phase is about
  std::atomic<int> done{0};
  std::atomic<bool> abort{false};
  int buf = 0;

  // Thread 0, now and then while mailboxes are awaited: has the stream failed?  (A stream that has
  // drained has written every mailbox, so only a runtime error ends the wait.)
  std::chrono::steady_clock::time_point wait_t0;   // set by run() at the start of a finish phase
  bool stream_failed() {
    if (seconds_since(wait_t0) > mailbox_timeout_s()) {
      b->err = "timed out waiting for the round's losses (a stream has not completed the round)";
      rc[0] = ABS_E_HIP; bad_sim[0] = -1;
      abort.store(true);
      return true;
    }
    hipError_t q = hipStreamQuery(b->stream);
    for (hipStream_t s : b->own)
      if (q == hipSuccess || q == hipErrorNotReady) q = hipStreamQuery(s);
    if (q == hipSuccess || q == hipErrorNotReady) return false;
    b->err = std::string("hipStreamQuery: ") + hipGetErrorString(q);
    rc[0] = ABS_E_HIP; bad_sim[0] = -1;
    abort.store(true);
    return true;
  }
  void prepare(int k) {                        // select the uploads, write the descriptors
    int km = 0;
    for (int i = lo + k; i < hi; i += T) {
      abs_ctx* ctx = b->ctx[(size_t)i];
      const int r = ctx->sched->select(sel[(size_t)i], ctx->err);
      if (r != ABS_OK) { if (rc[(size_t)k] == ABS_OK) { rc[(size_t)k] = r; bad_sim[(size_t)k] = i; } continue; }
      RoundDesc rd;
      fill_round_desc(ctx, sel[(size_t)i], ctx->sched->round(), rd);
      std::memcpy(b->h_rds[buf] + (size_t)i * b->rd_stride, &rd, 16 + (size_t)rd.K * sizeof(WorkerDesc));
      stamp[(size_t)i] = rd.stamp;
      km = std::max(km, (int)rd.K);
    }
    kmax[(size_t)k] = km;
  }
  void finish(int k) {                         // wait for the losses, apply Eq. 4-6
    for (int i = lo + k; i < hi; i += T) {
      const volatile LossMailbox* box = b->h_box + i;
      for (uint64_t spin = 1; box->stamp != stamp[(size_t)i]; ++spin) {
        if (abort.load(std::memory_order_relaxed)) return;
        if (k == 0 && (spin & 0x3FFF) == 0 && stream_failed()) return;
#if defined(__x86_64__)
        __builtin_ia32_pause();
#endif
      }
      std::atomic_thread_fence(std::memory_order_acquire);
      abs_ctx* ctx = b->ctx[(size_t)i];
      float losses[ABS_MAX_WORKERS];
      const int K = (int)sel[(size_t)i].size();
      for (int a = 0; a < K; ++a) losses[a] = b->h_box[i].loss[a];
      const int r = ctx->sched->complete(sel[(size_t)i], losses, true, ctx->err);
      if (r != ABS_OK && rc[(size_t)k] == ABS_OK) { rc[(size_t)k] = r; bad_sim[(size_t)k] = i; }
    }
  }
  void worker(int k) {
    int seen = 0;
    for (;;) {
      int p;
      while ((p = phase.load(std::memory_order_acquire)) == seen) {
#if defined(__x86_64__)
        __builtin_ia32_pause();
#endif
      }
      if (kind < 0) return;
      seen = p;
      if (kind == 0) prepare(k); else finish(k);
      done.fetch_add(1, std::memory_order_release);
    }
  }
  // run one phase for simulations [lo_, hi_) on all threads (this one is thread 0); returns the
  // first failing simulation's code
  int run(int kind_, int lo_, int hi_) {
    done.store(0, std::memory_order_relaxed);
    wait_t0 = std::chrono::steady_clock::now();
    kind = kind_; lo = lo_; hi = hi_;
    phase.fetch_add(1, std::memory_order_release);
    if (kind_ == 0) prepare(0); else finish(0);
    for (uint64_t spin = 1; done.load(std::memory_order_acquire) != T - 1; ++spin) {
      if (kind_ == 1 && (spin & 0x3FFF) == 0 && !abort.load()) stream_failed();   // the others may still wait for mailboxes
#if defined(__x86_64__)
      __builtin_ia32_pause();
#endif
    }
    int first = -2, code = ABS_OK;
    for (int k = 0; k < T; ++k)
      if (rc[(size_t)k] != ABS_OK && (first == -2 || bad_sim[(size_t)k] < first)) { first = bad_sim[(size_t)k]; code = rc[(size_t)k]; }
    if (code != ABS_OK && first >= 0) b->err = "simulation " + std::to_string(first) + ": " + b->ctx[(size_t)first]->err;
    return code;
  }
};
}  // namespace

// MLP simulations of a batch: a round of one is a chain of launches that leaves much of the device
// idle unless the layers are wide (3072-512-10: one workgroup per CU in its largest product), so up
// to kBatchGroups simulations run side by side, each through abs_round on a stream of its own and a
// host thread of its own; further simulations follow on the stream that gets free.
static int batch_round_mlp(abs_batch* b, int32_t n_rounds) {
  const int S = (int)b->ctx.size(), T = std::min(S, kBatchGroups);
  hipError_t e = T > 1 ? hipEventRecord(b->ev_in, b->stream) : hipSuccess;
  for (int k = 1; k < T && e == hipSuccess; ++k) e = hipStreamWaitEvent(b->own[k - 1], b->ev_in, 0);
  if (e != hipSuccess) { b->err = std::string("hipStreamWaitEvent: ") + hipGetErrorString(e); return ABS_E_HIP; }
  std::vector<int> rc((size_t)S, ABS_OK);
  auto work = [&](int k) {
    const hipStream_t s = k == 0 ? b->stream : b->own[k - 1];
    for (int i = k; i < S; i += T) {
      abs_ctx* c = b->ctx[(size_t)i];
      const hipStream_t keep = c->stream;
      c->stream = s;
      rc[(size_t)i] = abs_round(c, n_rounds);
      c->stream = keep;
    }
  };
  std::vector<std::thread> pool;
  for (int k = 1; k < T; ++k) pool.emplace_back(work, k);
  work(0);
  for (std::thread& t : pool) t.join();
  for (int k = 1; k < T && e == hipSuccess; ++k) {
    e = hipEventRecord(b->ev_out[k - 1], b->own[k - 1]);
    if (e == hipSuccess) e = hipStreamWaitEvent(b->stream, b->ev_out[k - 1], 0);
  }
  for (int i = 0; i < S; ++i)
    if (rc[(size_t)i] != ABS_OK) {
      b->err = "simulation " + std::to_string(i) + ": " + b->ctx[(size_t)i]->err;
      return rc[(size_t)i];
    }
  if (e != hipSuccess) { b->err = std::string("hipStreamWaitEvent: ") + hipGetErrorString(e); return ABS_E_HIP; }
  b->rounds += (uint64_t)n_rounds;
  return ABS_OK;
}

int abs_batch_round(abs_batch* b, int32_t n_rounds) {
  if (!b || n_rounds < 0) return ABS_E_ARG;
  const int S = (int)b->ctx.size();
  const abs_config& c0 = b->ctx[0]->cfg;
  if (chain_model(c0.model)) return batch_round_mlp(b, n_rounds);
  BatchRoundState st;
  st.b = b;
  st.S = S;
  st.T = std::max(1, std::min({8, S / 32, (int)std::thread::hardware_concurrency() / 2}));
  st.sel.resize((size_t)S);
  st.stamp.resize((size_t)S);
  st.kmax.assign((size_t)st.T, 0);
  st.rc.assign((size_t)st.T, ABS_OK);
  st.bad_sim.assign((size_t)st.T, -1);
  // Large batches advance as G groups, staggered in time: while the device works on one group's
  // round the host finishes and prepares another's (Eq. 5 makes a simulation's next selection wait
  // for its own losses, not for the other groups').
  // A linear round is one workgroup per simulation and lasts as long for 32 of them as for 256:
  // groups only pay from two workgroups per CU on.
  // The further groups' copies and kernels go to streams of their own (ordered after what the
  // handles' stream held at entry, and before what it gets after the call), so that the device
  // fills the tail of one group's kernel with the head of another's.
  const bool softmax = c0.model == ABS_MODEL_SOFTMAX;
  // (softmax, 784 x 10, N = 16: 8 simulations 3.7 -> 4.0, 16: 6.1 -> 7.1 M worker-gradients/s with two groups,
  // 64: 9.0 -> 17.5 M with three, 128 and more: 12.5 -> 20 M with four; linear, d = 100, N = 8:
  // 32 simulations 6.1 -> 7.0 M with two, 128: 13.0 -> 20.6 M, 1024: 38.4 -> 47.7 M, four groups lose)
  const int G = softmax ? (S >= 128 ? 4 : S >= 64 ? 3 : S >= 4 ? 2 : 1) : (S >= 32 ? 2 : 1);
  int lo[kBatchGroups], hi[kBatchGroups];
  hipStream_t gstream[kBatchGroups];
  for (int g = 0; g < G; ++g) {
    lo[g] = (int)((long)S * g / G); hi[g] = (int)((long)S * (g + 1) / G);
    gstream[g] = g == 0 ? b->stream : b->own[g - 1];
  }
  if (G > 1 && n_rounds > 0) {
    hipError_t e = hipEventRecord(b->ev_in, b->stream);
    for (int g = 1; g < G && e == hipSuccess; ++g) e = hipStreamWaitEvent(gstream[g], b->ev_in, 0);
    if (e != hipSuccess) { b->err = std::string("hipStreamWaitEvent: ") + hipGetErrorString(e); return ABS_E_HIP; }
  }
  std::vector<std::thread> pool;            // from here on every path joins them
  for (int k = 1; k < st.T; ++k) pool.emplace_back([&st, k] { st.worker(k); });
  bool inflight[kBatchGroups] = {};
  auto finish = [&](int g) {
    inflight[g] = false;
    return st.run(1, lo[g], hi[g]);
  };
  auto start = [&](int g) {
    int r = st.run(0, lo[g], hi[g]);
    if (r != ABS_OK) return r;
    int Kmax = 0;
    for (int k = 0; k < st.T; ++k) Kmax = std::max(Kmax, st.kmax[(size_t)k]);
    const size_t off = (size_t)lo[g] * b->rd_stride, n = (size_t)(hi[g] - lo[g]);
    hipError_t e = hipMemcpyAsync(b->d_rds[st.buf] + off, b->h_rds[st.buf] + off, n * b->rd_stride, hipMemcpyHostToDevice, gstream[g]);
    if (e == hipSuccess && c0.U > 1)
      e = launch_regression_local_round_batch(b->d_args + lo[g], b->d_rds[st.buf] + off, b->rd_stride, (int)n, softmax,
                                              c0.dims[0], c0.dims[1], c0.B, c0.U, Kmax, gstream[g]);
    else if (e == hipSuccess)
      e = launch_regression_round_batch(b->d_args + lo[g], b->d_rds[st.buf] + off, b->rd_stride, (int)n, softmax,
                                        c0.dims[0], c0.dims[1], c0.B, Kmax, b->d_slots != nullptr, gstream[g]);
    if (e != hipSuccess) { b->err = std::string("launch: ") + hipGetErrorString(e); return (int)ABS_E_HIP; }
    inflight[g] = true;
    return (int)ABS_OK;
  };
  int rc = ABS_OK;
  for (int32_t it = 0; it < n_rounds && rc == ABS_OK; ++it) {
    st.buf = (int)(it & 1);
    for (int g = 0; g < G && rc == ABS_OK; ++g) {
      if (inflight[g]) rc = finish(g);
      if (rc == ABS_OK) rc = start(g);
    }
    if (rc == ABS_OK) b->rounds += 1;
  }
  // rounds still on the device are completed also after an error (their uploads are selected and
  // their kernels enqueued); the first error is the one reported
  for (int g = 0; g < G; ++g) {
    if (!inflight[g]) continue;
    const std::string first = b->err;
    const int r = finish(g);
    if (rc == ABS_OK) rc = r; else b->err = first;
  }
  st.kind = -1;
  st.phase.fetch_add(1, std::memory_order_release);
  for (std::thread& t : pool) t.join();
  if (G > 1 && n_rounds > 0) {
    hipError_t e = hipSuccess;
    for (int g = 1; g < G && e == hipSuccess; ++g) {
      e = hipEventRecord(b->ev_out[g - 1], gstream[g]);
      if (e == hipSuccess) e = hipStreamWaitEvent(b->stream, b->ev_out[g - 1], 0);
    }
    if (e != hipSuccess && rc == ABS_OK) { b->err = std::string("hipStreamWaitEvent: ") + hipGetErrorString(e); rc = ABS_E_HIP; }
  }
  return rc;
}

const char* abs_batch_last_error(const abs_batch* b) { return b ? b->err.c_str() : g_batch_error.c_str(); }

int abs_get_model(abs_ctx* ctx, int64_t version, float* h_out, size_t n_floats) {
  if (!ctx || !h_out) return ABS_E_ARG;
  if (!ctx->cfg.device_mode) { ctx->err = "no model in schedule-only mode"; return ABS_E_ARG; }
  if (n_floats != ctx->P) { ctx->err = "n_floats must equal the parameter count"; return ABS_E_ARG; }
  const int64_t t = ctx->sched->round();
  if (version < 0) version = t;
  if (version > t || version < t - (ctx->R - 1) + 0 || version < 0) {
    ctx->err = "model version not in the ring"; return ABS_E_VERSION;
  }
  const char* src = ctx->ws + ctx->off_ring + (size_t)(version % ctx->R) * ctx->slot_stride * sizeof(float);
  ABS_HIP(ctx, hipMemcpyAsync(h_out, src, n_floats * sizeof(float), hipMemcpyDeviceToHost, ctx->stream));
  ABS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return ABS_OK;
}

// Checks the arguments common to both evaluation calls and enqueues the passes: per-row losses and
// hit flags into `scratch` (layout of eval_scratch_bytes(cap)), their fp64 sums into its first 16 bytes.
static int enqueue_evaluation(abs_ctx* ctx, int64_t version, const void* d_X, const void* d_y, int64_t n_rows,
                              char* scratch, LaunchHook* hook, EvalArgs& e) {
  if (!ctx->cfg.device_mode) { ctx->err = "no model in schedule-only mode"; return ABS_E_ARG; }
  if (!d_X || !d_y) { ctx->err = "evaluation set pointers are NULL"; return ABS_E_ARG; }
  if (n_rows < 1 || n_rows > 0xFFFFFFFFll) { ctx->err = "n_rows must be in [1, 2^32)"; return ABS_E_ARG; }
  const int64_t t = ctx->sched->round();
  if (version < 0) version = t;
  if (version > t || version < t - (ctx->R - 1) || version < 0) {
    ctx->err = "model version not in the ring"; return ABS_E_VERSION;
  }
  const abs_config& cfg = ctx->cfg;
  const uint32_t slot = (uint32_t)(version % ctx->R);
  const bool mlp = cfg.model == ABS_MODEL_MLP, cnn = cfg.model == ABS_MODEL_CNN;
  e.X = d_X; e.y = d_y; e.n_rows = n_rows;
  e.cap = mlp ? ctx->margs.plan.Mp : cnn ? ctx->cargs.plan.N * ctx->cargs.plan.B : kEvalChunk;
  e.acc = (double*)scratch;
  e.rowloss = (float*)(scratch + 256);
  e.correct = (float*)(scratch + 256 + ((size_t)e.cap * 4 + 255) / 256 * 256);
  hipError_t err;
  if (mlp) {
    err = launch_mlp_eval(ctx->margs, slot, e, ctx->stream, hook);
  } else if (cnn) {
    err = launch_cnn_eval(ctx->cargs, slot, e, ctx->stream, hook);
  } else {
    const float* w = (const float*)(ctx->ws + ctx->off_ring) + (size_t)slot * ctx->slot_stride;
    err = launch_regression_eval(w, cfg.dims[0], cfg.dims[1], cfg.model == ABS_MODEL_SOFTMAX, e, ctx->stream, hook);
  }
  if (err != hipSuccess) { ctx->err = std::string("kernel launch: ") + hipGetErrorString(err); return ABS_E_HIP; }
  return ABS_OK;
}

int abs_evaluate(abs_ctx* ctx, int64_t version, const void* d_X, const void* d_y, int64_t n_rows,
                 double* h_loss, double* h_accuracy) {
  if (!ctx || !h_loss || !h_accuracy) return ABS_E_ARG;
  const bool mlp = ctx->cfg.model == ABS_MODEL_MLP, cnn = ctx->cfg.model == ABS_MODEL_CNN;
  char* scratch = ctx->ws ? ctx->ws + (mlp ? ctx->margs.plan.off_eval : cnn ? ctx->cargs.plan.off_eval : ctx->rplan.off_eval) : nullptr;
  EvalArgs e;
  const int rc = enqueue_evaluation(ctx, version, d_X, d_y, n_rows, scratch, ctx, e);
  if (rc != ABS_OK) return rc;
  double acc[2];
  ABS_HIP(ctx, hipMemcpyAsync(acc, e.acc, sizeof(acc), hipMemcpyDeviceToHost, ctx->stream));
  ABS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  if (ctx->cfg.profile) ctx->harvest();
  *h_loss = acc[0] / (double)n_rows;
  *h_accuracy = ctx->cfg.model == ABS_MODEL_LINEAR ? std::nan("") : acc[1] / (double)n_rows;
  return ABS_OK;
}

int abs_evaluate_static(abs_ctx* ctx, int64_t version, const void* d_X, const void* d_y, int64_t n_rows,
                        double* d_out) {
  if (!ctx || !d_out) return ABS_E_ARG;
  const long pass_rows = !ctx->cfg.device_mode ? 0
                         : ctx->cfg.model == ABS_MODEL_MLP ? (long)ctx->margs.plan.Mp
                         : ctx->cfg.model == ABS_MODEL_CNN ? (long)ctx->cargs.plan.N * ctx->cargs.plan.B : 0;
  if (pass_rows > kStaticEvalRows) {
    ctx->err = "abs_evaluate_static: a pass of this handle is N x B (MLP: B rounded up to 128) = " +
               std::to_string(pass_rows) + " rows, more than the " + std::to_string(kStaticEvalRows) +
               " rows (ABS_STATIC_EVAL_ROWS) the library's fixed scratch holds; use abs_evaluate";
    return ABS_E_WORKSPACE;
  }
  NoHook quiet;      // no per-kernel events here: creating one would allocate
  EvalArgs e;
  const int rc = enqueue_evaluation(ctx, version, d_X, d_y, n_rows, (char*)ctx->static_scratch, &quiet, e);
  if (rc != ABS_OK) return rc;
  const hipError_t err = launch_eval_finish(e, ctx->cfg.model == ABS_MODEL_LINEAR, d_out, ctx->stream);
  if (err != hipSuccess) { ctx->err = std::string("kernel launch: ") + hipGetErrorString(err); return ABS_E_HIP; }
  return ABS_OK;
}

int abs_trace(abs_ctx* ctx, int64_t round_lo, int64_t round_hi, int32_t* h_out, size_t cap_words,
              size_t* words_written) {
  if (words_written) *words_written = 0;
  if (!ctx || !h_out) return ABS_E_ARG;
  const int64_t t = ctx->sched->round();
  if (round_lo < 0 || round_hi < round_lo || round_hi > t) { ctx->err = "round range outside [0, rounds done]"; return ABS_E_ARG; }
  const size_t stride = (size_t)ctx->sched->stride();
  const size_t words = (size_t)(round_hi - round_lo) * stride;
  if (words > cap_words) { ctx->err = "trace buffer too small"; return ABS_E_ARG; }
  if (words) std::memcpy(h_out, ctx->sched->trace().data() + (size_t)round_lo * stride, words * sizeof(int32_t));
  if (words_written) *words_written = words;
  return ABS_OK;
}

int abs_mlp_round_plan(const abs_config* cfg, int32_t K, char* h_out, size_t cap) {
  if (!cfg || !h_out || cap == 0) return ABS_E_ARG;
  h_out[0] = 0;
  std::string why;
  if (cfg->model != ABS_MODEL_MLP || !validate(*cfg, why)) return ABS_E_ARG;
  const std::string plan = mlp_round_plan(*cfg, K);
  if (plan.empty() || plan.size() + 1 > cap) return ABS_E_ARG;
  std::memcpy(h_out, plan.c_str(), plan.size() + 1);
  return ABS_OK;
}

int64_t abs_rounds_done(const abs_ctx* ctx) { return ctx ? ctx->sched->round() : -1; }

int abs_kernel_stats(abs_ctx* ctx, abs_kernel_stat* h_out, int32_t cap, int32_t* n_out) {
  if (!ctx || !h_out || !n_out) return ABS_E_ARG;
  int n = 0;
  for (int k = 0; k < KK_COUNT && n < cap; ++k) {
    if (!ctx->stats[k].launches) continue;
    std::memset(&h_out[n], 0, sizeof(abs_kernel_stat));
    std::snprintf(h_out[n].name, sizeof(h_out[n].name), "%s", kernel_kind_name(k));
    h_out[n].launches = ctx->stats[k].launches;
    h_out[n].total_ms = ctx->stats[k].ms;
    h_out[n].flops = ctx->stats[k].flops;
    h_out[n].bytes = ctx->stats[k].bytes;
    h_out[n].timed_launches = ctx->stats[k].timed_launches;
    h_out[n].timed_flops = ctx->stats[k].timed_flops;
    h_out[n].timed_bytes = ctx->stats[k].timed_bytes;
    ++n;
  }
  *n_out = n;
  return ABS_OK;
}

const char* abs_last_error(const abs_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

void abs_destroy(abs_ctx* ctx) {
  if (!ctx) return;
  if (ctx->cfg.device_mode) {
    (void)hipStreamSynchronize(ctx->stream);
    for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
    if (ctx->h_box) (void)hipHostFree(ctx->h_box);
  }
  delete ctx;
}

uint64_t abs_draw_time_ticks(const abs_config* cfg, int32_t n, int64_t j) {
  return cfg ? Scheduler::time_ticks(*cfg, n, j) : 0;
}

int abs_draw_batch_rows(const abs_config* cfg, int32_t n, int64_t j, int64_t* h_rows_out) {
  if (!cfg || !h_rows_out || cfg->N < 1 || cfg->M < cfg->N || n < 0 || n >= cfg->N) return ABS_E_ARG;
  const uint64_t shard = (uint64_t)(cfg->M / cfg->N);
  const uint64_t jk = job_key(stream_key(cfg->seed, kStreamBatch), (uint32_t)n, (uint32_t)j);
  for (int b = 0; b < cfg->B; ++b)
    h_rows_out[b] = (int64_t)((uint64_t)n * shard + draw(jk, (uint32_t)b) % shard);
  return ABS_OK;
}

}  // extern "C"
