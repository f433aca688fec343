// Launchers of the HIP kernels (defined in kernels_regression.hip / kernels_mlp.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <string>
#include "abs_common.h"

namespace abs_impl {

// Called around every launch so that the API layer can count / time kernels.
struct LaunchHook {
  virtual void begin(int kind, double flops, double bytes) = 0;
  virtual void end(int kind) = 0;
  // The same around a single launch that can carry its own start / stop events (hipExtLaunchKernel):
  // the kernel's begin and end are then stamped by its dispatch itself, with no marker packets between
  // the kernels of a round.  *e0 / *e1 come back null when the launch is not to be timed.  The default
  // falls back on begin / end.
  virtual void begin_kernel(int kind, double flops, double bytes, hipEvent_t* e0, hipEvent_t* e1) {
    *e0 = nullptr; *e1 = nullptr;
    begin(kind, flops, bytes);
  }
  virtual void end_kernel(int kind) { end(kind); }
  virtual ~LaunchHook() {}
};

enum KernelKind {
  KK_LINREG_ROUND = 0,
  KK_SOFTMAX_ROWS,
  KK_SOFTMAX_UPDATE,
  KK_MLP_INDEX,
  KK_MLP_GATHER_T,
  KK_MLP_FWD_L1,
  KK_MLP_FWD_HIDDEN,
  KK_MLP_FWD_LOGITS,
  KK_MLP_LOGITS_CE,
  KK_MLP_LOSS,
  KK_MLP_DGRAD_OUT,
  KK_MLP_DGRAD,
  KK_MLP_WGRAD_L1,
  KK_MLP_WGRAD,
  KK_MLP_UPDATE,
  KK_MLP_BIAS_LOSS,
  KK_LOCAL_STEPS,
  KK_DELTA_UPDATE,
  KK_EVAL,
  KK_MLP_WGRAD_OUT,
  KK_CNN_CONV_FWD,
  KK_CNN_DENSE,
  KK_CNN_DENSE_WGRAD,
  KK_CNN_CONV_BWD,
  KK_CNN_CONV_WGRAD,
  KK_CNN_COMBINE,
  KK_COUNT
};
const char* kernel_kind_name(int kind);

struct RegressionArgs {
  const float* X;        // [M, d] fp32
  const void*  y;        // fp32 [M] (linear) or int32 [M] (softmax)
  float* ring;           // [R slots][slot_stride] fp32
  size_t slot_stride;    // floats between slots
  int d, C, B;
  uint64_t shard_rows;   // rows per worker shard
  uint64_t batch_key;    // stream_key(seed, kStreamBatch)
  LossMailbox* mailbox;  // per-upload mean minibatch losses + completion stamp (device-visible host memory)
  // softmax scratch
  float* dz;             // [N*B][16]
  float* rowloss;        // [N*B]
  uint32_t* rowidx;      // [N*B]
  // local SGD (U > 1): per-upload accumulated change and mean local loss
  int U;
  float* delta;          // [N][slot_stride]
  float* lossbuf;        // [N]
};

hipError_t launch_linreg_round(const RegressionArgs& a, const RoundDesc& rd, hipStream_t s,
                               LaunchHook* hook);
hipError_t launch_softmax_round(const RegressionArgs& a, const RoundDesc& rd, hipStream_t s,
                                LaunchHook* hook);
// U > 1: every upload runs its U local steps in one workgroup, then the uploads' changes are averaged
hipError_t launch_regression_local_round(const RegressionArgs& a, const RoundDesc& rd, bool softmax,
                                         hipStream_t s, LaunchHook* hook);

// One round of S simulations of one shape in a single set of launches (blockIdx.y = simulation):
// d_args [S] and the S round descriptors (header + uploads, `stride` bytes apart) live in device
// memory; Kmax = the largest K^t among them.  slots: every simulation's `delta` ([N][slot_stride]) and
// `lossbuf` ([N]) are there, so the softmax round may keep per-upload gradients (the fused form).
hipError_t launch_regression_round_batch(const RegressionArgs* d_args, const char* d_rds, size_t stride, int S,
                                         bool softmax, int d, int C, int B, int Kmax, bool slots, hipStream_t s);
// the same for local SGD (U > 1 in every simulation's arguments; their `delta` / `lossbuf` exist)
hipError_t launch_regression_local_round_batch(const RegressionArgs* d_args, const char* d_rds, size_t stride, int S,
                                               bool softmax, int d, int C, int B, int U, int Kmax, hipStream_t s);
// Softmax local steps on the matrix cores (a workgroup per upload streams the job's U B rows through
// LDS, its private model there too): usable when softmax_local_fused_ok.  a1 / rd1: one simulation's
// arguments by value (then d_args == nullptr), else S simulations from device tables.  Writes the
// uploads' changes and mean local losses to `delta` / `lossbuf`; Eq. 3 over them is the caller's.
bool softmax_local_fused_ok(int B, int U);
hipError_t launch_softmax_local_fused(const RegressionArgs* a1, const RoundDesc* rd1, const RegressionArgs* d_args,
                                      const char* d_rds, size_t stride, int S, int d, int C, int B, int U, int Kmax,
                                      hipStream_t s);
// whether batched rounds of this shape use the per-upload slots (else they need not be allocated)
bool regression_batch_uses_slots(bool softmax, int B);

// ---- held-out evaluation (the read-outs of Section V-B: loss of the global model, accuracy) ----
// Per-row losses and "argmax is the label" flags go to a scratch of `cap` rows; a single
// workgroup adds them, in a fixed order and in fp64, to acc[0] (loss sum) and acc[1] (hits).
constexpr int kEvalChunk = 16384;          // rows per pass of the regression models
struct EvalArgs {
  const void* X;         // evaluation rows, dtype and layout of the training payload
  const void* y;         // their targets
  int64_t n_rows;
  double* acc;           // [2], cleared by the launch
  float* rowloss;        // [cap]
  float* correct;        // [cap]
  int cap;
};
inline size_t eval_scratch_bytes(size_t cap) { return 256 + 2 * ((cap * 4 + 255) / 256 * 256); }
hipError_t launch_eval_clear(const EvalArgs& e, hipStream_t s);
hipError_t launch_eval_reduce(const EvalArgs& e, int n, hipStream_t s, LaunchHook* hook);
// d_out[0] = acc[0] / n_rows (mean loss), d_out[1] = acc[1] / n_rows (accuracy; NaN when `linear`)
hipError_t launch_eval_finish(const EvalArgs& e, bool linear, double* d_out, hipStream_t s);
// w: the model version to evaluate (fp32, boundary layout); softmax = false: linear least squares
hipError_t launch_regression_eval(const float* w, int d, int C, bool softmax, const EvalArgs& e,
                                  hipStream_t s, LaunchHook* hook);

}  // namespace abs_impl

namespace abs_impl {

// ---- MLP path --------------------------------------------------------------------------
// Padded sizes and workspace offsets of the MLP path; filled by mlp_plan().
struct MlpPlan {
  int L;                 // weight matrices
  int d[8], dp[8];       // layer widths and their padded values
  int ld[8];             // row pitch (elements) of the bf16 arrays with dp[l] columns
  size_t ldm;            // row pitch of the transposed arrays [dp_l][Mp]
  int B, Bp;             // minibatch rows per upload, padded to the row tile
  int N, Mp;             // workers; Mp = N * Bp stacked rows at most
  int R;                 // ring slots
  size_t P;              // parameters
  size_t slot_stride;    // floats between fp32 ring slots
  size_t w_off[8], b_off[8];      // W_l / b_l inside a slot (floats), l = 0 .. L-1
  size_t shadow_stride;           // bf16 elements between shadow slots
  size_t wt_off[8], wn_off[8];    // bf16 W_l^T [dp_out][ld_in] / W_l [dp_in][ld_out] inside a shadow slot
  // byte offsets into the workspace
  size_t off_ring, off_shadow, off_rowidx, off_label, off_xgt;
  size_t off_h[8], off_ht[8];     // H_l [Mp][ld_l], H_l^T [dp_l][ldm], l = 1 .. L-1
  size_t off_z;                   // logits fp32 [Mp][dp_L]
  size_t off_dz[8], off_dzt[8];   // dZ_l [Mp][ld_l], dZ_l^T [dp_l][ldm], l = 1 .. L
  size_t off_rowloss;
  size_t off_partial[8];          // split partials of layer l's weight gradient, fp32 [splits][dp_l][dp_{l+1} + pad] (a region per layer:
                                  // a layer's update may run inside the next layer's weight-gradient launch)
  size_t off_colsum[8];           // column sums of dZ_l per block of 64 rows, fp32 [Mp / 64][dp_l], l = 1 .. L
  size_t off_maskbits[8];         // ReLU mask of H_l, one bit per element in the tile kernel's accumulator order, l = 1 .. L-1
  // local SGD (U > 1): the uploads' private models (same slot layouts as the two rings),
  // their running mean losses, and the averaged change of Eq. 3
  int U;
  size_t off_priv, off_priv_shadow, off_lossacc, off_delta;
  size_t off_eval;       // evaluation scratch for Mp rows
  size_t total;
};
// Returns false (with a message) if the configuration is not supported.
bool mlp_plan(const abs_config& cfg, MlpPlan& plan, const char** why);

struct MlpArgs {
  MlpPlan plan;
  char* ws;              // workspace base (device)
  const uint16_t* X;     // bf16 payload [M, d0]
  const int32_t* y;
  uint64_t shard_rows, batch_key;
  LossMailbox* mailbox;
};
// One-time preparation on the stream: zero the padded buffers, build the bf16 copies of w^0.
hipError_t mlp_prepare(const MlpArgs& a, hipStream_t s);
hipError_t launch_mlp_round(const MlpArgs& a, const RoundDesc& rd, hipStream_t s, LaunchHook* hook);
// What a round of K uploads launches (kernel, tile shape / split count per product), as text; from
// the launch code itself run in a recording mode that launches nothing.  Empty if cfg is not an
// MLP configuration the library supports or K is outside [1, N].
std::string mlp_round_plan(const abs_config& cfg, int K);
// forward pass of ring slot `slot` over e.n_rows evaluation rows, Mp rows at a time (e.cap >= Mp)
hipError_t launch_mlp_eval(const MlpArgs& a, uint32_t slot, const EvalArgs& e, hipStream_t s, LaunchHook* hook);

// ---- convolutional model (Section V-A: two convolutional + three dense layers), fp32 ---------
// Geometry and workspace offsets; filled by cnn_plan().
struct CnnPlan {
  int C0, C1, C2, F0, F1, F2, C, k;   // channels, dense widths (F0 = C2 S2 S2), classes, kernel size
  int S, S1, S2;                      // image side; pooled sides after the first / second convolution
  int B, N, R;
  size_t P, slot_stride;              // parameters; floats between ring slots
  size_t w_off[5], b_off[5];          // W_l / b_l inside a slot (floats): conv1, conv2, dense1..3
  // byte offsets into the workspace; per stacked row (N B at most):
  size_t off_ring, off_rowidx, off_label;
  size_t off_p1, off_a1;              // first pooled map fp32 [C1 S1 S1] and which entry of each window it was
  size_t off_p2, off_a2;              // second pooled map [F0] (the dense stack's input) and the same
  size_t off_h1, off_h2;              // dense activations
  size_t off_dz1, off_dz2, off_dz3;   // dense output gradients (coefficient of Eq. 3 included)
  size_t off_dp2, off_dp1;            // gradients of the pooled maps (zero where the window is dead)
  size_t off_lossbuf;                 // [N] mean minibatch loss per upload
  int U;                              // local steps per job
  size_t off_rowloss;                 // per-row losses
  size_t off_priv;                    // [N][slot_stride]: U = 1: the uploads' shares of the dense layers' gradient;
                                      // U > 1: the uploads' private models
  size_t off_grow1, off_grow2;        // the rows' shares of the two convolutions' gradients [N B][weights + biases]
  size_t off_eval;                    // evaluation scratch for N B rows
  size_t total;
};
bool cnn_plan(const abs_config& cfg, CnnPlan& plan, const char** why);
struct CnnArgs {
  CnnPlan plan;
  char* ws;
  const float* X;        // fp32 [M, C0 S S], an image row is (channel, row, column)
  const int32_t* y;
  uint64_t shard_rows, batch_key;
  LossMailbox* mailbox;
};
hipError_t cnn_prepare();       // once per process: LDS opt-in of the kernels
hipError_t launch_cnn_round(const CnnArgs& a, const RoundDesc& rd, hipStream_t s, LaunchHook* hook);
// forward pass of ring slot `slot` over e.n_rows evaluation rows, N B rows at a time (e.cap >= N B)
hipError_t launch_cnn_eval(const CnnArgs& a, uint32_t slot, const EvalArgs& e, hipStream_t s, LaunchHook* hook);

}  // namespace abs_impl
