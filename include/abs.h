/*
 * libabs: one simulated parameter-server round of ABS (Adaptive Bounded
 * Staleness, Tan & Gao) on one AMD MI355X (gfx950).
 *
 * The paper's setting (Section II-A): N workers hold disjoint shards of a
 * dataset; in round t the server waits for the K^t fastest uploads, each a
 * minibatch stochastic gradient taken at the worker's own stale copy
 * w^{t - tau} of the global model, and applies Eq. 3.  Section III adds the
 * two adaptive rules: the wait count K^t (Eq. 5) and the staleness threshold
 * tau_max^t (Eq. 4) that forces over-stale workers to restart (Eq. 6,
 * Algorithm 1).  This library runs that loop with U >= 1 local steps: a host
 * event-queue scheduler draws execution times, selects the K^t fastest
 * workers and applies Eq. 4-6; HIP kernels compute the K^t gradients at mixed
 * model versions out of a device-resident ring of past global models, reduce
 * them, update the model and write the new snapshot.
 *
 * All entry points are plain C.  Pointers named d_* are DEVICE pointers owned
 * by the caller, h_* are HOST pointers owned by the caller.  Every call
 * returns ABS_OK or a negative error code; no exception crosses the boundary.
 * A handle is not thread-safe.
 *
 * Which calls carry the paper's method and which are plumbing.  abs_create is the
 * initialisation of Algorithm 1, abs_round its server loop with the workers' steps
 * (Eq. 2-6), abs_evaluate the read-outs of Section V-B, abs_batch_* the sweeps of
 * Section V, abs_draw_* the random draws of Sections II-A and V-A.  Everything else
 * has no passage behind it and exists because a C library needs it: abs_config_bytes,
 * abs_workspace_size, abs_batch_workspace_size (sizes of the caller's allocations),
 * abs_get_model, abs_trace, abs_rounds_done, abs_kernel_stats, abs_mlp_round_plan
 * (reading results and bookkeeping out), abs_last_error, abs_batch_last_error,
 * abs_destroy, abs_batch_destroy, abs_evaluate_static (abs_evaluate without allocations),
 * abs_calibrate_mfma (a measurement aid).
 */
#ifndef ABS_H
#define ABS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ABS_MAX_LAYERS   7      /* weight matrices of the MLP                          */
#define ABS_MAX_WORKERS  128    /* N                                                    */
#define ABS_TRACE_HEADER 12     /* int32 words before the per-worker lists              */

enum {
  ABS_OK = 0,
  ABS_E_ARG = -1,        /* bad argument / unsupported configuration                    */
  ABS_E_WORKSPACE = -2,  /* workspace smaller than abs_workspace_size()                 */
  ABS_E_HIP = -3,        /* a HIP runtime call failed                                   */
  ABS_E_VERSION = -4,    /* requested model version is no longer (or not yet) in the ring */
  ABS_E_NONFINITE = -5,  /* a worker loss came back non-finite                          */
  ABS_E_REPLAY = -6      /* k_mode 2: the replay array has no entry for this round      */
};

enum { ABS_MODEL_LINEAR = 0, ABS_MODEL_SOFTMAX = 1, ABS_MODEL_MLP = 2, ABS_MODEL_CNN = 3 };
enum { ABS_X_FP32 = 0, ABS_X_BF16 = 1 };
enum { ABS_K_ADAPTIVE = 0, ABS_K_FIXED = 1, ABS_K_REPLAY = 2, ABS_K_ADAPTIVE_FREE = 3 };
enum { ABS_TAU_ADAPTIVE = 0, ABS_TAU_FIXED = 1, ABS_TAU_INF = 2 };
enum { ABS_TIME_EXP = 0, ABS_TIME_PARETO = 1, ABS_TIME_CONST = 2 };

typedef struct abs_ctx abs_ctx;   /* opaque: one simulation */

/*
 * One simulation's parameters.  Symbols follow the paper: N workers, minibatch
 * size B, initial wait count K^0, constant a of Eq. 4, step size eta (lr).
 *
 *  model      0: linear least squares f = 1/2 (x.w - y)^2, dims = {d, 1}, no bias,
 *                X fp32 [M, d], y fp32 [M].
 *             1: softmax regression, dims = {d, C}, C <= 16, d % 4 == 0,
 *                X fp32 [M, d], y int32 [M] in [0, C).
 *             2: ReLU MLP with softmax cross-entropy, dims = {d_0, ..., d_L},
 *                L = n_layers >= 2, d_0 % 8 == 0, d_L <= 256; X bf16 (uint16
 *                payload) [M, d_0]; bf16 operands, fp32 accumulation and master
 *                weights.
 *             3: the convolutional network of Section V-A (two convolutional and three
 *                fully connected layers; the paper gives no shapes, this is the reading):
 *                n_layers = 5, dims = {C0*S*S, C1, C2, F1, F2, C, C0, k}: k x k convolutions,
 *                stride 1, no padding, C0 -> C1 -> C2 channels, each followed by ReLU and
 *                2 x 2 max-pooling (S - k + 1 and the pooled side - k + 1 even), then dense
 *                layers F0 = C2*S2*S2 -> F1 -> F2 -> C with ReLU between them, softmax
 *                cross-entropy.  X fp32 [M, C0*S*S], an image stored (channel, row,
 *                column); y int32 [M]; fp32 throughout.  Model vector: per
 *                layer W then b; a convolution's W is [C_in*k*k][C_out], row
 *                (ci*k + u)*k + v; a dense layer's [d_in][d_out].
 *  k_mode     0: Eq. 5, floor'ed, kept non-decreasing;  1: K^t = K0;
 *             2: K^t = k_replay[t] (host array, copied at create);
 *             3: Eq. 5 floor'ed and clamped to [1, N] only.
 *  tau_mode   0: Eq. 4 with the threshold additionally capped at tau_cap;
 *             1: fixed threshold tau_cap;  2: no threshold (no forced restarts).
 *  tau_cap    bounds the ring of model versions (tau_cap + 3 slots); modes 0/1.
 *             In mode 2 it only sizes the ring and the caller must make it large
 *             enough (a selected worker staler than tau_cap + 1 is an error).
 *  sa_penalty 1: a gradient of staleness tau is applied with eta / max(1, tau).
 *  time_dist  execution time of a job, in units of 2^-20: 0: 1 + Exp(1);
 *             1: Pareto(x_m = 1, alpha = time_param); 2: constant 1.  Workers
 *             0 .. n_slow-1 are slowed by slow_factor.
 *  seed       seeds execution times and minibatch draws (counter-based).
 *  device_mode 1: run the device work.  0: schedule only (no HIP call is made, the
 *             device pointers may be NULL, k_mode must be 1 or 2, losses are NaN);
 *             used to plan or check the event trace on a machine without a GPU.
 *  profile    1: bracket every kernel with events and accumulate per-kernel time
 *             (read with abs_kernel_stats); costs a few microseconds per launch.
 *             n > 1: the same in every n-th round only (rounds t with t mod n = 0), a
 *             uniform sample of the job at 1/n of the cost.
 *  U          local SGD steps per job (Eq. 2), 1 <= U <= 64; 0 is read as 1.  With U > 1 every upload is
 *             the change w^{t,0} - w^{t,U} of a private copy of the model after U steps
 *             on fresh minibatches (worker part of Algorithm 1) and the reported loss is
 *             the job's mean local loss; 0 is read as 1.
 */
typedef struct abs_config {
  int32_t model;
  int32_t n_layers;
  int32_t dims[8];
  int32_t x_dtype;
  int32_t N;
  int64_t M;
  int32_t B;
  int32_t K0;
  int32_t k_mode;
  int32_t tau_mode;
  int32_t tau_cap;
  int32_t a;
  float   lr;
  int32_t sa_penalty;
  int32_t time_dist;
  int32_t n_slow;
  double  time_param;
  double  slow_factor;
  uint64_t seed;
  const int32_t* k_replay;     /* host pointer, k_mode 2 only */
  int64_t k_replay_len;
  int32_t device_mode;
  int32_t profile;
  int32_t U;
  int32_t reserved;            /* must be 0 */
} abs_config;

/* sizeof(abs_config) as the library was built, so a binding can check its mirror. */
int32_t abs_config_bytes(void);

/* Bytes of device scratch abs_create needs for this configuration (ring of model
 * versions, bf16 weight copies, activations, partial sums); 0 if the configuration
 * is invalid. */
size_t abs_workspace_size(const abs_config* cfg);

/*
 * Start a simulation (Algorithm 1, initialisation): w^0 goes to every worker,
 * tau = 0, K = K^0, every worker's first execution time is drawn.
 *  d_X, d_y   dataset, row-major, layouts above; read-only, must outlive the handle.
 *  d_w0       initial parameters, fp32, boundary layout: per layer W_l [d_in, d_out]
 *             row-major then b_l [d_out] (the linear model: w [d] only); copied.
 *  d_workspace  >= abs_workspace_size(cfg) bytes, 256-byte aligned, owned by the
 *             caller, used exclusively by this handle until abs_destroy.
 *  hip_stream a hipStream_t (NULL = the null stream); all device work is issued on it.
 * On failure *out is NULL and abs_last_error(NULL) describes the problem.
 */
int abs_create(const abs_config* cfg, const void* d_X, const void* d_y, const float* d_w0,
               void* d_workspace, size_t workspace_bytes, void* hip_stream, abs_ctx** out);

/* Advance n_rounds parameter-server rounds (Algorithm 1, server part, with the
 * workers' U local steps of Eq. 2 and the update of Eq. 3).  Returns when the
 * host has every round's trace record, i.e. after the last round's losses arrived;
 * the tail of that round's device work (backward pass, update, snapshot) may still be
 * running on the stream.  abs_get_model and abs_destroy synchronise the stream. */
int abs_round(abs_ctx* ctx, int32_t n_rounds);

/* Copy global model w^version (fp32, boundary layout, n_floats = parameter count)
 * to host memory; version -1 = the latest.  Synchronises the stream.  (Plumbing: the
 * paper's server simply holds w^t; the versions still readable are those of the ring,
 * t - tau_cap - 2 .. t, ABS_E_VERSION otherwise.) */
int abs_get_model(abs_ctx* ctx, int64_t version, float* h_out, size_t n_floats);

/*
 * Held-out evaluation of global model w^version (-1 = the latest): the read-outs the paper
 * plots against wall-clock time and communication rounds (Section V-B).  *h_loss is the mean
 * per-sample loss f(w; xi) of Eq. 1 over the n_rows evaluation rows, *h_accuracy the fraction of
 * rows whose largest logit is the label (ties: the lowest class; NaN for the linear model).
 *  d_X, d_y   DEVICE, caller-owned, [n_rows, d_0] and [n_rows] in the dtypes of the training
 *             payload; read only.  1 <= n_rows < 2^32.
 * The forward pass is the training one (MLP: bf16 weights of that version, bf16 hidden
 * activations, fp32 logits); row losses are added in a fixed order in fp64.  Runs on the
 * handle's stream after the rounds enqueued so far and synchronises it.  The version must still
 * be in the ring (ABS_E_VERSION otherwise).  Does not change the simulation.
 */
int abs_evaluate(abs_ctx* ctx, int64_t version, const void* d_X, const void* d_y, int64_t n_rows,
                 double* h_loss, double* h_accuracy);

/*
 * abs_evaluate for callers that cannot allocate or synchronise: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The same kernels as abs_evaluate, but their
 * scratch (the two fp64 sums, one pass's per-row losses and hit flags) is a fixed array of
 * 256 + 8 ABS_STATIC_EVAL_ROWS bytes that the library itself holds in device memory, one copy per
 * GPU from the library's load to the end of the process, and the result stays on the device:
 *  d_out      DEVICE, caller-owned, two doubles: d_out[0] = mean loss, d_out[1] = accuracy (NaN
 *             for the linear model), the values abs_evaluate returns, bit for bit.
 * The call enqueues on the handle's stream and returns; it makes no hipMalloc / hipFree /
 * hipHostMalloc, creates no event or stream, copies nothing to the host and does not wait.  Per-kernel
 * timing (abs_config.profile) leaves these launches out.
 * Limits: an MLP handle evaluates N x (B rounded up to 128) rows per pass, a handle of the convolutional
 * model N x B, and that must not exceed ABS_STATIC_EVAL_ROWS (ABS_E_WORKSPACE otherwise; the regression
 * models pass 16384 rows at a time);
 * n_rows itself is not limited.  All handles on a GPU share the one array, which keeps the last
 * call's contents (the call clears what it accumulates into): two such calls that overlap in time on
 * one GPU - different streams, different handles - race; calls on one stream are safe.
 */
#define ABS_STATIC_EVAL_ROWS 65536
int abs_evaluate_static(abs_ctx* ctx, int64_t version, const void* d_X, const void* d_y, int64_t n_rows,
                        double* d_out);

/*
 * Copy trace records of rounds [round_lo, round_hi) to h_out.  One record is
 * ABS_TRACE_HEADER + 3 N int32 words:
 *   0 t   1 K^t   2 floor(tau_max^t) (INT32_MAX: none)   3,4 completion tick lo,hi
 *   5 number of forced restarts   6,7 cumulative uploads lo,hi (sum of K^t)
 *   8,9 cumulative restart messages lo,hi   10 loss estimate of round t as fp32 bits
 *   11 K^{t+1}   then ids[K^t] in arrival order, versions[K^t], staleness[K^t],
 *   restarted ids ascending; unused tail = -1.
 * The paper's communication-round count (Section V-B) is uploads + restarts.
 */
int abs_trace(abs_ctx* ctx, int64_t round_lo, int64_t round_hi, int32_t* h_out,
              size_t cap_words, size_t* words_written);

/*
 * MLP configurations, host only (no device work, no handle): what a round that waits for K uploads
 * launches, as text - one "product:tile rows x tile columns/split count" item per kernel of the
 * round's chain (forward, logits, input gradients, weight gradients, updates), in launch order.
 * Two values of K with the same text run the same kernels with the same tile shapes and split
 * counts (grid sizes aside).  For tests that want to cover every plan of a shape, and for reading
 * profiles.  Writes a NUL-terminated string of at most cap bytes to h_out; ABS_E_ARG if cfg is not
 * a supported MLP configuration, K is outside [1, N] or the text does not fit.
 */
int abs_mlp_round_plan(const abs_config* cfg, int32_t K, char* h_out, size_t cap);

/* Rounds completed so far. */
int64_t abs_rounds_done(const abs_ctx* ctx);

/* Per-kernel accounting: launches always; total_ms only with profile >= 1, over the
 * launches of the bracketed rounds (timed_*).  flops and bytes are the algorithmic work
 * of the launches so far (not counter readings). */
typedef struct abs_kernel_stat {
  char    name[48];
  int64_t launches;
  double  total_ms;
  double  flops;
  double  bytes;
  int64_t timed_launches;   /* the launches that total_ms covers (= launches with profile = 1) */
  double  timed_flops;      /* ... and their algorithmic work */
  double  timed_bytes;
} abs_kernel_stat;
int abs_kernel_stats(abs_ctx* ctx, abs_kernel_stat* h_out, int32_t cap, int32_t* n_out);

/* Text of the last error of this handle (ctx == NULL: of the last failed abs_create /
 * abs_workspace_size on this thread).  Never NULL. */
const char* abs_last_error(const abs_ctx* ctx);

void abs_destroy(abs_ctx* ctx);

/*
 * Batched simulations.  The paper's results are sweeps over seeds and hyper-parameters (a, K^0,
 * the step size; Section V), and a single round of the small workloads is too little work for
 * one launch: a batch advances n simulations of one shape together, for the regression models
 * every round of all of them in one set of launches (one workgroup column per simulation).
 *  abs_batch_workspace_size  bytes of device memory a batch of these handles needs (per-simulation
 *                     kernel arguments, round descriptors, and for softmax rounds one gradient slot
 *                     per upload: about 0.5 MB per simulation of 784 x 10, N = 16); 0 for MLP handles,
 *                     and 0 with abs_batch_last_error(NULL) set if the handles cannot form a batch.
 *  abs_batch_create   ctxs: n handles (1 <= n <= 4096) created with the same model, dims, N, B, U
 *                     and stream, profile = 0; seeds, K0, a, tau settings, step sizes, time
 *                     models and datasets may differ.  d_workspace: DEVICE, caller-owned, at least
 *                     abs_batch_workspace_size() bytes, 256-byte aligned, used by the batch until
 *                     abs_batch_destroy (may be NULL when the size is 0).  The library itself
 *                     allocates only pinned host memory (descriptors, loss mailboxes), three
 *                     streams and a few events.  The batch
 *                     borrows the handles: they must outlive it, and stay usable on their own
 *                     (abs_get_model, abs_trace, abs_evaluate, abs_round) between batch calls.
 *  abs_batch_round    n_rounds rounds of every simulation (each continues from its own round
 *                     count).  A simulation's result does not depend on what else is in the
 *                     batch.  Linear model, and both models with U > 1 (local SGD): bitwise the
 *                     result of abs_round on the handle alone.  Softmax model with U = 1 and
 *                     B <= 1024: the batched round adds up each upload's gradient before Eq. 3
 *                     sums the uploads, another rounding order than abs_round's, so models agree
 *                     with abs_round to fp32 rounding (and an adaptive-K decision of Eq. 5 that
 *                     hangs on the last bit of a loss may differ).  MLP model: every simulation
 *                     keeps its own launches (a round of it is a chain of kernels, not one);
 *                     up to four of them run side by side, each on a stream and a host thread
 *                     of its own, bitwise the result of abs_round, and an error of one does not
 *                     stop the others (the first failing simulation is the one reported).
 *                     Batches (softmax: 4 simulations and more, linear: 32 and more)
 *                     advance as two to four groups, staggered in time, so that the host's part
 *                     of one overlaps the device's part of the others; the first group's work
 *                     goes to the handles' stream, the others' to streams the batch owns, which
 *                     start after everything the handles' stream held at the call and which
 *                     that stream waits for before it runs anything enqueued after the call.
 *                     At return every simulation has done its n_rounds.  On an error of one
 *                     simulation the call stops and names it; rounds already on the device are
 *                     completed first, so the other simulations end on that round, the one
 *                     before or (another group) the one after: abs_rounds_done tells.  A
 *                     handle that did not complete a round repeats it, with the same result,
 *                     the next time it is advanced.
 *  abs_batch_last_error  text of the last error (b == NULL: of the last failed abs_batch_create
 *                     on this thread).
 */
typedef struct abs_batch abs_batch;
size_t abs_batch_workspace_size(abs_ctx** ctxs, int32_t n);
int abs_batch_create(abs_ctx** ctxs, int32_t n, void* d_workspace, size_t workspace_bytes, abs_batch** out);
int abs_batch_round(abs_batch* b, int32_t n_rounds);
const char* abs_batch_last_error(const abs_batch* b);
void abs_batch_destroy(abs_batch* b);

/*
 * Measurement aid, not part of the method: run nothing but the matrix-core instructions of a GEMM
 * tile (the flops of a 128 x 64 x 64 wavefront step per iteration, as 32 MFMA 32x32x16 bf16 or as 64 MFMA
 * 16x16x32 bf16; 8 wavefronts per workgroup, operands in registers, no memory traffic) and report the
 * sustained rate, so that the GEMM kernels' figures can be read against what the chip's matrix cores
 * deliver at the clock they settle at.
 *  data_mode   0: all operand elements 1.0;  1: random bf16 values (sign, mantissa, exponent 2^-2..2^0);
 *              + 2: the 16x16x32 form (the large-tile kernel's) instead of 32x32x16
 *  iters       loop iterations per wavefront;  workgroups: grid size (e.g. 512 = two per CU)
 *  d_scratch   DEVICE, at least workgroups * 512 floats (not written in practice)
 *  h_ms, h_tflops  HOST: duration of one launch (HIP events on hip_stream) and its flops (2 x 128 x 64 x 64
 *              per wavefront and iteration) over it.  Synchronises the stream.
 */
int abs_calibrate_mfma(int32_t data_mode, int32_t iters, int32_t workgroups, float* d_scratch,
                       void* hip_stream, double* h_ms, double* h_tflops);

/* Host-side helpers exposing the simulation's counter-based draws (for checking a
 * binding or planning a run; no device work): execution time of job j of worker n in
 * ticks, and the B dataset rows of that job's minibatch (h_rows_out: B entries). */
uint64_t abs_draw_time_ticks(const abs_config* cfg, int32_t n, int64_t j);
int abs_draw_batch_rows(const abs_config* cfg, int32_t n, int64_t j, int64_t* h_rows_out);

#ifdef __cplusplus
}
#endif
#endif /* ABS_H */
