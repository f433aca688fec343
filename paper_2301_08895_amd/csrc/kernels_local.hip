// Local SGD (U > 1 steps of Eq. 2 per job) for the two regression models.
//
// A worker's job is U sequential minibatch steps on a private copy of the model it
// received (worker part of Algorithm 1), so the K^t uploads of a round are independent
// chains: one workgroup per upload keeps the private model in LDS, runs the U steps on
// fresh minibatches and writes the upload w^{t,0} - w^{t,U} and the job's mean local loss.
// A second kernel averages the K^t uploads in arrival order (Eq. 3), writes w^{t+1} into
// the next ring slot and publishes the losses.  Rows of dZ carry c = eta_k / B.
#include <hip/hip_runtime.h>
#include "kernels.h"

namespace abs_impl {

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// minibatch draw b of local step u of job w.job of worker w.id (counter index u * B + b)
__device__ __forceinline__ uint64_t local_row(const WorkerDesc& w, uint64_t batch_key, uint64_t shard_rows,
                                              uint32_t u, uint32_t B, uint32_t b) {
  const uint64_t jk = job_key(batch_key, w.id, w.job);
  return (uint64_t)w.id * shard_rows + draw(jk, u * B + b) % shard_rows;
}

constexpr int kLocWaves = 4;
constexpr int kLinDMax = 512;

// ---- linear least squares: private w in LDS; a lane owns features lane, lane+64, ...
__device__ __forceinline__ void linreg_local_body(const RegressionArgs& a, const RoundDesc& rd) {
  __shared__ float s_w[kLinDMax];
  __shared__ float s_g[kLocWaves][kLinDMax];
  __shared__ float s_l[kLocWaves];
  constexpr int Q = kLinDMax / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int up = blockIdx.x, d = a.d, B = a.B;
  if (up >= rd.K) return;
  const WorkerDesc w = rd.w[up];
  const float* start = a.ring + (size_t)w.slot * a.slot_stride;
  const float* y = (const float*)a.y;
  for (int i = threadIdx.x; i < d; i += blockDim.x) s_w[i] = start[i];
  float loss = 0.f;                       // this wavefront's share, lane 0
  __syncthreads();
  for (int u = 0; u < a.U; ++u) {
    float g[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) g[q] = 0.f;
    for (int b = wave; b < B; b += kLocWaves) {
      const uint64_t row = local_row(w, a.batch_key, a.shard_rows, (uint32_t)u, (uint32_t)B, (uint32_t)b);
      const float* xr = a.X + row * (uint64_t)d;
      float x[Q], dot = 0.f;
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        const int i = lane + 64 * q;
        x[q] = i < d ? xr[i] : 0.f;
        dot = fmaf(x[q], i < d ? s_w[i] : 0.f, dot);
      }
      const float res = wave_sum(dot) - y[row];
      const float coef = w.c * res;
#pragma unroll
      for (int q = 0; q < Q; ++q) g[q] = fmaf(coef, x[q], g[q]);
      loss += 0.5f * res * res;
    }
#pragma unroll
    for (int q = 0; q < Q; ++q) s_g[wave][lane + 64 * q] = g[q];
    __syncthreads();
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
      float G = 0.f;
#pragma unroll
      for (int v = 0; v < kLocWaves; ++v) G += s_g[v][i];
      s_w[i] -= G;                        // Eq. 2
    }
    __syncthreads();
  }
  if (lane == 0) s_l[wave] = loss;
  float* delta = a.delta + (size_t)up * a.slot_stride;
  for (int i = threadIdx.x; i < d; i += blockDim.x) delta[i] = start[i] - s_w[i];
  __syncthreads();
  if (threadIdx.x == 0) {
    float l = 0.f;
#pragma unroll
    for (int v = 0; v < kLocWaves; ++v) l += s_l[v];
    a.lossbuf[up] = l / (float)(B * a.U);
  }
}

__global__ __launch_bounds__(kLocWaves * 64) void linreg_local_kernel(RegressionArgs a, RoundDesc rd) {
  linreg_local_body(a, rd);
}
// Batched forms: blockIdx.y = simulation, arguments and round descriptors from device tables.
__global__ __launch_bounds__(kLocWaves * 64) void linreg_local_batch_kernel(const RegressionArgs* as, const char* rds,
                                                                           size_t stride) {
  const RegressionArgs a = as[blockIdx.y];
  linreg_local_body(a, *(const RoundDesc*)(rds + (size_t)blockIdx.y * stride));
}

// ---- softmax regression: private W, b in LDS.  Per batch of up to 256 rows: (1) a
// wavefront per row computes the row of dZ = c (softmax - onehot) from the LDS model,
// (2) every thread owns features t, t + 256, ... and adds x^T dZ over the batch's rows;
// after the step's last batch the thread applies its own rows of the gradient.
constexpr int kSoftDMax = 1024;
constexpr int kRowBatch = 256;

template <int C>
__device__ __forceinline__ void softmax_local_body(const RegressionArgs& a, const RoundDesc& rd) {
  __shared__ float s_W[(kSoftDMax + 1) * C];
  __shared__ float s_dz[kRowBatch][C];
  __shared__ uint32_t s_row[kRowBatch];
  __shared__ float s_l[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, t = threadIdx.x;
  const int up = blockIdx.x, d = a.d, B = a.B;
  if (up >= rd.K) return;
  const WorkerDesc w = rd.w[up];
  const float* start = a.ring + (size_t)w.slot * a.slot_stride;
  const int P = (d + 1) * C;
  for (int i = t; i < P; i += 256) s_W[i] = start[i];
  float loss = 0.f;
  __syncthreads();
  for (int u = 0; u < a.U; ++u) {
    float acc[4][C];                      // features t + 256 f, f < 4  (d <= 1024)
    float bacc = 0.f;                     // bias gradient, threads t < C
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int c = 0; c < C; ++c) acc[f][c] = 0.f;
    for (int b0 = 0; b0 < B; b0 += kRowBatch) {
      const int nb = min(kRowBatch, B - b0);
      // (1) rows of dZ
      for (int bl = wave; bl < nb; bl += 4) {
        const uint64_t row = local_row(w, a.batch_key, a.shard_rows, (uint32_t)u, (uint32_t)B, (uint32_t)(b0 + bl));
        const float* xr = a.X + row * (uint64_t)d;
        float z[C];
#pragma unroll
        for (int c = 0; c < C; ++c) z[c] = 0.f;
        for (int i = lane; i < d; i += 64) {
          const float x = xr[i];
#pragma unroll
          for (int c = 0; c < C; ++c) z[c] = fmaf(x, s_W[i * C + c], z[c]);
        }
        float zmax = -INFINITY;
#pragma unroll
        for (int c = 0; c < C; ++c) { z[c] = wave_sum(z[c]) + s_W[d * C + c]; zmax = fmaxf(zmax, z[c]); }
        const int label = ((const int32_t*)a.y)[row];
        float ssum = 0.f, zy = 0.f;
#pragma unroll
        for (int c = 0; c < C; ++c) {
          if (c == label) zy = z[c] - zmax;
          z[c] = expf(z[c] - zmax);
          ssum += z[c];
        }
        if (lane < C) {
          float p = 0.f;
#pragma unroll
          for (int c = 0; c < C; ++c) if (c == lane) p = z[c] / ssum;
          s_dz[bl][lane] = w.c * (p - (lane == label ? 1.f : 0.f));
        }
        if (lane == 0) { s_row[bl] = (uint32_t)row; loss += logf(ssum) - zy; }
      }
      __syncthreads();
      // (2) this thread's features against the batch's rows
      for (int bl = 0; bl < nb; ++bl) {
        const float* xr = a.X + (uint64_t)s_row[bl] * (uint64_t)d;
#pragma unroll
        for (int f = 0; f < 4; ++f) {
          const int i = t + 256 * f;
          if (i < d) {
            const float x = xr[i];
#pragma unroll
            for (int c = 0; c < C; ++c) acc[f][c] = fmaf(x, s_dz[bl][c], acc[f][c]);
          }
        }
        if (t < C) bacc += s_dz[bl][t];
      }
      __syncthreads();
    }
    // Eq. 2: every thread updates the rows of W it owns
#pragma unroll
    for (int f = 0; f < 4; ++f) {
      const int i = t + 256 * f;
      if (i < d) {
#pragma unroll
        for (int c = 0; c < C; ++c) s_W[i * C + c] -= acc[f][c];
      }
    }
    if (t < C) s_W[d * C + t] -= bacc;
    __syncthreads();
  }
  if (lane == 0) s_l[wave] = loss;
  float* delta = a.delta + (size_t)up * a.slot_stride;
  for (int i = t; i < P; i += 256) delta[i] = start[i] - s_W[i];
  __syncthreads();
  if (t == 0) a.lossbuf[up] = (s_l[0] + s_l[1] + s_l[2] + s_l[3]) / (float)(B * a.U);
}

template <int C>
__global__ __launch_bounds__(256) void softmax_local_kernel(RegressionArgs a, RoundDesc rd) {
  softmax_local_body<C>(a, rd);
}
template <int C>
__global__ __launch_bounds__(256) void softmax_local_batch_kernel(const RegressionArgs* as, const char* rds,
                                                                  size_t stride) {
  const RegressionArgs a = as[blockIdx.y];
  softmax_local_body<C>(a, *(const RoundDesc*)(rds + (size_t)blockIdx.y * stride));
}

// ---- Eq. 3 over the uploads' changes: w^{t+1} = w^t - (1/K) sum_a delta_a, arrival order
__device__ __forceinline__ void delta_update_body(const RegressionArgs& a, const RoundDesc& rd, int P) {
  __shared__ float s_loss[ABS_MAX_WORKERS];
  const float* cur = a.ring + (size_t)rd.slot_cur * a.slot_stride;
  float* nxt = a.ring + (size_t)rd.slot_next * a.slot_stride;
  if (blockIdx.x == 0) {                  // first: the host prepares the next round meanwhile
    for (int up = threadIdx.x; up < rd.K; up += 256) s_loss[up] = a.lossbuf[up];
    __syncthreads();
    publish_losses(a.mailbox, s_loss, rd.K, rd.stamp);
  }
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < P) {
    float s = 0.f;
    for (int up = 0; up < rd.K; ++up) s += a.delta[(size_t)up * a.slot_stride + i];
    nxt[i] = cur[i] - s / (float)rd.K;
  }
}

__global__ __launch_bounds__(256) void delta_update_kernel(RegressionArgs a, RoundDesc rd, int P) {
  delta_update_body(a, rd, P);
}
__global__ __launch_bounds__(256) void delta_update_batch_kernel(const RegressionArgs* as, const char* rds,
                                                                 size_t stride, int P) {
  const RegressionArgs a = as[blockIdx.y];
  delta_update_body(a, *(const RoundDesc*)(rds + (size_t)blockIdx.y * stride), P);
}

}  // namespace

hipError_t launch_regression_local_round(const RegressionArgs& a, const RoundDesc& rd, bool softmax,
                                         hipStream_t s, LaunchHook* hook) {
  const double rows = (double)rd.K * a.B * a.U;
  const int P = softmax ? (a.d + 1) * a.C : a.d;
  hook->begin(KK_LOCAL_STEPS, rows * a.d * (softmax ? a.C : 1) * 4.0, rows * (a.d + 1) * 4.0);
  if (!softmax) {
    linreg_local_kernel<<<dim3(rd.K), dim3(kLocWaves * 64), 0, s>>>(a, rd);
  } else if (softmax_local_fused_ok(a.B, a.U)) {
    const hipError_t e = launch_softmax_local_fused(&a, &rd, nullptr, nullptr, 0, 1, a.d, a.C, a.B, a.U, rd.K, s);
    if (e != hipSuccess) return e;
  } else {
    switch (a.C) {
#define ABS_CASE(c) case c: softmax_local_kernel<c><<<dim3(rd.K), dim3(256), 0, s>>>(a, rd); break;
      ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8) ABS_CASE(9)
      ABS_CASE(10) ABS_CASE(11) ABS_CASE(12) ABS_CASE(13) ABS_CASE(14) ABS_CASE(15) ABS_CASE(16)
#undef ABS_CASE
      default: return hipErrorInvalidValue;
    }
  }
  hook->end(KK_LOCAL_STEPS);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hook->begin(KK_DELTA_UPDATE, (double)rd.K * P, ((double)rd.K + 2.0) * P * 4.0);
  delta_update_kernel<<<dim3((P + 255) / 256), dim3(256), 0, s>>>(a, rd, P);
  hook->end(KK_DELTA_UPDATE);
  return hipGetLastError();
}

// One local-SGD round of S simulations of one shape (U > 1; blockIdx.y = simulation).
hipError_t launch_regression_local_round_batch(const RegressionArgs* d_args, const char* d_rds, size_t stride, int S,
                                               bool softmax, int d, int C, int B, int U, int Kmax, hipStream_t s) {
  if (!softmax) {
    linreg_local_batch_kernel<<<dim3(Kmax, S), dim3(kLocWaves * 64), 0, s>>>(d_args, d_rds, stride);
  } else if (softmax_local_fused_ok(B, U)) {
    const hipError_t e = launch_softmax_local_fused(nullptr, nullptr, d_args, d_rds, stride, S, d, C, B, U, Kmax, s);
    if (e != hipSuccess) return e;
  } else {
    switch (C) {
#define ABS_CASE(c) case c: softmax_local_batch_kernel<c><<<dim3(Kmax, S), dim3(256), 0, s>>>(d_args, d_rds, stride); break;
      ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8) ABS_CASE(9)
      ABS_CASE(10) ABS_CASE(11) ABS_CASE(12) ABS_CASE(13) ABS_CASE(14) ABS_CASE(15) ABS_CASE(16)
#undef ABS_CASE
      default: return hipErrorInvalidValue;
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int P = softmax ? (d + 1) * C : d;
  delta_update_batch_kernel<<<dim3((P + 255) / 256, S), dim3(256), 0, s>>>(d_args, d_rds, stride, P);
  return hipGetLastError();
}

}  // namespace abs_impl
