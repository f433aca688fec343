// Held-out evaluation of one model version: mean per-sample loss (Eq. 1) and accuracy, the
// quantities the paper plots against wall-clock time and communication rounds (Section V-B).
// Not part of a parameter-server round; shares nothing with the training kernels but the layout
// of the model vector.
#include <hip/hip_runtime.h>
#include "kernels.h"

namespace abs_impl {

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One wavefront per row.  Linear: loss 1/2 (x.w - y)^2.  Softmax: W [d][C] then b [C];
// loss -log softmax(xW + b)_y, hit = the first largest logit is the label.
__global__ __launch_bounds__(256) void reg_eval_rows_kernel(const float* X, const void* y, const float* w, int d,
                                                            int C, int softmax, int64_t row0, int n,
                                                            float* rowloss, float* correct) {
  const int lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= n) return;
  const int64_t row = row0 + m;
  const float* xr = X + row * (int64_t)d;
  if (!softmax) {
    float dot = 0.f;
    for (int i = lane; i < d; i += 64) dot = fmaf(xr[i], w[i], dot);
    const float r = wave_sum(dot) - ((const float*)y)[row];
    if (lane == 0) { rowloss[m] = 0.5f * r * r; correct[m] = 0.f; }
    return;
  }
  float z[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) z[c] = 0.f;
  for (int i = lane; i < d; i += 64) {
    const float x = xr[i];
#pragma unroll
    for (int c = 0; c < 16; ++c)
      if (c < C) z[c] = fmaf(x, w[(size_t)i * C + c], z[c]);
  }
  const int label = ((const int32_t*)y)[row];
  float zmax = -INFINITY, zy = 0.f;
  int best = 0;
#pragma unroll
  for (int c = 0; c < 16; ++c) {
    if (c < C) {
      z[c] = wave_sum(z[c]) + w[(size_t)d * C + c];
      if (z[c] > zmax) { zmax = z[c]; best = c; }
      if (c == label) zy = z[c];
    }
  }
  float ssum = 0.f;
#pragma unroll
  for (int c = 0; c < 16; ++c)
    if (c < C) ssum += expf(z[c] - zmax);
  if (lane == 0) { rowloss[m] = logf(ssum) - (zy - zmax); correct[m] = best == label ? 1.f : 0.f; }
}

__global__ void eval_clear_kernel(double* acc) {
  if (threadIdx.x < 2) acc[threadIdx.x] = 0.0;
}

__global__ __launch_bounds__(1024) void eval_reduce_kernel(const float* rowloss, const float* correct, int n,
                                                          double* acc) {
  __shared__ double s_l[1024], s_c[1024];
  double l = 0.0, c = 0.0;
  for (int i = threadIdx.x; i < n; i += 1024) { l += (double)rowloss[i]; c += (double)correct[i]; }
  s_l[threadIdx.x] = l; s_c[threadIdx.x] = c;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) { s_l[threadIdx.x] += s_l[threadIdx.x + o]; s_c[threadIdx.x] += s_c[threadIdx.x + o]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { acc[0] += s_l[0]; acc[1] += s_c[0]; }
}

__global__ void eval_finish_kernel(const double* acc, double n_rows, int linear, double* out) {
  if (threadIdx.x == 0) {
    out[0] = acc[0] / n_rows;
    out[1] = linear ? __longlong_as_double(0x7FF8000000000000ll) : acc[1] / n_rows;
  }
}

}  // namespace

hipError_t launch_eval_finish(const EvalArgs& e, bool linear, double* d_out, hipStream_t s) {
  eval_finish_kernel<<<dim3(1), dim3(64), 0, s>>>(e.acc, (double)e.n_rows, linear ? 1 : 0, d_out);
  return hipGetLastError();
}

hipError_t launch_eval_clear(const EvalArgs& e, hipStream_t s) {
  eval_clear_kernel<<<dim3(1), dim3(64), 0, s>>>(e.acc);
  return hipGetLastError();
}

hipError_t launch_eval_reduce(const EvalArgs& e, int n, hipStream_t s, LaunchHook* hook) {
  hook->begin(KK_EVAL, 2.0 * n, 8.0 * n);
  eval_reduce_kernel<<<dim3(1), dim3(1024), 0, s>>>(e.rowloss, e.correct, n, e.acc);
  hook->end(KK_EVAL);
  return hipGetLastError();
}

hipError_t launch_regression_eval(const float* w, int d, int C, bool softmax, const EvalArgs& e,
                                  hipStream_t s, LaunchHook* hook) {
  hipError_t err = launch_eval_clear(e, s);
  for (int64_t row0 = 0; row0 < e.n_rows && err == hipSuccess; row0 += e.cap) {
    const int n = (int)(e.n_rows - row0 < e.cap ? e.n_rows - row0 : e.cap);
    hook->begin(KK_EVAL, 2.0 * n * d * (softmax ? C : 1), 4.0 * n * (d + 1));
    reg_eval_rows_kernel<<<dim3((n + 3) / 4), dim3(256), 0, s>>>((const float*)e.X, e.y, w, d, C, softmax ? 1 : 0,
                                                               row0, n, e.rowloss, e.correct);
    hook->end(KK_EVAL);
    err = hipGetLastError();
    if (err == hipSuccess) err = launch_eval_reduce(e, n, s, hook);
  }
  return err;
}

}  // namespace abs_impl
