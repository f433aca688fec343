// One parameter-server round for the convolutional model of Section V-A (two convolutional and
// three fully connected layers), fp32.
//
// The paper states no layer shapes; the reading: k x k convolutions (stride 1, no padding) with C1 and
// C2 channels, each followed by ReLU and 2 x 2 max-pooling, then F0 -> F1 -> F2 -> C dense layers
// with ReLU between them and softmax cross-entropy; relu'(0) = 0; the pooling gradient goes to the
// first maximum of a window in the order (0,0), (0,1), (1,0), (1,1).  abs_config.dims =
// {C0 S S, C1, C2, F1, F2, C, C0, k}.  Model vector: per layer W then b; a convolution's W is
// [C_in k k][C_out] with row (ci k + u) k + v, a dense layer's [d_in][d_out].
//
// Shape of the work: B = 32 images per upload and N <= 128 uploads per round - a few hundred images
// of 62 K parameters.  Nothing here is bound by arithmetic or bandwidth; the kernels are laid out so
// that every stage has one workgroup per image (or per upload, or per weight row) and the round is
// seven short launches:
//   conv_pool_fwd x 2   a workgroup per stacked row: image (or pooled map) and the upload's stale
//                       filters in LDS; a thread computes the four convolution outputs of one pooling
//                       window, keeps max(., 0) and which of the four it was (255: window dead)
//   dense_fwd_bwd       a workgroup per upload: its B rows through the three dense layers at the
//                       upload's model version, loss, and back down to the gradient of the pooled map
//                       (every dZ already carries the upload's coefficient of Eq. 3)
//   dense_wgrad_update  a thread per dense weight: Eq. 3's sum over all K B stacked rows in row order,
//                       w^{t+1} = w^t - sum; its first workgroup publishes the uploads' losses
//   conv2_bwd           a workgroup per row: gradient of the first pooled map
//   conv_wgrad_update x 2   a workgroup per filter row (ci, u, v): sum over rows and pooling windows,
//                       fixed-order reduction, w^{t+1} = w^t - sum
// Pooling is applied to the pre-activations and the ReLU after it (the maximum of the four ReLUs is
// the ReLU of the maximum, and a window whose maximum is not positive passes no gradient either way).
// All sums have a fixed order: two runs are bitwise identical.
#include <hip/hip_runtime.h>
#include "kernels.h"

namespace abs_impl {

namespace {

constexpr int kDead = 255;

__device__ __forceinline__ uint64_t cnn_batch_row(const WorkerDesc& w, uint64_t batch_key, uint64_t shard_rows,
                                                  uint32_t b) {
  const uint64_t jk = job_key(batch_key, w.id, w.job);
  return (uint64_t)w.id * shard_rows + draw(jk, b) % shard_rows;
}

struct CnnDev {
  CnnPlan p;
  char* ws;
  const float* X;
  const int32_t* y;
  uint64_t shard_rows, batch_key;
  int fixed_slot;        // >= 0: every row reads this ring slot (evaluation); else the upload's own
  int64_t row0;          // evaluation: stacked row r is dataset row row0 + r
  int n_rows;            // stacked rows of this launch
  int step;              // local SGD (U > 1): the local step in hand, else -1.  From step 1 on upload a
                         // computes at its private model; every step's update goes to the private model
  int U;
};

template <typename T>
__device__ __forceinline__ T* wsp(const CnnDev& d, size_t off) { return (T*)(d.ws + off); }

__device__ __forceinline__ const float* slot_of(const CnnDev& d, const RoundDesc& rd, int upload) {
  if (d.step > 0) return wsp<const float>(d, d.p.off_priv) + (size_t)upload * d.p.slot_stride;
  const uint32_t slot = d.fixed_slot >= 0 ? (uint32_t)d.fixed_slot : rd.w[upload].slot;
  return wsp<const float>(d, d.p.off_ring) + (size_t)slot * d.p.slot_stride;
}
// where a weight-gradient kernel reads the model it steps from and writes the stepped model: the
// round's slots (U = 1), or upload a's stale version / private model (local steps)
__device__ __forceinline__ void step_models(const CnnDev& d, const RoundDesc& rd, int upload, const float** cur,
                                            float** next) {
  if (d.step < 0) {
    *cur = wsp<const float>(d, d.p.off_ring) + (size_t)rd.slot_cur * d.p.slot_stride;
    *next = wsp<float>(d, d.p.off_ring) + (size_t)rd.slot_next * d.p.slot_stride;
  } else {
    *cur = slot_of(d, rd, upload);
    *next = wsp<float>(d, d.p.off_priv) + (size_t)upload * d.p.slot_stride;
  }
}

// layer 0: dataset rows -> first pooled map; layer 1: first pooled map -> second pooled map (the
// dense stack's input).
__global__ __launch_bounds__(256) void cnn_conv_pool_fwd_kernel(CnnDev d, RoundDesc rd, int layer) {
  extern __shared__ float sm[];
  const CnnPlan& p = d.p;
  const int r = blockIdx.x, a = r / p.B, t = threadIdx.x;
  const int Cin = layer ? p.C1 : p.C0, Cout = layer ? p.C2 : p.C1;
  const int Sin = layer ? p.S1 : p.S, Sp = layer ? p.S2 : p.S1, k = p.k;
  const int n_in = Cin * Sin * Sin, n_w = Cin * k * k * Cout, n_out = Cout * Sp * Sp;
  float* sx = sm;
  float* sw = sx + n_in;
  float* sb = sw + n_w;
  const float* src;
  if (layer) {
    src = wsp<const float>(d, p.off_p1) + (size_t)r * n_in;
  } else {
    const uint64_t row = d.fixed_slot >= 0 ? (uint64_t)(d.row0 + r)
                                           : cnn_batch_row(rd.w[a], d.batch_key, d.shard_rows,
                                                           (uint32_t)(max(d.step, 0) * p.B + r - a * p.B));
    src = d.X + row * (uint64_t)n_in;
    if (t == 0) {
      wsp<uint32_t>(d, p.off_rowidx)[r] = (uint32_t)(d.fixed_slot >= 0 ? r : row);
      wsp<int32_t>(d, p.off_label)[r] = d.y[row];
    }
  }
  const float* w = slot_of(d, rd, a);
  for (int i = t; i < n_in; i += 256) sx[i] = src[i];
  for (int i = t; i < n_w; i += 256) sw[i] = w[p.w_off[layer] + i];
  for (int i = t; i < Cout; i += 256) sb[i] = w[p.b_off[layer] + i];
  __syncthreads();
  float* out = wsp<float>(d, layer ? p.off_p2 : p.off_p1) + (size_t)r * n_out;
  uint8_t* arg_out = wsp<uint8_t>(d, layer ? p.off_a2 : p.off_a1) + (size_t)r * n_out;
  for (int o = t; o < n_out; o += 256) {
    const int co = o / (Sp * Sp), pi = (o / Sp) % Sp, pj = o % Sp;
    float a0 = sb[co], a1 = a0, a2 = a0, a3 = a0;
    for (int ci = 0; ci < Cin; ++ci)
      for (int u = 0; u < k; ++u) {
        const float* x0 = sx + (ci * Sin + 2 * pi + u) * Sin + 2 * pj;
        const float* wr = sw + ((ci * k + u) * k) * Cout + co;
        for (int v = 0; v < k; ++v) {
          const float wv = wr[v * Cout];
          a0 = fmaf(x0[v], wv, a0);
          a1 = fmaf(x0[v + 1], wv, a1);
          a2 = fmaf(x0[v + Sin], wv, a2);
          a3 = fmaf(x0[v + Sin + 1], wv, a3);
        }
      }
    float m = a0; int q = 0;
    if (a1 > m) { m = a1; q = 1; }
    if (a2 > m) { m = a2; q = 2; }
    if (a3 > m) { m = a3; q = 3; }
    out[o] = fmaxf(m, 0.f);
    arg_out[o] = (uint8_t)(m > 0.f ? q : kDead);
  }
}

// out[b][j] = bias[j] + sum_i in[b][i] W[i][j] for the B rows in LDS; a thread takes 8 rows of one
// column, so a weight is fetched once per 8 rows and neighbouring threads read neighbouring weights.
__device__ __forceinline__ void dense_rows(const float* s_in, int Fin, const float* W, const float* bias, int Fout,
                                           int B, bool relu, float* s_out, float* g_out) {
  const int groups = (B + 7) / 8;
  for (int item = threadIdx.x; item < groups * Fout; item += 256) {
    const int j = item % Fout, b0 = (item / Fout) * 8;
    float acc[8];
    const float bv = bias[j];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = bv;
    for (int i = 0; i < Fin; ++i) {
      const float wv = W[(size_t)i * Fout + j];
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[q] = fmaf(s_in[min(b0 + q, B - 1) * Fin + i], wv, acc[q]);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q)
      if (b0 + q < B) {
        const float v = relu ? fmaxf(acc[q], 0.f) : acc[q];
        s_out[(b0 + q) * Fout + j] = v;
        if (g_out) g_out[(size_t)(b0 + q) * Fout + j] = v;
      }
  }
}

// dIn[b][i] = gate(b, i) ? sum_j dOut[b][j] W[i][j] : 0
template <typename Gate>
__device__ __forceinline__ void dense_rows_back(const float* s_dout, int Fout, const float* W, int Fin, int B,
                                                Gate gate, float* s_din, float* g_din) {
  for (int item = threadIdx.x; item < B * Fin; item += 256) {
    const int b = item / Fin, i = item - b * Fin;
    float acc = 0.f;
    if (gate(b, i)) {
      const float* wr = W + (size_t)i * Fout;
      const float* dz = s_dout + b * Fout;
      for (int j = 0; j < Fout; ++j) acc = fmaf(dz[j], wr[j], acc);
    }
    if (s_din) s_din[item] = acc;
    g_din[(size_t)b * Fin + i] = acc;
  }
}

// Training: one workgroup per upload (B rows).  Evaluation (eval_loss != nullptr): one workgroup per
// block of B rows of the evaluation pass, forward only, per-row loss and hit flag.
__global__ __launch_bounds__(256) void cnn_dense_kernel(CnnDev d, RoundDesc rd, float* eval_loss, float* eval_hit) {
  extern __shared__ float sm[];
  const CnnPlan& p = d.p;
  const int a = blockIdx.x, t = threadIdx.x;
  const int r0 = a * p.B;
  const int B = min(p.B, d.n_rows - r0);
  float* sH0 = sm;
  float* sH1 = sH0 + p.B * p.F0;
  float* sH2 = sH1 + p.B * p.F1;
  float* sZ = sH2 + p.B * p.F2;
  float* sD2 = sZ + p.B * p.C;          // dZ of the second dense layer
  float* sD1 = sD2 + p.B * p.F2;        // dZ of the first dense layer
  float* sL = sD1 + p.B * p.F1;         // per-row losses
  const float* w = slot_of(d, rd, a);
  const float* p2 = wsp<const float>(d, p.off_p2) + (size_t)r0 * p.F0;
  for (int i = t; i < B * p.F0; i += 256) sH0[i] = p2[i];
  __syncthreads();
  const bool train = eval_loss == nullptr;
  dense_rows(sH0, p.F0, w + p.w_off[2], w + p.b_off[2], p.F1, B, true, sH1,
             train ? wsp<float>(d, p.off_h1) + (size_t)r0 * p.F1 : nullptr);
  __syncthreads();
  dense_rows(sH1, p.F1, w + p.w_off[3], w + p.b_off[3], p.F2, B, true, sH2,
             train ? wsp<float>(d, p.off_h2) + (size_t)r0 * p.F2 : nullptr);
  __syncthreads();
  dense_rows(sH2, p.F2, w + p.w_off[4], w + p.b_off[4], p.C, B, false, sZ, nullptr);
  __syncthreads();
  const int32_t* label = wsp<const int32_t>(d, p.off_label) + r0;
  if (t < B) {
    // softmax cross-entropy of row t; dZ = c (p - onehot) with the upload's coefficient of Eq. 3
    float* z = sZ + t * p.C;
    const int y = label[t];
    float zmax = z[0]; int best = 0;
    for (int c = 1; c < p.C; ++c) if (z[c] > zmax) { zmax = z[c]; best = c; }
    float ssum = 0.f;
    for (int c = 0; c < p.C; ++c) ssum += expf(z[c] - zmax);
    const float loss = logf(ssum) - (z[y] - zmax);
    if (train) {
      const float coef = rd.w[a].c, inv = 1.f / ssum;
      float* dz3 = wsp<float>(d, p.off_dz3) + (size_t)(r0 + t) * p.C;
      for (int c = 0; c < p.C; ++c) {
        const float v = coef * (expf(z[c] - zmax) * inv - (c == y ? 1.f : 0.f));
        z[c] = v;
        dz3[c] = v;
      }
      sL[t] = loss;
    } else {
      eval_loss[r0 + t] = loss;
      eval_hit[r0 + t] = best == y ? 1.f : 0.f;
    }
  }
  if (!train) return;
  __syncthreads();
  if (t == 0) {
    float sum = 0.f;
    for (int b = 0; b < B; ++b) sum += sL[b];
    // the upload's mean minibatch loss; with local steps, the mean over its U steps
    float* lb = wsp<float>(d, p.off_lossbuf) + a;
    const float mean = sum / (float)B;
    *lb = d.step <= 0 ? (d.step < 0 ? mean : mean / (float)d.U) : *lb + mean / (float)d.U;
  }
  dense_rows_back(sZ, p.C, w + p.w_off[4], p.F2, B, [&](int b, int i) { return sH2[b * p.F2 + i] > 0.f; }, sD2,
                  wsp<float>(d, p.off_dz2) + (size_t)r0 * p.F2);
  __syncthreads();
  dense_rows_back(sD2, p.F2, w + p.w_off[3], p.F1, B, [&](int b, int i) { return sH1[b * p.F1 + i] > 0.f; }, sD1,
                  wsp<float>(d, p.off_dz1) + (size_t)r0 * p.F1);
  __syncthreads();
  const uint8_t* a2 = wsp<const uint8_t>(d, p.off_a2) + (size_t)r0 * p.F0;
  dense_rows_back(sD1, p.F1, w + p.w_off[2], p.F0, B, [&](int b, int i) { return a2[b * p.F0 + i] != kDead; }, nullptr,
                  wsp<float>(d, p.off_dp2) + (size_t)r0 * p.F0);
}

// Eq. 3 for the dense layers: element e of the three weight matrices and biases, summed over the
// stacked rows in row order (every dZ carries its upload's coefficient).
__global__ __launch_bounds__(256) void cnn_dense_wgrad_update_kernel(CnnDev d, RoundDesc rd, LossMailbox* mailbox) {
  const CnnPlan& p = d.p;
  if (blockIdx.x == 0 && mailbox) {
    const float* lossbuf = wsp<const float>(d, p.off_lossbuf);
    if ((int)threadIdx.x < rd.K) mailbox->loss[threadIdx.x] = lossbuf[threadIdx.x];
    if (threadIdx.x < ABS_MAX_WORKERS) __threadfence_system();
    __syncthreads();
    if (threadIdx.x == 0) mailbox->stamp = rd.stamp;
  }
  const int Fin[3] = {p.F0, p.F1, p.F2}, Fout[3] = {p.F1, p.F2, p.C};
  const size_t in_off[3] = {p.off_p2, p.off_h1, p.off_h2}, dz_off[3] = {p.off_dz1, p.off_dz2, p.off_dz3};
  long e = (long)blockIdx.x * 256 + threadIdx.x;
  // local steps: blockIdx.y = upload, the sum runs over its own rows only (Eq. 2)
  const int ra = d.step < 0 ? 0 : (int)blockIdx.y * p.B, rb = d.step < 0 ? d.n_rows : ra + p.B;
  const float* w_cur; float* w_next;
  step_models(d, rd, (int)blockIdx.y, &w_cur, &w_next);
  for (int l = 0; l < 3; ++l) {
    const long nw = (long)Fin[l] * Fout[l], n = nw + Fout[l];
    if (e < n) {
      const float* dz = wsp<const float>(d, dz_off[l]);
      float g = 0.f;
      size_t at;
      if (e < nw) {
        const int i = (int)(e / Fout[l]), j = (int)(e - (long)i * Fout[l]);
        const float* in = wsp<const float>(d, in_off[l]);
        for (int r = ra; r < rb; ++r) g = fmaf(in[(size_t)r * Fin[l] + i], dz[(size_t)r * Fout[l] + j], g);
        at = p.w_off[2 + l] + (size_t)e;
      } else {
        const int j = (int)(e - nw);
        for (int r = ra; r < rb; ++r) g += dz[(size_t)r * Fout[l] + j];
        at = p.b_off[2 + l] + (size_t)j;
      }
      w_next[at] = w_cur[at] - g;
      return;
    }
    e -= n;
  }
}

// Gradient of the first pooled map of row r: the second convolution's output gradient is non-zero
// only where a pooling window had its (positive) maximum.
__global__ __launch_bounds__(256) void cnn_conv2_bwd_kernel(CnnDev d, RoundDesc rd) {
  extern __shared__ float sm[];
  const CnnPlan& p = d.p;
  const int r = blockIdx.x, a = r / p.B, t = threadIdx.x, k = p.k;
  const int S2c = 2 * p.S2, n_dc = p.C2 * S2c * S2c, n_w = p.C1 * k * k * p.C2;
  float* sdc = sm;             // [C2][S2c][S2c]
  float* sw = sdc + n_dc;      // second convolution's filters of this upload's version
  const float* w = slot_of(d, rd, a);
  for (int i = t; i < n_dc; i += 256) sdc[i] = 0.f;
  for (int i = t; i < n_w; i += 256) sw[i] = w[p.w_off[1] + i];
  __syncthreads();
  const float* dp2 = wsp<const float>(d, p.off_dp2) + (size_t)r * p.F0;
  const uint8_t* a2 = wsp<const uint8_t>(d, p.off_a2) + (size_t)r * p.F0;
  for (int o = t; o < p.F0; o += 256) {
    const int q = a2[o];
    if (q != kDead) {
      const int co = o / (p.S2 * p.S2), pi = (o / p.S2) % p.S2, pj = o % p.S2;
      sdc[(co * S2c + 2 * pi + (q >> 1)) * S2c + 2 * pj + (q & 1)] = dp2[o];
    }
  }
  __syncthreads();
  const int n1 = p.C1 * p.S1 * p.S1;
  const uint8_t* a1 = wsp<const uint8_t>(d, p.off_a1) + (size_t)r * n1;
  float* dp1 = wsp<float>(d, p.off_dp1) + (size_t)r * n1;
  for (int o = t; o < n1; o += 256) {
    float acc = 0.f;
    if (a1[o] != kDead) {
      const int ci = o / (p.S1 * p.S1), y = (o / p.S1) % p.S1, x = o % p.S1;
      for (int u = 0; u < k; ++u) {
        const int i = y - u;
        if (i < 0 || i >= S2c) continue;
        for (int v = 0; v < k; ++v) {
          const int j = x - v;
          if (j < 0 || j >= S2c) continue;
          const float* wr = sw + ((ci * k + u) * k + v) * p.C2;
          for (int co = 0; co < p.C2; ++co) acc = fmaf(sdc[(co * S2c + i) * S2c + j], wr[co], acc);
        }
      }
    }
    dp1[o] = acc;
  }
}

// Eq. 3 for a convolution: workgroup q < Cin k k sums filter row q = (ci, u, v) over all rows and
// pooling windows (a window contributes the input under its maximum), workgroup Cin k k the bias.
// Thread partial sums are added in thread order.
constexpr int kMaxCout = 32;
__global__ __launch_bounds__(256) void cnn_conv_wgrad_update_kernel(CnnDev d, RoundDesc rd, int layer) {
  __shared__ float sred[kMaxCout][257];
  const CnnPlan& p = d.p;
  const int t = threadIdx.x, k = p.k;
  const int Cin = layer ? p.C1 : p.C0, Cout = layer ? p.C2 : p.C1;
  const int Sin = layer ? p.S1 : p.S, Sp = layer ? p.S2 : p.S1;
  const int n_in = Cin * Sin * Sin, n_out = Cout * Sp * Sp, win = Sp * Sp;
  const int q = blockIdx.x;
  const bool bias = q == Cin * k * k;
  const int ci = q / (k * k), u = (q / k) % k, v = q % k;
  const float* dP = wsp<const float>(d, layer ? p.off_dp2 : p.off_dp1);
  const uint8_t* A = wsp<const uint8_t>(d, layer ? p.off_a2 : p.off_a1);
  const float* P1 = wsp<const float>(d, p.off_p1);
  const uint32_t* rowidx = wsp<const uint32_t>(d, p.off_rowidx);
  float acc[kMaxCout];
#pragma unroll
  for (int co = 0; co < kMaxCout; ++co) acc[co] = 0.f;
  const int ra = d.step < 0 ? 0 : (int)blockIdx.y * p.B, nr = d.step < 0 ? d.n_rows : p.B;
  for (int it = t; it < nr * win; it += 256) {
    const int r = ra + it / win, w_ = it % win, pi = w_ / Sp, pj = w_ - pi * Sp;
    const float* in = layer ? P1 + (size_t)r * n_in : d.X + (size_t)rowidx[r] * n_in;
    const float* g = dP + (size_t)r * n_out + w_;
    const uint8_t* ar = A + (size_t)r * n_out + w_;
#pragma unroll
    for (int co = 0; co < kMaxCout; ++co) {
      if (co < Cout) {
        const int m = ar[co * win];
        if (m != kDead) {
          const float gv = g[co * win];
          acc[co] += bias ? gv : in[(ci * Sin + 2 * pi + (m >> 1) + u) * Sin + 2 * pj + (m & 1) + v] * gv;
        }
      }
    }
  }
#pragma unroll
  for (int co = 0; co < kMaxCout; ++co)
    if (co < Cout) sred[co][t] = acc[co];
  __syncthreads();
  if (t < Cout) {
    float g = 0.f;
    for (int i = 0; i < 256; ++i) g += sred[t][i];
    const float* w_cur; float* w_next;
    step_models(d, rd, (int)blockIdx.y, &w_cur, &w_next);
    const size_t at = bias ? p.b_off[layer] + t : p.w_off[layer] + (size_t)q * Cout + t;
    w_next[at] = w_cur[at] - g;
  }
}

// Eq. 3 after U local steps: w^{t+1} = w^t - (1/K) sum_a (w^{t - tau_a} - w_a^U), uploads in arrival
// order; the first workgroup publishes the uploads' mean local losses.
__global__ __launch_bounds__(256) void cnn_delta_update_kernel(CnnDev d, RoundDesc rd, LossMailbox* mailbox) {
  const CnnPlan& p = d.p;
  if (blockIdx.x == 0 && mailbox) {
    const float* lossbuf = wsp<const float>(d, p.off_lossbuf);
    if ((int)threadIdx.x < rd.K) mailbox->loss[threadIdx.x] = lossbuf[threadIdx.x];
    if (threadIdx.x < ABS_MAX_WORKERS) __threadfence_system();
    __syncthreads();
    if (threadIdx.x == 0) mailbox->stamp = rd.stamp;
  }
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= p.P) return;
  const float* ring = wsp<const float>(d, p.off_ring);
  const float* priv = wsp<const float>(d, p.off_priv);
  float sum = 0.f;
  for (int a = 0; a < rd.K; ++a)
    sum += ring[(size_t)rd.w[a].slot * p.slot_stride + e] - priv[(size_t)a * p.slot_stride + e];
  wsp<float>(d, p.off_ring)[(size_t)rd.slot_next * p.slot_stride + e] =
      ring[(size_t)rd.slot_cur * p.slot_stride + e] - sum / (float)rd.K;
}

size_t conv_fwd_lds(const CnnPlan& p, int layer) {
  const int Cin = layer ? p.C1 : p.C0, Cout = layer ? p.C2 : p.C1, Sin = layer ? p.S1 : p.S;
  return ((size_t)Cin * Sin * Sin + (size_t)Cin * p.k * p.k * Cout + Cout) * 4;
}
size_t dense_lds(const CnnPlan& p) {
  return (size_t)p.B * (p.F0 + 2 * p.F1 + 2 * p.F2 + p.C + 1) * 4;
}
size_t conv2_bwd_lds(const CnnPlan& p) {
  return ((size_t)p.C2 * 4 * p.S2 * p.S2 + (size_t)p.C1 * p.k * p.k * p.C2) * 4;
}

CnnDev dev_of(const CnnArgs& a) {
  CnnDev d{};
  d.p = a.plan; d.ws = a.ws; d.X = a.X; d.y = a.y;
  d.shard_rows = a.shard_rows; d.batch_key = a.batch_key;
  d.fixed_slot = -1; d.row0 = 0; d.n_rows = 0;
  d.step = -1; d.U = 1;
  return d;
}

}  // namespace

bool cnn_plan(const abs_config& c, CnnPlan& p, const char** why) {
  auto bad = [&](const char* m) { if (why) *why = m; return false; };
  if (c.n_layers != 5) return bad("CNN: n_layers must be 5 (two convolutional + three dense layers)");
  p.C1 = c.dims[1]; p.C2 = c.dims[2]; p.F1 = c.dims[3]; p.F2 = c.dims[4]; p.C = c.dims[5];
  p.C0 = c.dims[6]; p.k = c.dims[7];
  if (p.C0 < 1 || p.C0 > 4 || p.k < 1 || p.k > 7) return bad("CNN: 1 <= C0 <= 4, 1 <= k <= 7");
  if (c.dims[0] < 1 || c.dims[0] % p.C0) return bad("CNN: dims[0] must be C0 * S * S");
  int S = 1;
  while (S * S < c.dims[0] / p.C0) ++S;
  if (S * S * p.C0 != c.dims[0] || S > 64) return bad("CNN: dims[0] must be C0 * S * S with S <= 64");
  p.S = S;
  const int S1c = S - p.k + 1;
  if (S1c < 2 || S1c % 2) return bad("CNN: S - k + 1 must be even and positive");
  p.S1 = S1c / 2;
  const int S2c = p.S1 - p.k + 1;
  if (S2c < 2 || S2c % 2) return bad("CNN: S1 - k + 1 must be even and positive");
  p.S2 = S2c / 2;
  p.F0 = p.C2 * p.S2 * p.S2;
  if (p.C1 < 1 || p.C1 > kMaxCout || p.C2 < 1 || p.C2 > kMaxCout) return bad("CNN: 1 <= C1, C2 <= 32");
  if (p.F1 < 1 || p.F1 > 1024 || p.F2 < 1 || p.F2 > 1024 || p.C < 2 || p.C > 64) return bad("CNN: dense widths out of range");
  if (c.x_dtype != ABS_X_FP32) return bad("CNN: X must be fp32");
  p.B = c.B; p.N = c.N; p.R = c.tau_cap + 3;
  if (conv_fwd_lds(p, 0) > 150 * 1024 || conv_fwd_lds(p, 1) > 150 * 1024 || dense_lds(p) > 150 * 1024 ||
      conv2_bwd_lds(p) > 150 * 1024)
    return bad("CNN: a stage does not fit the LDS (smaller B, image or layers)");
  const int kk = p.k * p.k;
  const int rows[5] = {p.C0 * kk, p.C1 * kk, p.F0, p.F1, p.F2}, cols[5] = {p.C1, p.C2, p.F1, p.F2, p.C};
  size_t o = 0;
  for (int l = 0; l < 5; ++l) {
    p.w_off[l] = o; o += (size_t)rows[l] * cols[l];
    p.b_off[l] = o; o += (size_t)cols[l];
  }
  p.P = o;
  p.slot_stride = (o + 63) / 64 * 64;
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  const size_t Rm = (size_t)p.N * p.B, n1 = (size_t)p.C1 * p.S1 * p.S1;
  size_t off = 0;
  p.off_ring = off;    off = up(off + (size_t)p.R * p.slot_stride * 4);
  p.off_rowidx = off;  off = up(off + Rm * 4);
  p.off_label = off;   off = up(off + Rm * 4);
  p.off_p1 = off;      off = up(off + Rm * n1 * 4);
  p.off_a1 = off;      off = up(off + Rm * n1);
  p.off_p2 = off;      off = up(off + Rm * p.F0 * 4);
  p.off_a2 = off;      off = up(off + Rm * p.F0);
  p.off_h1 = off;      off = up(off + Rm * p.F1 * 4);
  p.off_h2 = off;      off = up(off + Rm * p.F2 * 4);
  p.off_dz1 = off;     off = up(off + Rm * p.F1 * 4);
  p.off_dz2 = off;     off = up(off + Rm * p.F2 * 4);
  p.off_dz3 = off;     off = up(off + Rm * p.C * 4);
  p.off_dp2 = off;     off = up(off + Rm * p.F0 * 4);
  p.off_dp1 = off;     off = up(off + Rm * n1 * 4);
  p.off_lossbuf = off; off = up(off + (size_t)p.N * 4);
  p.U = c.U < 1 ? 1 : c.U;
  p.off_priv = off;    if (p.U > 1) off = up(off + (size_t)p.N * p.slot_stride * 4);
  p.off_eval = off;    off = up(off + eval_scratch_bytes(Rm));
  p.total = off;
  return true;
}

hipError_t launch_cnn_round(const CnnArgs& a, const RoundDesc& rd, hipStream_t s, LaunchHook* hook) {
  const CnnPlan& p = a.plan;
  CnnDev d = dev_of(a);
  const int rows = rd.K * p.B;
  d.n_rows = rows;
  d.U = p.U;
  const bool local = p.U > 1;
  const unsigned ups = local ? (unsigned)rd.K : 1u;      // weight-gradient launches: one sum per upload
  const double ar = (double)rows, kk = (double)p.k * p.k;
  const double f1 = 2.0 * ar * p.C1 * 4.0 * p.S1 * p.S1 * p.C0 * kk, f2 = 2.0 * ar * p.C2 * 4.0 * p.S2 * p.S2 * p.C1 * kk;
  const double fd = 2.0 * ar * ((double)p.F0 * p.F1 + (double)p.F1 * p.F2 + (double)p.F2 * p.C);
  const double n1 = (double)p.C1 * p.S1 * p.S1;
  const long n_dense = (long)p.F0 * p.F1 + p.F1 + (long)p.F1 * p.F2 + p.F2 + (long)p.F2 * p.C + p.C;
  for (int step = 0; step < p.U; ++step) {
    d.step = local ? step : -1;
    hook->begin(KK_CNN_CONV_FWD, f1 + f2, ar * 4.0 * (p.C0 * (double)p.S * p.S + 2.0 * n1 + p.F0));
    cnn_conv_pool_fwd_kernel<<<dim3(rows), dim3(256), conv_fwd_lds(p, 0), s>>>(d, rd, 0);
    cnn_conv_pool_fwd_kernel<<<dim3(rows), dim3(256), conv_fwd_lds(p, 1), s>>>(d, rd, 1);
    hook->end(KK_CNN_CONV_FWD);
    hook->begin(KK_CNN_DENSE, 2.0 * fd, ar * 4.0 * (2.0 * p.F0 + 2.0 * p.F1 + 2.0 * p.F2 + p.C));
    cnn_dense_kernel<<<dim3(rd.K), dim3(256), dense_lds(p), s>>>(d, rd, nullptr, nullptr);
    hook->end(KK_CNN_DENSE);
    // the second convolution's input gradient needs that layer's filters as they were in the forward
    // pass: before its weight-gradient launch steps a private model in place
    hook->begin(KK_CNN_CONV_BWD, 2.0 * ar * n1 * kk * p.C2, ar * 4.0 * (p.F0 + n1));
    cnn_conv2_bwd_kernel<<<dim3(rows), dim3(256), conv2_bwd_lds(p), s>>>(d, rd);
    hook->end(KK_CNN_CONV_BWD);
    hook->begin(KK_CNN_DENSE_WGRAD, fd, (double)n_dense * 8.0 + ar * 4.0 * (p.F0 + 2.0 * p.F1 + 2.0 * p.F2 + p.C));
    cnn_dense_wgrad_update_kernel<<<dim3((unsigned)((n_dense + 255) / 256), ups), dim3(256), 0, s>>>(
        d, rd, local ? nullptr : a.mailbox);
    hook->end(KK_CNN_DENSE_WGRAD);
    hook->begin(KK_CNN_CONV_WGRAD, (f1 + f2) / 4.0, ar * 4.0 * (p.C0 * (double)p.S * p.S + 2.0 * n1 + p.F0));
    cnn_conv_wgrad_update_kernel<<<dim3(p.C1 * p.k * p.k + 1, ups), dim3(256), 0, s>>>(d, rd, 1);
    cnn_conv_wgrad_update_kernel<<<dim3(p.C0 * p.k * p.k + 1, ups), dim3(256), 0, s>>>(d, rd, 0);
    hook->end(KK_CNN_CONV_WGRAD);
  }
  if (local) {
    hook->begin(KK_DELTA_UPDATE, (double)p.P * rd.K, (double)p.P * 4.0 * (2.0 * rd.K + 2.0));
    cnn_delta_update_kernel<<<dim3((unsigned)((p.P + 255) / 256)), dim3(256), 0, s>>>(d, rd, a.mailbox);
    hook->end(KK_DELTA_UPDATE);
  }
  return hipGetLastError();
}

hipError_t launch_cnn_eval(const CnnArgs& a, uint32_t slot, const EvalArgs& e, hipStream_t s, LaunchHook* hook) {
  const CnnPlan& p = a.plan;
  RoundDesc rd{};
  hipError_t err = launch_eval_clear(e, s);
  const int64_t pass = (int64_t)p.N * p.B;
  for (int64_t row0 = 0; row0 < e.n_rows && err == hipSuccess; row0 += pass) {
    const int n = (int)(e.n_rows - row0 < pass ? e.n_rows - row0 : pass);
    CnnDev d = dev_of(a);
    d.X = (const float*)e.X; d.y = (const int32_t*)e.y;
    d.fixed_slot = (int)slot; d.row0 = row0; d.n_rows = n;
    hook->begin(KK_EVAL, 0.0, 4.0 * n * p.C0 * p.S * p.S);
    cnn_conv_pool_fwd_kernel<<<dim3(n), dim3(256), conv_fwd_lds(p, 0), s>>>(d, rd, 0);
    cnn_conv_pool_fwd_kernel<<<dim3(n), dim3(256), conv_fwd_lds(p, 1), s>>>(d, rd, 1);
    cnn_dense_kernel<<<dim3((n + p.B - 1) / p.B), dim3(256), dense_lds(p), s>>>(d, rd, e.rowloss, e.correct);
    hook->end(KK_EVAL);
    err = hipGetLastError();
    if (err == hipSuccess) err = launch_eval_reduce(e, n, s, hook);
  }
  return err;
}

hipError_t cnn_prepare() {
  // stages whose LDS need exceeds the default limit must opt in once per process
  static hipError_t done = [] {
    hipError_t e = hipFuncSetAttribute((const void*)cnn_conv_pool_fwd_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)cnn_dense_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)cnn_conv2_bwd_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    return e;
  }();
  return done;
}

}  // namespace abs_impl
