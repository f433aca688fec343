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
constexpr int kMaxCout = 32;

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
// layer 0: dataset rows -> first pooled map; layer 1: first pooled map -> second pooled map (the
// dense stack's input).
// KS: the filter size when it is 3 or 5 (loops over a filter row unrolled, a row of inputs fetched
// once for its KS taps), 0: any size.
template <int KS>
__global__ __launch_bounds__(256) void cnn_conv_pool_fwd_kernel(CnnDev d, RoundDesc rd, int layer) {
  extern __shared__ __attribute__((aligned(16))) float sm[];
  const CnnPlan& p = d.p;
  const int r = blockIdx.x, a = r / p.B, t = threadIdx.x;
  const int Cin = layer ? p.C1 : p.C0, Cout = layer ? p.C2 : p.C1;
  const int Sin = layer ? p.S1 : p.S, Sp = layer ? p.S2 : p.S1, k = KS ? KS : p.k;
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
        if (KS) {
          float xa[KS + 1], xb[KS + 1];
#pragma unroll
          for (int v = 0; v <= KS; ++v) { xa[v] = x0[v]; xb[v] = x0[v + Sin]; }
#pragma unroll
          for (int v = 0; v < KS; ++v) {
            const float wv = wr[v * Cout];
            a0 = fmaf(xa[v], wv, a0);
            a1 = fmaf(xa[v + 1], wv, a1);
            a2 = fmaf(xb[v], wv, a2);
            a3 = fmaf(xb[v + 1], wv, a3);
          }
        } else {
          for (int v = 0; v < k; ++v) {
            const float wv = wr[v * Cout];
            a0 = fmaf(x0[v], wv, a0);
            a1 = fmaf(x0[v + 1], wv, a1);
            a2 = fmaf(x0[v + Sin], wv, a2);
            a3 = fmaf(x0[v + Sin + 1], wv, a3);
          }
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

constexpr int kGroup = 8;       // stacked rows per workgroup of the dense stage

// out[b][j] = bias[j] + sum_i in[b][i] W[i][j] for the workgroup's nb <= 8 rows in LDS: a thread
// takes one column, so a weight is fetched once for all rows and neighbouring threads read
// neighbouring weights; eight weights of a column are in flight at a time.
__device__ __forceinline__ void dense_rows(const float* s_in, int Fin, const float* W, const float* bias, int Fout,
                                           int nb, bool relu, float* s_out, float* g_out) {
  for (int j = threadIdx.x; j < Fout; j += blockDim.x) {
    float acc[kGroup];
    const float bv = bias[j];
#pragma unroll
    for (int q = 0; q < kGroup; ++q) acc[q] = bv;
    int i = 0;
    for (; i + 8 <= Fin; i += 8) {
      float wv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) wv[e] = W[(size_t)(i + e) * Fout + j];
#pragma unroll
      for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int q = 0; q < kGroup; ++q) acc[q] = fmaf(s_in[q * Fin + i + e], wv[e], acc[q]);
    }
    for (; i < Fin; ++i) {
      const float wv = W[(size_t)i * Fout + j];
#pragma unroll
      for (int q = 0; q < kGroup; ++q) acc[q] = fmaf(s_in[q * Fin + i], wv, acc[q]);
    }
#pragma unroll
    for (int q = 0; q < kGroup; ++q)
      if (q < nb) {
        const float v = relu ? fmaxf(acc[q], 0.f) : acc[q];
        s_out[q * Fout + j] = v;
        if (g_out) g_out[(size_t)q * Fout + j] = v;
      }
  }
}

// dIn[b][i] = gate(b, i) ? sum_j dOut[b][j] W[i][j] : 0 for the group's rows: a thread takes input
// feature i for all rows, so a weight row is fetched once.
template <typename Gate>
__device__ __forceinline__ void dense_rows_back(const float* s_dout, int Fout, const float* W, int Fin, int nb,
                                                Gate gate, float* s_din, float* g_din) {
  for (int i = threadIdx.x; i < Fin; i += blockDim.x) {
    float acc[kGroup];
#pragma unroll
    for (int q = 0; q < kGroup; ++q) acc[q] = 0.f;
    const float* wr = W + (size_t)i * Fout;
    int j = 0;
    for (; j + 4 <= Fout; j += 4) {
      const float w0 = wr[j], w1 = wr[j + 1], w2 = wr[j + 2], w3 = wr[j + 3];
#pragma unroll
      for (int q = 0; q < kGroup; ++q) {
        const float* dz = s_dout + q * Fout + j;
        acc[q] = fmaf(dz[0], w0, acc[q]); acc[q] = fmaf(dz[1], w1, acc[q]);
        acc[q] = fmaf(dz[2], w2, acc[q]); acc[q] = fmaf(dz[3], w3, acc[q]);
      }
    }
    for (; j < Fout; ++j) {
      const float wv = wr[j];
#pragma unroll
      for (int q = 0; q < kGroup; ++q) acc[q] = fmaf(s_dout[q * Fout + j], wv, acc[q]);
    }
#pragma unroll
    for (int q = 0; q < kGroup; ++q)
      if (q < nb) {
        const float v = gate(q, i) ? acc[q] : 0.f;
        if (s_din) s_din[q * Fin + i] = v;
        g_din[(size_t)q * Fin + i] = v;
      }
  }
}

// The dense stack for a group of up to 8 rows of one upload (training) or of the evaluation pass:
// forward at the rows' model version, per-row loss, and (training) back down to the gradient of the
// second pooled map; every dZ carries the upload's coefficient of Eq. 3.
__global__ __launch_bounds__(256) void cnn_dense_kernel(CnnDev d, RoundDesc rd, float* eval_loss, float* eval_hit) {
  extern __shared__ __attribute__((aligned(16))) float sm[];
  const CnnPlan& p = d.p;
  const int t = threadIdx.x;
  const int gpu_ = (p.B + kGroup - 1) / kGroup;            // groups per upload
  const int a = blockIdx.x / gpu_, g = blockIdx.x - a * gpu_;
  const int r0 = a * p.B + g * kGroup;
  const int nb = min(kGroup, min(p.B - g * kGroup, d.n_rows - r0));
  if (nb <= 0) return;
  float* sH0 = sm;
  float* sH1 = sH0 + kGroup * p.F0;
  float* sH2 = sH1 + kGroup * p.F1;
  float* sZ = sH2 + kGroup * p.F2;
  float* sD2 = sZ + kGroup * p.C;       // dZ of the second dense layer
  float* sD1 = sD2 + kGroup * p.F2;     // dZ of the first dense layer
  const float* w = slot_of(d, rd, a);
  const float* p2 = wsp<const float>(d, p.off_p2) + (size_t)r0 * p.F0;
  for (int i = t; i < kGroup * p.F0; i += 256) sH0[i] = i < nb * p.F0 ? p2[i] : 0.f;
  __syncthreads();
  const bool train = eval_loss == nullptr;
  dense_rows(sH0, p.F0, w + p.w_off[2], w + p.b_off[2], p.F1, nb, true, sH1,
             train ? wsp<float>(d, p.off_h1) + (size_t)r0 * p.F1 : nullptr);
  __syncthreads();
  dense_rows(sH1, p.F1, w + p.w_off[3], w + p.b_off[3], p.F2, nb, true, sH2,
             train ? wsp<float>(d, p.off_h2) + (size_t)r0 * p.F2 : nullptr);
  __syncthreads();
  dense_rows(sH2, p.F2, w + p.w_off[4], w + p.b_off[4], p.C, nb, false, sZ, nullptr);
  __syncthreads();
  const int32_t* label = wsp<const int32_t>(d, p.off_label) + r0;
  if (t < nb) {
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
      wsp<float>(d, p.off_rowloss)[r0 + t] = loss;
    } else {
      eval_loss[r0 + t] = loss;
      eval_hit[r0 + t] = best == y ? 1.f : 0.f;
    }
  }
  if (!train) return;
  __syncthreads();
  dense_rows_back(sZ, p.C, w + p.w_off[4], p.F2, nb, [&](int b, int i) { return sH2[b * p.F2 + i] > 0.f; }, sD2,
                  wsp<float>(d, p.off_dz2) + (size_t)r0 * p.F2);
  __syncthreads();
  dense_rows_back(sD2, p.F2, w + p.w_off[3], p.F1, nb, [&](int b, int i) { return sH1[b * p.F1 + i] > 0.f; }, sD1,
                  wsp<float>(d, p.off_dz1) + (size_t)r0 * p.F1);
  __syncthreads();
  const uint8_t* a2 = wsp<const uint8_t>(d, p.off_a2) + (size_t)r0 * p.F0;
  dense_rows_back(sD1, p.F1, w + p.w_off[2], p.F0, nb, [&](int b, int i) { return a2[b * p.F0 + i] != kDead; }, nullptr,
                  wsp<float>(d, p.off_dp2) + (size_t)r0 * p.F0);
}

// The dense layers' share of an upload's gradient (blockIdx.y = upload): element e of the three
// weight matrices and biases summed over the upload's B rows in row order.  U = 1: the sum goes to
// the upload's slot of G (Eq. 3 adds the slots in arrival order, cnn_combine_kernel); local steps:
// the upload's private model takes the step at once (Eq. 2).
__global__ __launch_bounds__(256) void cnn_dense_wgrad_kernel(CnnDev d, RoundDesc rd) {
  const CnnPlan& p = d.p;
  const int a = blockIdx.y;
  const int Fin[3] = {p.F0, p.F1, p.F2}, Fout[3] = {p.F1, p.F2, p.C};
  const size_t in_off[3] = {p.off_p2, p.off_h1, p.off_h2}, dz_off[3] = {p.off_dz1, p.off_dz2, p.off_dz3};
  long e = (long)blockIdx.x * 256 + threadIdx.x;
  const int ra = a * p.B, rb = ra + p.B;
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
      float* priv = wsp<float>(d, p.off_priv) + (size_t)a * p.slot_stride;
      priv[at] = d.step < 0 ? g : slot_of(d, rd, a)[at] - g;
      return;
    }
    e -= n;
  }
}

// Gradient of the first pooled map of row r: the second convolution's output gradient is non-zero
// only where a pooling window had its (positive) maximum.
// LDS: the output gradient as [row][column][channel] and the filters as [(ci, u, v)][channel], channels
// padded to a multiple of 4, so that the sum over output channels runs on 16-byte reads.
template <int KS>
__global__ __launch_bounds__(256) void cnn_conv2_bwd_kernel(CnnDev d, RoundDesc rd) {
  extern __shared__ __attribute__((aligned(16))) float sm[];
  const CnnPlan& p = d.p;
  const int r = blockIdx.x, a = r / p.B, t = threadIdx.x, k = KS ? KS : p.k;
  const int S2c = 2 * p.S2, Cp = (p.C2 + 3) & ~3, n_dc = S2c * S2c * Cp, n_q = p.C1 * k * k;
  float* sdc = sm;             // [S2c][S2c][Cp]
  float* sw = sdc + n_dc;      // [C1 k k][Cp]: second convolution's filters of this upload's version
  const float* w = slot_of(d, rd, a);
  for (int i = t; i < n_dc; i += 256) sdc[i] = 0.f;
  for (int i = t; i < n_q * Cp; i += 256) {
    const int q = i / Cp, co = i - q * Cp;
    sw[i] = co < p.C2 ? w[p.w_off[1] + (size_t)q * p.C2 + co] : 0.f;
  }
  __syncthreads();
  const float* dp2 = wsp<const float>(d, p.off_dp2) + (size_t)r * p.F0;
  const uint8_t* a2 = wsp<const uint8_t>(d, p.off_a2) + (size_t)r * p.F0;
  for (int o = t; o < p.F0; o += 256) {
    const int q = a2[o];
    if (q != kDead) {
      const int co = o / (p.S2 * p.S2), pi = (o / p.S2) % p.S2, pj = o % p.S2;
      sdc[((2 * pi + (q >> 1)) * S2c + 2 * pj + (q & 1)) * Cp + co] = dp2[o];
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
#pragma unroll
      for (int u = 0; u < (KS ? KS : k); ++u) {
        const int i = y - u;
        if (i < 0 || i >= S2c) continue;
#pragma unroll
        for (int v = 0; v < (KS ? KS : k); ++v) {
          const int j = x - v;
          if (j < 0 || j >= S2c) continue;
          const float4* wr = (const float4*)(sw + ((ci * k + u) * k + v) * Cp);
          const float4* gr = (const float4*)(sdc + (i * S2c + j) * Cp);
          for (int c4 = 0; c4 < Cp / 4; ++c4) {
            const float4 gv = gr[c4], wv = wr[c4];
            acc = fmaf(gv.x, wv.x, acc); acc = fmaf(gv.y, wv.y, acc);
            acc = fmaf(gv.z, wv.z, acc); acc = fmaf(gv.w, wv.w, acc);
          }
        }
      }
    }
    dp1[o] = acc;
  }
}

// A convolution's share of one row's gradient (workgroup = stacked row): the row's input map, the
// gradient of its pooled map and the windows' maxima in LDS; a thread sums one filter weight
// (ci, u, v, co) over the pooling windows (a window contributes the input under its maximum), the
// last Cout entries are the bias.  Result: Grow[r][weights..., biases...], in the model's own order.
__global__ __launch_bounds__(256) void cnn_conv_wgrad_rows_kernel(CnnDev d, int layer) {
  extern __shared__ __attribute__((aligned(16))) float sm[];
  const CnnPlan& p = d.p;
  const int r = blockIdx.x, t = threadIdx.x, k = p.k;
  const int Cin = layer ? p.C1 : p.C0, Cout = layer ? p.C2 : p.C1;
  const int Sin = layer ? p.S1 : p.S, Sp = layer ? p.S2 : p.S1;
  const int n_in = Cin * Sin * Sin, n_out = Cout * Sp * Sp, win = Sp * Sp, nW = Cin * k * k * Cout;
  float* sx = sm;
  float* sg = sx + n_in;
  int* sa = (int*)(sg + n_out);
  const float* in = layer ? wsp<const float>(d, p.off_p1) + (size_t)r * n_in
                          : d.X + (size_t)wsp<const uint32_t>(d, p.off_rowidx)[r] * n_in;
  const float* g = wsp<const float>(d, layer ? p.off_dp2 : p.off_dp1) + (size_t)r * n_out;
  const uint8_t* A = wsp<const uint8_t>(d, layer ? p.off_a2 : p.off_a1) + (size_t)r * n_out;
  for (int i = t; i < n_in; i += 256) sx[i] = in[i];
  for (int i = t; i < n_out; i += 256) {
    const int m = A[i], w_ = i % win, pi = w_ / Sp, pj = w_ - pi * Sp;
    sg[i] = m == kDead ? 0.f : g[i];
    // offset of the window's maximum inside an input plane (a dead window contributes 0 x its corner)
    sa[i] = (2 * pi + (m == kDead ? 0 : (m >> 1))) * Sin + 2 * pj + (m == kDead ? 0 : (m & 1));
  }
  __syncthreads();
  float* out = wsp<float>(d, layer ? p.off_grow2 : p.off_grow1) + (size_t)r * (nW + Cout);
  for (int e = t; e < nW + Cout; e += 256) {
    float acc = 0.f;
    if (e < nW) {
      const int co = e % Cout, q = e / Cout, ci = q / (k * k), u = (q / k) % k, v = q % k;
      const float* x0 = sx + (ci * Sin + u) * Sin + v;
      const float* gg = sg + co * win;
      const int* aa = sa + co * win;
      for (int w_ = 0; w_ < win; ++w_) acc = fmaf(x0[aa[w_]], gg[w_], acc);
    } else {
      const float* gg = sg + (e - nW) * win;
      for (int w_ = 0; w_ < win; ++w_) acc += gg[w_];
    }
    out[e] = acc;
  }
}

// From the rows' and uploads' shares to the stepped model, parameter e per thread:
//   kPerUpload (blockIdx.y = upload): a convolution parameter's shares of the upload's own rows, added in
//     row order; with local steps the upload's private model takes the step (Eq. 2; the dense
//     parameters took theirs in cnn_dense_wgrad_kernel), at U = 1 the sum joins the dense shares in the
//     upload's slot of G;
//   kAcrossUploads (U = 1): Eq. 3, w^{t+1} = w^t - the uploads' shares added in arrival order.
// The first workgroup of kPerUpload / local and of kAcrossUploads turns the row losses into the uploads'
// mean minibatch losses and, at U = 1, publishes them.
enum { kPerUpload = 0, kAcrossUploads = 1 };
__global__ __launch_bounds__(256) void cnn_combine_kernel(CnnDev d, RoundDesc rd, int mode, LossMailbox* mailbox) {
  const CnnPlan& p = d.p;
  const bool local = d.step >= 0;
  if (blockIdx.x == 0 && blockIdx.y == 0 && (local || mode == kAcrossUploads)) {
    const int a = threadIdx.x;
    if (a < rd.K) {
      const float* rl = wsp<const float>(d, p.off_rowloss) + (size_t)a * p.B;
      float sum = 0.f;
      for (int b = 0; b < p.B; ++b) sum += rl[b];
      const float mean = sum / (float)p.B;
      float* lb = wsp<float>(d, p.off_lossbuf) + a;
      if (!local) *lb = mean;
      else *lb = (d.step == 0 ? 0.f : *lb) + mean / (float)d.U;       // mean over the job's U steps
      if (mailbox) mailbox->loss[a] = mean;
    }
    if (mailbox) {
      if (threadIdx.x < ABS_MAX_WORKERS) __threadfence_system();
      __syncthreads();
      if (threadIdx.x == 0) mailbox->stamp = rd.stamp;
    }
  }
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= p.P) return;
  const int a = blockIdx.y;
  float sum = 0.f;
  if (mode == kPerUpload) {
    if (e >= p.w_off[2]) return;                       // convolution parameters only
    const int layer = e >= p.w_off[1] ? 1 : 0;
    const size_t n = (layer ? p.w_off[2] : p.w_off[1]) - p.w_off[layer], idx = e - p.w_off[layer];
    const float* G = wsp<const float>(d, layer ? p.off_grow2 : p.off_grow1);
    for (int r = a * p.B; r < (a + 1) * p.B; ++r) sum += G[(size_t)r * n + idx];
    float* priv = wsp<float>(d, p.off_priv) + (size_t)a * p.slot_stride;
    priv[e] = local ? slot_of(d, rd, a)[e] - sum : sum;
  } else {
    const float* G = wsp<const float>(d, p.off_priv);
    for (int k = 0; k < rd.K; ++k) sum += G[(size_t)k * p.slot_stride + e];
    const float* ring = wsp<const float>(d, p.off_ring);
    wsp<float>(d, p.off_ring)[(size_t)rd.slot_next * p.slot_stride + e] = ring[(size_t)rd.slot_cur * p.slot_stride + e] - sum;
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
  return (size_t)kGroup * (p.F0 + 2 * p.F1 + 2 * p.F2 + p.C) * 4;
}
size_t conv_wgrad_lds(const CnnPlan& p, int layer) {
  const int Cin = layer ? p.C1 : p.C0, Cout = layer ? p.C2 : p.C1, Sin = layer ? p.S1 : p.S, Sp = layer ? p.S2 : p.S1;
  return ((size_t)Cin * Sin * Sin + 2 * (size_t)Cout * Sp * Sp) * 4;
}
size_t conv2_bwd_lds(const CnnPlan& p) {
  const size_t Cp = (size_t)((p.C2 + 3) & ~3);
  return (Cp * 4 * p.S2 * p.S2 + (size_t)p.C1 * p.k * p.k * Cp) * 4;
}

void launch_conv_fwd(const CnnDev& d, const RoundDesc& rd, int rows, hipStream_t s) {
  const CnnPlan& p = d.p;
  for (int layer = 0; layer < 2; ++layer) {
    const size_t lds = conv_fwd_lds(p, layer);
    switch (p.k) {
      case 3: cnn_conv_pool_fwd_kernel<3><<<dim3(rows), dim3(256), lds, s>>>(d, rd, layer); break;
      case 5: cnn_conv_pool_fwd_kernel<5><<<dim3(rows), dim3(256), lds, s>>>(d, rd, layer); break;
      default: cnn_conv_pool_fwd_kernel<0><<<dim3(rows), dim3(256), lds, s>>>(d, rd, layer);
    }
  }
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
      conv2_bwd_lds(p) > 150 * 1024 || conv_wgrad_lds(p, 0) > 150 * 1024 || conv_wgrad_lds(p, 1) > 150 * 1024)
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
  p.off_rowloss = off; off = up(off + Rm * 4);
  p.U = c.U < 1 ? 1 : c.U;
  p.off_priv = off;    off = up(off + (size_t)p.N * p.slot_stride * 4);
  p.off_grow1 = off;   off = up(off + Rm * (p.w_off[1] - p.w_off[0]) * 4);
  p.off_grow2 = off;   off = up(off + Rm * (p.w_off[2] - p.w_off[1]) * 4);
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
  const double ar = (double)rows, kk = (double)p.k * p.k;
  const double f1 = 2.0 * ar * p.C1 * 4.0 * p.S1 * p.S1 * p.C0 * kk, f2 = 2.0 * ar * p.C2 * 4.0 * p.S2 * p.S2 * p.C1 * kk;
  const double fd = 2.0 * ar * ((double)p.F0 * p.F1 + (double)p.F1 * p.F2 + (double)p.F2 * p.C);
  const double n1 = (double)p.C1 * p.S1 * p.S1;
  const long n_dense = (long)p.F0 * p.F1 + p.F1 + (long)p.F1 * p.F2 + p.F2 + (long)p.F2 * p.C + p.C;
  const unsigned groups = (unsigned)(rd.K * ((p.B + kGroup - 1) / kGroup));
  for (int step = 0; step < p.U; ++step) {
    d.step = local ? step : -1;
    hook->begin(KK_CNN_CONV_FWD, f1 + f2, ar * 4.0 * (p.C0 * (double)p.S * p.S + 2.0 * n1 + p.F0));
    launch_conv_fwd(d, rd, rows, s);
    hook->end(KK_CNN_CONV_FWD);
    hook->begin(KK_CNN_DENSE, 2.0 * fd, ar * 4.0 * (2.0 * p.F0 + 2.0 * p.F1 + 2.0 * p.F2 + p.C));
    cnn_dense_kernel<<<dim3(groups), dim3(256), dense_lds(p), s>>>(d, rd, nullptr, nullptr);
    hook->end(KK_CNN_DENSE);
    // everything that reads a model comes before the kernels that step a private model in place
    hook->begin(KK_CNN_CONV_BWD, 2.0 * ar * n1 * kk * p.C2, ar * 4.0 * (p.F0 + n1));
    switch (p.k) {
      case 3: cnn_conv2_bwd_kernel<3><<<dim3(rows), dim3(256), conv2_bwd_lds(p), s>>>(d, rd); break;
      case 5: cnn_conv2_bwd_kernel<5><<<dim3(rows), dim3(256), conv2_bwd_lds(p), s>>>(d, rd); break;
      default: cnn_conv2_bwd_kernel<0><<<dim3(rows), dim3(256), conv2_bwd_lds(p), s>>>(d, rd);
    }
    hook->end(KK_CNN_CONV_BWD);
    hook->begin(KK_CNN_DENSE_WGRAD, fd, (double)n_dense * 8.0 + ar * 4.0 * (p.F0 + 2.0 * p.F1 + 2.0 * p.F2 + p.C));
    cnn_dense_wgrad_kernel<<<dim3((unsigned)((n_dense + 255) / 256), (unsigned)rd.K), dim3(256), 0, s>>>(d, rd);
    hook->end(KK_CNN_DENSE_WGRAD);
    hook->begin(KK_CNN_CONV_WGRAD, (f1 + f2) / 4.0, ar * 4.0 * (p.C0 * (double)p.S * p.S + 2.0 * n1 + p.F0));
    cnn_conv_wgrad_rows_kernel<<<dim3(rows), dim3(256), conv_wgrad_lds(p, 1), s>>>(d, 1);
    cnn_conv_wgrad_rows_kernel<<<dim3(rows), dim3(256), conv_wgrad_lds(p, 0), s>>>(d, 0);
    hook->end(KK_CNN_CONV_WGRAD);
    hook->begin(KK_CNN_COMBINE, (double)p.P * rd.K, 4.0 * (ar * (double)p.w_off[2] + (double)rd.K * n_dense + 2.0 * p.P));
    cnn_combine_kernel<<<dim3((unsigned)((p.w_off[2] + 255) / 256), (unsigned)rd.K), dim3(256), 0, s>>>(d, rd, kPerUpload, nullptr);
    if (!local)
      cnn_combine_kernel<<<dim3((unsigned)((p.P + 255) / 256)), dim3(256), 0, s>>>(d, rd, kAcrossUploads, a.mailbox);
    hook->end(KK_CNN_COMBINE);
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
    launch_conv_fwd(d, rd, n, s);
    cnn_dense_kernel<<<dim3((unsigned)(((n + p.B - 1) / p.B) * ((p.B + kGroup - 1) / kGroup))), dim3(256), dense_lds(p), s>>>(
        d, rd, e.rowloss, e.correct);
    hook->end(KK_EVAL);
    err = hipGetLastError();
    if (err == hipSuccess) err = launch_eval_reduce(e, n, s, hook);
  }
  return err;
}

hipError_t cnn_prepare() {
  // stages whose LDS need exceeds the default limit must opt in once per process
  static hipError_t done = [] {
    const void* fns[] = {(const void*)cnn_conv_pool_fwd_kernel<0>, (const void*)cnn_conv_pool_fwd_kernel<3>,
                         (const void*)cnn_conv_pool_fwd_kernel<5>, (const void*)cnn_dense_kernel,
                         (const void*)cnn_conv2_bwd_kernel<0>, (const void*)cnn_conv2_bwd_kernel<3>,
                         (const void*)cnn_conv2_bwd_kernel<5>};
    hipError_t e = hipSuccess;
    for (const void* f : fns)
      if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)cnn_conv_wgrad_rows_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    return e;
  }();
  return done;
}

}  // namespace abs_impl
