// Bandwidth-bound rounds: linear least squares and softmax regression (fp32).
//
// One round = Eq. 2 (U = 1) for each of the K^t uploads at its own stale model,
// the K-of-N reduction and update of Eq. 3, and the snapshot write into the ring.
// Per-upload gradients are never materialised: every row's contribution is scaled
// by its upload's coefficient c = eta_k / (K^t B) and summed straight into the
// aggregate.  All reductions have a fixed order (no floating-point atomics), so a
// round is bitwise reproducible.
#include <hip/hip_runtime.h>
#include <atomic>
#include "kernels.h"

namespace abs_impl {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ uint64_t batch_row(const WorkerDesc& w, uint64_t batch_key,
                                              uint64_t shard_rows, uint32_t b) {
  // minibatch draw b of job w.job of worker w.id: uniform over the worker's own shard
  const uint64_t jk = job_key(batch_key, w.id, w.job);
  return (uint64_t)w.id * shard_rows + draw(jk, b) % shard_rows;
}

// ------------------------------------------------------------------ linear least squares
// One workgroup of 16 wavefronts.  A wavefront owns a contiguous run of the K*B stacked
// rows; a lane owns features lane, lane+64, ... of x, w and the gradient.  Per row: the
// residual by a wavefront reduction, then g += c * r * x in registers.  The 16 partial
// gradients are combined through LDS in wavefront order, followed by w^{t+1} = w^t - G.
constexpr int kLinWaves = 16;

template <int Q>
__device__ __forceinline__ void linreg_round_body(const RegressionArgs& a, const RoundDesc& rd) {
  __shared__ float s_g[kLinWaves][Q * 64];
  __shared__ float s_loss[kLinWaves][ABS_MAX_WORKERS];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int K = rd.K, d = a.d, B = a.B;
  const int R = K * B;
  const float* y = (const float*)a.y;
  for (int i = threadIdx.x; i < kLinWaves * ABS_MAX_WORKERS; i += blockDim.x) (&s_loss[0][0])[i] = 0.f;
  __syncthreads();

  float g[Q];
#pragma unroll
  for (int q = 0; q < Q; ++q) g[q] = 0.f;
  const int per = (R + kLinWaves - 1) / kLinWaves;
  const int r0 = wave * per, r1 = min(R, r0 + per);
  // 64 rows at a time: lane i prepares row i of the chunk (minibatch draw, target, upload),
  // then the rows are processed eight at a time so that their loads overlap.
  for (int c0 = r0; c0 < r1; c0 += 64) {
    const int mine = c0 + lane;
    uint64_t my_row = 0;
    float my_y = 0.f, my_c = 0.f;
    int my_up = 0, my_slot = 0;
    if (mine < r1) {
      my_up = mine / B;
      const WorkerDesc w = rd.w[my_up];
      my_row = batch_row(w, a.batch_key, a.shard_rows, (uint32_t)(mine - my_up * B));
      my_y = y[my_row];
      my_c = w.c;
      my_slot = (int)w.slot;
    }
    const int n = min(64, r1 - c0);
    for (int j0 = 0; j0 < n; j0 += 8) {
      float x[8][Q], dot[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int src = min(j0 + j, n - 1);           // the tail repeats the last row, masked below
        const uint64_t row = __shfl(my_row, src, 64);
        const int slot = __shfl(my_slot, src, 64);
        const float* xr = a.X + row * (uint64_t)d;
        const float* wv = a.ring + (size_t)slot * a.slot_stride;
        dot[j] = 0.f;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
          const int i = lane + 64 * q;
          x[j][q] = i < d ? xr[i] : 0.f;
          const float wi = i < d ? wv[i] : 0.f;
          dot[j] = fmaf(x[j][q], wi, dot[j]);
        }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int src = min(j0 + j, n - 1);
        const float res = wave_sum(dot[j]) - __shfl(my_y, src, 64);
        const float coef = j0 + j < n ? __shfl(my_c, src, 64) * res : 0.f;
        const int up = __shfl(my_up, src, 64);
#pragma unroll
        for (int q = 0; q < Q; ++q) g[q] = fmaf(coef, x[j][q], g[q]);
        if (lane == 0 && j0 + j < n) s_loss[wave][up] += 0.5f * res * res;
      }
    }
  }
#pragma unroll
  for (int q = 0; q < Q; ++q) s_g[wave][lane + 64 * q] = g[q];
  __syncthreads();
  // the losses first: the host prepares the next round while the update is written
  for (int up = threadIdx.x; up < K; up += blockDim.x) {   // thread `up` owns column `up` of s_loss
    float l = 0.f;
#pragma unroll
    for (int w = 0; w < kLinWaves; ++w) l += s_loss[w][up];
    s_loss[0][up] = l / (float)B;
  }
  __syncthreads();
  publish_losses(a.mailbox, &s_loss[0][0], K, rd.stamp);
  const float* cur = a.ring + (size_t)rd.slot_cur * a.slot_stride;
  float* nxt = a.ring + (size_t)rd.slot_next * a.slot_stride;
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    float G = 0.f;
#pragma unroll
    for (int w = 0; w < kLinWaves; ++w) G += s_g[w][i];
    nxt[i] = cur[i] - G;
  }
}
template <int Q>
__global__ __launch_bounds__(kLinWaves * 64) void linreg_round_kernel(RegressionArgs a, RoundDesc rd) {
  linreg_round_body<Q>(a, rd);
}
// Batched form: blockIdx.y = simulation; its arguments and this round's descriptor (a header and
// the K^t uploads, `stride` bytes apart) come from device memory.
template <int Q>
__global__ __launch_bounds__(kLinWaves * 64) void linreg_round_batch_kernel(const RegressionArgs* as, const char* rds,
                                                                            size_t stride) {
  const RegressionArgs a = as[blockIdx.y];
  linreg_round_body<Q>(a, *(const RoundDesc*)(rds + (size_t)blockIdx.y * stride));
}

hipError_t launch_linreg_round(const RegressionArgs& a, const RoundDesc& rd, hipStream_t s,
                               LaunchHook* hook) {
  const double rows = (double)rd.K * a.B;
  hook->begin(KK_LINREG_ROUND, rows * a.d * 4.0, rows * (a.d + 1) * 4.0 + 2.0 * a.d * 4.0);
  const dim3 grid(1), block(kLinWaves * 64);
  if (a.d <= 128)       linreg_round_kernel<2><<<grid, block, 0, s>>>(a, rd);
  else if (a.d <= 256)  linreg_round_kernel<4><<<grid, block, 0, s>>>(a, rd);
  else                  linreg_round_kernel<8><<<grid, block, 0, s>>>(a, rd);   // d <= 512
  hook->end(KK_LINREG_ROUND);
  return hipGetLastError();
}

// ------------------------------------------------------------------ softmax regression
// Kernel 1 (a workgroup per 4 RPW rows of one upload; a wavefront takes RPW rows, RPW = 4 when the
// launch has rows to spare, else 1):
// logits of the row at its upload's stale model, softmax cross-entropy, and the row of
// dZ = c (softmax - onehot).  A lane owns float4 chunks lane, lane+64, ... of x; the matching
// 4 x C block of W is 4C contiguous floats, read as C float4 once per chunk and used for the
// wavefront's RPW rows (a row on its own fetches all of W, ten times its own bytes, from L2).
// The rows' loads are all issued first.  Logits are completed by wavefront reductions.
constexpr int kSoftQF = 4;          // float4 chunks per lane  ->  d <= 1024
constexpr int kDzPitch = 16;        // floats per dZ row (C <= 16)
constexpr int kRowsToSpare = 8192;  // stacked rows of a launch from which a wavefront takes 4 rows

template <int C, int RPW>
__device__ __forceinline__ void softmax_rows_body(const RegressionArgs& a, const RoundDesc& rd) {
  constexpr int kRowsPerBlock = 4 * RPW;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int B = a.B, d = a.d;
  const int bpu = (B + kRowsPerBlock - 1) / kRowsPerBlock;
  const int up = blockIdx.x / bpu, chunk = blockIdx.x - up * bpu;
  if (up >= rd.K) return;
  const WorkerDesc w = rd.w[up];
  const float* Wv = a.ring + (size_t)w.slot * a.slot_stride;
  float bz[C];
#pragma unroll
  for (int c = 0; c < C; ++c) bz[c] = Wv[(size_t)d * C + c];
  const int nchunk = d >> 2;
  // this wavefront's (up to) RPW rows: all their loads first
  float4 xv[RPW][kSoftQF];
  uint64_t rows[RPW];
  int labels[RPW];
#pragma unroll
  for (int k = 0; k < RPW; ++k) {
    const int b = chunk * kRowsPerBlock + wave + 4 * k;
    rows[k] = 0; labels[k] = 0;
    if (b < B) {
      rows[k] = batch_row(w, a.batch_key, a.shard_rows, (uint32_t)b);
      const float4* xr = (const float4*)(a.X + rows[k] * (uint64_t)d);
#pragma unroll
      for (int q = 0; q < kSoftQF; ++q) {
        const int ch = lane + 64 * q;
        xv[k][q] = ch < nchunk ? xr[ch] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
      labels[k] = ((const int32_t*)a.y)[rows[k]];
    }
  }
  // the lane's 4 x C block of W for each of its chunks is fetched once and used for all RPW rows
  float accs[RPW][C];
#pragma unroll
  for (int k = 0; k < RPW; ++k)
#pragma unroll
    for (int c = 0; c < C; ++c) accs[k][c] = 0.f;
#pragma unroll
  for (int q = 0; q < kSoftQF; ++q) {
    const int ch = lane + 64 * q;
    if (ch < nchunk) {
      const float4* wp = (const float4*)(Wv + (size_t)ch * 4 * C);
      float wf[4 * C];
#pragma unroll
      for (int i = 0; i < C; ++i) {
        const float4 t = wp[i];
        wf[4 * i + 0] = t.x; wf[4 * i + 1] = t.y; wf[4 * i + 2] = t.z; wf[4 * i + 3] = t.w;
      }
#pragma unroll
      for (int k = 0; k < RPW; ++k)
#pragma unroll
        for (int c = 0; c < C; ++c) {
          accs[k][c] = fmaf(xv[k][q].x, wf[0 * C + c], accs[k][c]);
          accs[k][c] = fmaf(xv[k][q].y, wf[1 * C + c], accs[k][c]);
          accs[k][c] = fmaf(xv[k][q].z, wf[2 * C + c], accs[k][c]);
          accs[k][c] = fmaf(xv[k][q].w, wf[3 * C + c], accs[k][c]);
        }
    }
  }
#pragma unroll
  for (int k = 0; k < RPW; ++k) {
    const int b = chunk * kRowsPerBlock + wave + 4 * k;
    if (b >= B) break;
    const int r = up * B + b;
    float acc[C];
#pragma unroll
    for (int c = 0; c < C; ++c) acc[c] = accs[k][c];
    float zmax = -INFINITY;
#pragma unroll
    for (int c = 0; c < C; ++c) {
      acc[c] = wave_sum(acc[c]) + bz[c];
      zmax = fmaxf(zmax, acc[c]);
    }
    const int label = labels[k];
    float ssum = 0.f, zy = 0.f, mine = 0.f;
#pragma unroll
    for (int c = 0; c < C; ++c) {
      if (c == label) zy = acc[c] - zmax;
      acc[c] = expf(acc[c] - zmax);
      ssum += acc[c];
    }
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const float p = acc[c] / ssum;
      if (c == lane) mine = w.c * (p - (c == label ? 1.f : 0.f));
    }
    if (lane < kDzPitch) a.dz[(size_t)r * kDzPitch + lane] = lane < C ? mine : 0.f;
    if (lane == 0) {
      // -log softmax_y = log(sum exp(z - zmax)) - (z_y - zmax)
      a.rowloss[r] = logf(ssum) - zy;
      a.rowidx[r] = (uint32_t)rows[k];
    }
  }
}

// Kernel 2: G = X^T dZ over all K*B stacked rows, sliced by feature, then the update
// w^{t+1} = w^t - G written into the next ring slot.  A workgroup owns 8 features; its
// 1024 threads are 8 features x 128 row groups; the 128 partial sums are combined through
// LDS in group order.  One more workgroup, the first, reduces the per-upload losses and the
// bias gradient.
constexpr int kUpdF = 8, kUpdG = 128;

template <int C>
__device__ __forceinline__ void softmax_update_body(const RegressionArgs& a, const RoundDesc& rd) {
  __shared__ float s_red[kUpdG][kUpdF * C + 1];
  __shared__ float s_loss[ABS_MAX_WORKERS];
  const int B = a.B, d = a.d, R = rd.K * B;
  const float* cur = a.ring + (size_t)rd.slot_cur * a.slot_stride;
  float* nxt = a.ring + (size_t)rd.slot_next * a.slot_stride;
  // workgroup 0 (the first to be dispatched) publishes the losses, so that the host prepares the
  // next round while the others still work; workgroups 1 .. are the feature slices
  const int slice = (int)blockIdx.x - 1;
  if (slice >= 0) {
    const int f = threadIdx.x % kUpdF, g = threadIdx.x / kUpdF;
    const int i = slice * kUpdF + f;
    float acc[C];
#pragma unroll
    for (int c = 0; c < C; ++c) acc[c] = 0.f;
    if (i < d) {
      // four rows per trip so that the dependent loads (row index -> x) of different rows overlap
      for (int r = g; r < R; r += 4 * kUpdG) {
        float x[4];
        float dzr[4][16];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int rr = r + u * kUpdG;
          const bool ok = rr < R;
          const int rs = ok ? rr : r;
          x[u] = ok ? a.X[(uint64_t)a.rowidx[rs] * (uint64_t)d + i] : 0.f;
          const float4* dzp = (const float4*)(a.dz + (size_t)rs * kDzPitch);
#pragma unroll
          for (int v = 0; v < (C + 3) / 4; ++v) {
            const float4 t = dzp[v];
            dzr[u][4 * v] = t.x; dzr[u][4 * v + 1] = t.y; dzr[u][4 * v + 2] = t.z; dzr[u][4 * v + 3] = t.w;
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int c = 0; c < C; ++c) acc[c] = fmaf(x[u], dzr[u][c], acc[c]);
      }
    }
#pragma unroll
    for (int c = 0; c < C; ++c) s_red[g][f * C + c] = acc[c];
    __syncthreads();
    if ((int)threadIdx.x < kUpdF * C) {
      const int ff = threadIdx.x / C, c = threadIdx.x % C;
      const int ii = slice * kUpdF + ff;
      if (ii < d) {
        float G = 0.f;
#pragma unroll 8
        for (int gg = 0; gg < kUpdG; ++gg) G += s_red[gg][threadIdx.x];
        nxt[(size_t)ii * C + c] = cur[(size_t)ii * C + c] - G;
      }
    }
    return;
  }
  // per-upload mean minibatch loss (the "average local loss" each worker uploads)
  {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int up = wave; up < rd.K; up += 16) {
      float s = 0.f;
      for (int b = lane; b < B; b += 64) s += a.rowloss[up * B + b];
      s = wave_sum(s);
      if (lane == 0) s_loss[up] = s / (float)B;
    }
    __syncthreads();
    publish_losses(a.mailbox, s_loss, rd.K, rd.stamp);
  }
  __syncthreads();
  // bias gradient: column sums of dZ (16 columns x 64 row groups), then b^{t+1}
  {
    const int c = threadIdx.x % 16, g = threadIdx.x / 16;
    float s = 0.f;
    for (int r = g; r < R; r += 64) s += a.dz[(size_t)r * kDzPitch + c];
    float* red = &s_red[0][0];
    red[g * 16 + c] = s;
    __syncthreads();
    if ((int)threadIdx.x < C) {
      float G = 0.f;
#pragma unroll
      for (int gg = 0; gg < 64; ++gg) G += red[gg * 16 + threadIdx.x];
      nxt[(size_t)d * C + threadIdx.x] = cur[(size_t)d * C + threadIdx.x] - G;
    }
  }
}

template <int C, int RPW>
__global__ __launch_bounds__(256) void softmax_rows_kernel(RegressionArgs a, RoundDesc rd) {
  softmax_rows_body<C, RPW>(a, rd);
}
template <int C>
__global__ __launch_bounds__(1024) void softmax_update_kernel(RegressionArgs a, RoundDesc rd) {
  softmax_update_body<C>(a, rd);
}
// Batched forms: blockIdx.y = simulation (see linreg_round_batch_kernel).
template <int C, int RPW>
__global__ __launch_bounds__(256) void softmax_rows_batch_kernel(const RegressionArgs* as, const char* rds,
                                                                 size_t stride) {
  const RegressionArgs a = as[blockIdx.y];
  softmax_rows_body<C, RPW>(a, *(const RoundDesc*)(rds + (size_t)blockIdx.y * stride));
}
template <int C>
__global__ __launch_bounds__(1024) void softmax_update_batch_kernel(const RegressionArgs* as, const char* rds,
                                                                    size_t stride) {
  const RegressionArgs a = as[blockIdx.y];
  softmax_update_body<C>(a, *(const RoundDesc*)(rds + (size_t)blockIdx.y * stride));
}

// ------------------------------------------------------------------ batched softmax rounds, fused
// With many simulations per launch there are enough uploads to give each a workgroup of its own,
// and then the round reads every minibatch row from HBM once.  Two forms.  This one, for wide models
// (d + 1 > 896): the upload's stale model sits in LDS, transposed ([class][feature]).  The other,
// further down and the usual one: the model sits in registers.  In both the rows pass through LDS
// in tiles (here TR = 8 or 16 rows), the next tile in flight in registers meanwhile, and both
// products of a tile run on the fp32 matrix cores (16x16x4 tiles, classes padded to 16):
//   (1) logits Z = X_tile W: the eight wavefronts split the features, their partial 16 x 16 tiles
//       are added through LDS, and 16 TR threads (row, class) finish softmax, loss and the rows of
//       dZ = c (softmax - onehot), with reductions over the 16 classes inside a DPP row;
//   (2) G += X_tile^T dZ: a wavefront owns blocks of 16 features, whose 16 x 16 gradient tiles
//       stay in its accumulators for the whole upload.
// The upload's gradient goes to a scratch slot; a second kernel adds the K^t slots in arrival
// order (Eq. 3) and writes w^{t+1} and the losses.
// LOCAL (U > 1 local steps per job, Eq. 2): the same stream of tiles runs over the job's U B rows;
// at the end of every step the gradient is applied to the model in LDS, which is the worker's
// private copy, and the upload is w^{t,0} - w^{t,U} with the mean of the local losses.
constexpr int kFuseThreads = 512, kFuseWaves = 8, kFuseMaxB = 1024, kFuseMaxLocalRows = 2048;
constexpr size_t kLdsPerCu = 160 * 1024;
constexpr int kWreg = 0;                  // in place of TR: 16-row tiles with the model in registers (below)
constexpr int kWregNB = 7;                // its blocks of 16 features per wavefront
constexpr int kWregMaxD = 16 * kWregNB * kFuseWaves - 4;     // d + 1 features in its blocks, d % 4 == 0
typedef float f32x4_ __attribute__((ext_vector_type(4)));
typedef float f32x2_ __attribute__((ext_vector_type(2)));
// loads known to be from global memory (a pointer read from memory is generic to the compiler)
template <class T>
__device__ __forceinline__ T load_global(const T* p) { return *(const __attribute__((address_space(1))) T*)p; }
__device__ __forceinline__ float4 load_global_f4(const float* p) {
  const f32x4_ v = *(const __attribute__((address_space(1))) f32x4_*)p;
  return make_float4(v.x, v.y, v.z, v.w);
}

// Reductions over the 16 lanes of a DPP row by four lane permutations (lane ^ 1, lane ^ 2, mirror
// of 8, mirror of 16); every lane ends with the result.  All lanes of the wavefront must be active.
template <int CTRL>
__device__ __forceinline__ float dpp_perm(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_perm<0xB1>(v);      // quad_perm [1,0,3,2]
  v += dpp_perm<0x4E>(v);      // quad_perm [2,3,0,1]
  v += dpp_perm<0x141>(v);     // row_half_mirror
  v += dpp_perm<0x140>(v);     // row_mirror
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_perm<0xB1>(v));
  v = fmaxf(v, dpp_perm<0x4E>(v));
  v = fmaxf(v, dpp_perm<0x141>(v));
  v = fmaxf(v, dpp_perm<0x140>(v));
  return v;
}

// Row pitch (floats) of the x tile and the model in LDS, chosen for the bank pattern of the matrix
// cores' operand reads (64 banks).  The logits product reads 16 bytes per lane from tile rows m16
// at 4 g4 floats: with 16 rows, a pitch of 4 modulo 64 gives every row its own four banks; with 8
// rows any pitch of 8 modulo 16 does.  The gradient product reads one float per lane, 16 features
// of four rows: those rows must be a multiple of 16 banks apart, which rows 2 g4 + j of an 8-row
// tile are at a pitch of 8 modulo 16.  (At least d + 1, so that the model's region can hold the
// gradient with its bias row at the end.)
__host__ __device__ inline int fuse_pitch(int d, int TR) { return TR == 16 ? d + 4 : d + (23 - d % 16) % 16 + 1; }
// dynamic LDS: x tile and model, partial logits, dZ, bias, then the upload's row indices and labels
static size_t fuse_lds_bytes(int d, int C, int rows, int TR) {
  if (TR == kWreg) return ((size_t)16 * (d + 4) + (kFuseWaves + 1) * 256 + 2 * (size_t)rows) * 4;   // no model, no bias
  return ((size_t)(TR + C) * fuse_pitch(d, TR) + (kFuseWaves + 1) * TR * 16 + 16 + 2 * (size_t)rows) * 4;
}

// TR rows per tile: 16 fills the matrix-core tile; 8 (half of the logits tile idle) when that lets
// two workgroups share a CU, so that one's set-up and tail overlap the other's streaming.  Measured
// on the 784 x 10 workload, 256 simulations: 389 us per round against 430 us with 16 rows and one
// workgroup; 12-row tiles (register spills) 459 us; logits of 8-row tiles on sixteen 4 x 4 x 1
// blocks instead of a half-idle 16 x 16 x 4 tile 424 us.
template <int C, int TR, bool LOCAL>
__device__ __forceinline__ void softmax_upload_body(const RegressionArgs& a, const RoundDesc& rd, int up) {
  constexpr int LD = TR / 2;              // 16-byte chunks per thread and tile (d <= 1024)
  constexpr int NB = 8;                   // blocks of 16 features per wavefront (d <= 1024)
  constexpr int RJ = TR / 4;              // groups of 4 rows per tile
  extern __shared__ __align__(16) float s_mem[];
  if (up >= rd.K) return;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int d = a.d, B = a.B, dq = d >> 2, dp = fuse_pitch(d, TR);
  const int total = LOCAL ? a.U * B : B;  // rows of the job: draw i of its counter stream is row i
  float* s_x = s_mem;                     // [TR][dp]
  float* s_Wt = s_x + TR * dp;            // [C][dp]; one step: at the end the upload's gradient, boundary layout
  float* s_zp = s_Wt + C * dp;            // [8 wavefronts][TR rows][16 classes]
  float* s_dz = s_zp + kFuseWaves * TR * 16;   // [TR][16]
  float* s_b = s_dz + TR * 16;            // [16]
  uint32_t* s_rowi = (uint32_t*)(s_b + 16);  // [total]
  int* s_lab = (int*)(s_rowi + total);       // [total]
  const WorkerDesc w = rd.w[up];
  const float* Wv = a.ring + (size_t)w.slot * a.slot_stride;

  // set-up, its loads all in flight together: the model (needs nothing), then - once the
  // minibatch draws are known - labels and the first tile
  const int nW4 = (d * C) >> 2;           // d % 4 == 0
  float4 wv[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) wv[u] = load_global_f4(Wv + 4 * min(t + u * kFuseThreads, nW4 - 1));
  const float bias = load_global(Wv + d * C + min(t, C - 1));
  for (int b = t; b < total; b += kFuseThreads)
    s_rowi[b] = (uint32_t)batch_row(w, a.batch_key, a.shard_rows, (uint32_t)b);
  __syncthreads();
  constexpr int NLAB = LOCAL ? kFuseMaxLocalRows / kFuseThreads : kFuseMaxB / kFuseThreads;
  int lab[NLAB];
#pragma unroll
  for (int u = 0; u < NLAB; ++u)
    lab[u] = load_global((const int32_t*)a.y + s_rowi[min(t + u * kFuseThreads, total - 1)]);
  // chunk t + 512 j of a tile is chunk pc[j] of tile row pr[j]
  int pr[LD], pc[LD];
  {
    const int sr = kFuseThreads / dq, sc = kFuseThreads - sr * dq;
    int r = t / dq, ch = t - r * dq;
#pragma unroll
    for (int j = 0; j < LD; ++j) {
      pr[j] = r; pc[j] = ch;
      ch += sc; r += sr;
      if (ch >= dq) { ch -= dq; r += 1; }
    }
  }
  // a tile's loads: row indices first, then all chunks (lanes past the tile's rows read the
  // dataset's first chunk, which costs a cache hit and no branch)
  float4 pre[LD];
#define ABS_PREFETCH(base_, nrows_)                                                                          \
  {                                                                                                          \
    uint32_t ri[LD];                                                                                         \
    _Pragma("unroll") for (int j = 0; j < LD; ++j) ri[j] = s_rowi[(base_) + min(pr[j], (nrows_) - 1)];       \
    _Pragma("unroll") for (int j = 0; j < LD; ++j) {                                                         \
      const uint64_t off = pr[j] < (nrows_) ? (uint64_t)ri[j] * (uint64_t)d + 4 * pc[j] : 0;                 \
      pre[j] = load_global_f4(a.X + off);                                                                    \
    }                                                                                                        \
  }
  ABS_PREFETCH(0, min(TR, B))
  // the model goes into LDS transposed
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int idx = 4 * (t + u * kFuseThreads);
    if (idx < 4 * nW4) {
      const float e[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int i = (idx + v) / C, c = (idx + v) - i * C;
        s_Wt[c * dp + i] = e[v];
      }
    }
  }
  for (int j = t + 4 * kFuseThreads; j < nW4; j += kFuseThreads) {     // d C > 8192 only
    const float4 x4 = load_global_f4(Wv + 4 * j);
    const float e[4] = {x4.x, x4.y, x4.z, x4.w};
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int i = (4 * j + v) / C, c = (4 * j + v) - i * C;
      s_Wt[c * dp + i] = e[v];
    }
  }
  if (t < 16) s_b[t] = t < C ? bias : 0.f;
#pragma unroll
  for (int u = 0; u < NLAB; ++u)
    if (t + u * kFuseThreads < total) s_lab[t + u * kFuseThreads] = lab[u];

  const int m16 = lane & 15, g4 = lane >> 4;      // the lane's row / column and k index inside a tile
  const int nstep = (d + 15) >> 4;                // steps of 16 features = blocks of 16 features
  f32x4_ G[NB];
#pragma unroll
  for (int bi = 0; bi < NB; ++bi) G[bi] = f32x4_{0.f, 0.f, 0.f, 0.f};
  float bacc = 0.f, loss = 0.f;
  // off: the tile's first row in the job's stream of rows; base: the same inside its step
  for (int off = 0, base = 0; off < total;) {
    const int nrows = min(TR, B - base);
    const int noff = off + nrows, nbase = base + nrows == B ? 0 : base + nrows;
    __syncthreads();                      // the previous tile has been used up
#pragma unroll
    for (int j = 0; j < LD; ++j)
      if (pr[j] < nrows) *(float4*)(s_x + pr[j] * dp + 4 * pc[j]) = pre[j];
    __syncthreads();
    if (noff < total) ABS_PREFETCH(noff, min(TR, B - nbase))
    // (1a) this wavefront's share of the logits: steps wave, wave + 8, ... of 16 features; lane
    // (m16, g4) feeds row m16 of x (mod TR) and class m16 of W at features 16 st + 4 g4 .. + 3
    {
      f32x4_ z = {0.f, 0.f, 0.f, 0.f};
      const float* xrow = s_x + (m16 & (TR - 1)) * dp;
      const float* wrow = s_Wt + min(m16, C - 1) * dp;
      for (int st = wave; st < nstep; st += kFuseWaves) {
        const int kk = 16 * st + 4 * g4;
        const bool ok = kk < d;
        const int kc = ok ? kk : 0;
        float4 av = *(const float4*)(xrow + kc);
        const float4 bv = *(const float4*)(wrow + kc);
        if (!ok) av = make_float4(0.f, 0.f, 0.f, 0.f);
        z = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv.x, z, 0, 0, 0);
        z = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, bv.y, z, 0, 0, 0);
        z = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, bv.z, z, 0, 0, 0);
        z = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, bv.w, z, 0, 0, 0);
      }
      // the lane holds rows 4 g4 .. 4 g4 + 3 of column m16
      if (4 * g4 < TR) {
        float* zp = s_zp + wave * (TR * 16) + (4 * g4) * 16 + m16;
        zp[0] = z[0]; zp[16] = z[1]; zp[32] = z[2]; zp[48] = z[3];
      }
    }
    __syncthreads();
    // (1b) thread (row t / 16, class t % 16): the logit, softmax over the DPP row, dZ, loss
    if (wave < TR / 4) {
      const int r = t >> 4, c = m16;
      float zz = s_b[c];
#pragma unroll
      for (int v = 0; v < kFuseWaves; ++v) zz += s_zp[v * (TR * 16) + t];
      if (c >= C) zz = -INFINITY;
      const float zmax = row16_max(zz);
      const float e = c < C ? expf(zz - zmax) : 0.f;
      const float ssum = row16_sum(e);
      const bool live = r < nrows;
      const int label = live ? s_lab[off + r] : -1;
      const float p = e / ssum;
      s_dz[t] = live && c < C ? w.c * (p - (c == label ? 1.f : 0.f)) : 0.f;
      if (c == label) loss += logf(ssum) - (zz - zmax);
    }
    __syncthreads();
    // (2) G += X_tile^T dZ: in step j lane (m16, g4) feeds feature f0 + m16 of tile row r(j, g4) and
    // dZ[r][m16]; which four rows a step takes is free: 4 j + g4 for 16-row tiles, 2 g4 + j for
    // 8-row tiles (bank pattern, see fuse_pitch)
    {
      const int r_g4 = TR == 16 ? g4 : RJ * g4, r_j = TR == 16 ? 4 : 1;
      float bq[RJ];
#pragma unroll
      for (int j = 0; j < RJ; ++j) bq[j] = s_dz[(r_g4 + r_j * j) * 16 + m16];
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        const int blk = wave + kFuseWaves * bi;
        if (blk < nstep) {
          const int f = min(16 * blk + m16, d - 1);
#pragma unroll
          for (int j = 0; j < RJ; ++j) {
            const int r = r_g4 + r_j * j;
            float xa = s_x[r * dp + f];
            if (r >= nrows) xa = 0.f;     // rows past the tile hold whatever the last tile left
            G[bi] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa, bq[j], G[bi], 0, 0, 0);
          }
        }
      }
      if (t < 16) {
#pragma unroll
        for (int r = 0; r < TR; ++r) bacc += s_dz[r * 16 + t];
      }
    }
    if (LOCAL && nbase == 0) {
      // end of a local step (Eq. 2): the step's gradient onto the private model; the lane holds
      // G[feature 16 blk + 4 g4 + i][class m16].  The next tile's barriers order this before
      // anybody reads the model again.
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        const int blk = wave + kFuseWaves * bi, f0 = 16 * blk + 4 * g4;
        if (f0 < d && m16 < C) {          // d % 4 == 0: all four features or none
          float4* q = (float4*)(s_Wt + m16 * dp + f0);
          float4 v = *q;
          v.x -= G[bi][0]; v.y -= G[bi][1]; v.z -= G[bi][2]; v.w -= G[bi][3];
          *q = v;
        }
        G[bi] = f32x4_{0.f, 0.f, 0.f, 0.f};
      }
      if (t < 16) { s_b[t] -= bacc; bacc = 0.f; }
    }
    off = noff; base = nbase;
  }
#undef ABS_PREFETCH
  // losses sit in the lanes whose class is the row's label: add them up
  loss = row16_sum(loss);
  __syncthreads();
  if (wave < TR / 4 && m16 == 0) s_zp[t >> 4] = loss;      // TR row sums (s_zp is free now)
  float* part = a.delta + (size_t)up * a.slot_stride;
  if (LOCAL) {
    // the upload: what the U steps changed, w^{t,0} - w^{t,U}, and the mean of the local losses
    __syncthreads();
    const int P = (d + 1) * C;
    for (int idx = t; idx < P; idx += kFuseThreads) {
      const int i = idx / C, c = idx - i * C;
      const float now = i < d ? s_Wt[c * dp + i] : s_b[c];
      part[idx] = load_global(Wv + idx) - now;
    }
    if (t == 0) {
      float l = 0.f;
#pragma unroll
      for (int v = 0; v < TR; ++v) l += s_zp[v];
      a.lossbuf[up] = l / (float)total;
    }
    return;
  }
  // the gradient, staged through LDS in the boundary layout for full-width stores; the lane holds
  // G[feature 16 blk + 4 g4 + i][class m16]
  float* s_G = s_Wt;
#pragma unroll
  for (int bi = 0; bi < NB; ++bi) {
    const int blk = wave + kFuseWaves * bi;
    if (blk < nstep && m16 < C) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int f = 16 * blk + 4 * g4 + i;
        if (f < d) s_G[f * C + m16] = G[bi][i];
      }
    }
  }
  if (t < C) s_G[d * C + t] = bacc;
  __syncthreads();
  for (int j = t; j < nW4; j += kFuseThreads) {
    const float4 g = ((const float4*)s_G)[j];
    *(__attribute__((address_space(1))) f32x4_*)(part + 4 * j) = f32x4_{g.x, g.y, g.z, g.w};
  }
  if (t < C) part[(size_t)d * C + t] = s_G[d * C + t];
  if (t == 0) {
    float l = 0.f;
#pragma unroll
    for (int v = 0; v < TR; ++v) l += s_zp[v];
    a.lossbuf[up] = l / (float)B;
  }
}

// The same round with the model in registers instead of LDS, for d + 1 <= 896: the split of the
// logits product over the wavefronts is static (wavefront w always takes the blocks of 16 features
// w, w + 8, ...), so lane (m16, g4) only ever needs W[16 blk + 4 g4 + v][class m16] of its own
// blocks - exactly the elements of the gradient it accumulates.  Without the model, a full
// 16-row tile (no idle half in the logits product) and two workgroups fit a CU's LDS; a local
// step (Eq. 2) is a subtraction between two sets of registers.
// The bias is feature d of x~ = [x, 1]: the model's slot holds it right behind W, and the tile's
// pad column holds the 1, so both products and the local step cover it without extra code.
// The x tile has pitch d + 4: the 16 rows start 4 banks apart, and rows 4 g4 + j of the gradient
// product 16 banks apart.
template <int C, bool LOCAL>
__device__ __forceinline__ void softmax_upload_wreg_body(const RegressionArgs& a, const RoundDesc& rd, int up) {
  constexpr int TR = 16, NB = kWregNB;
  extern __shared__ __align__(16) float s_mem[];
  if (up >= rd.K) return;
  const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int d = a.d, B = a.B, dp = d + 4;
  const int total = LOCAL ? a.U * B : B;  // rows of the job: draw i of its counter stream is row i
  float* s_x = s_mem;                     // [16][dp]; first the model, at the end the upload, boundary layout
  float* s_zp = s_x + TR * dp;            // [8 wavefronts][16 rows][16 classes]
  float* s_dz = s_zp + kFuseWaves * 256;  // [16][16]
  uint32_t* s_rowi = (uint32_t*)(s_dz + 256);  // [total]
  int* s_lab = (int*)(s_rowi + total);         // [total]
  const WorkerDesc w = rd.w[up];
  const float* Wv = a.ring + (size_t)w.slot * a.slot_stride;
  const int m16 = lane & 15, g4 = lane >> 4;      // the lane's row / column and k index inside a tile
  const int P = (d + 1) * C, nP4 = P >> 2;        // the model with its bias row: (d + 1) x C

  // set-up: the model is asked for first and has arrived by the time the minibatch draws are
  // known; it passes through the tile's place in LDS (boundary layout) into the lanes' registers
  // while the labels and the first tile are on their way
  float4 wv[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) wv[u] = load_global_f4(Wv + 4 * min(t + u * kFuseThreads, nP4 - 1));
  const float wtail = load_global(Wv + min(4 * nP4 + t, P - 1));
  for (int b = t; b < total; b += kFuseThreads)
    s_rowi[b] = (uint32_t)batch_row(w, a.batch_key, a.shard_rows, (uint32_t)b);
  __syncthreads();
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (t + u * kFuseThreads < nP4) ((float4*)s_x)[t + u * kFuseThreads] = wv[u];
  for (int j = t + 4 * kFuseThreads; j < nP4; j += kFuseThreads) ((float4*)s_x)[j] = load_global_f4(Wv + 4 * j);
  if (4 * nP4 + t < P) s_x[4 * nP4 + t] = wtail;
  constexpr int NLAB = LOCAL ? kFuseMaxLocalRows / kFuseThreads : kFuseMaxB / kFuseThreads;
  int lab[NLAB];
#pragma unroll
  for (int u = 0; u < NLAB; ++u)
    lab[u] = load_global((const int32_t*)a.y + s_rowi[min(t + u * kFuseThreads, total - 1)]);
  // A wavefront loads, stores and reads only the feature columns of its own blocks (both products
  // of wavefront w touch features 16 blk .. + 15 of blk = w, w + 8, ... and nothing else), so the
  // tile in LDS needs no workgroup barrier: lane l takes the 16 bytes at chunk l % 4 of the block's
  // 64 bytes in tile row l / 4 (lanes past the tile's rows read its last row again)
  const int prow = lane >> 2, pch = lane & 3;
  float4 pre[NB];
#define ABS_PREFETCH(base_, nrows_)                                                                          \
  {                                                                                                          \
    const uint32_t ri = s_rowi[(base_) + min(prow, (nrows_) - 1)];                                           \
    const float* src = a.X + (uint64_t)ri * (uint64_t)d + 16 * wave + 4 * pch;                               \
    _Pragma("unroll") for (int bi = 0; bi < NB; ++bi)                                                        \
      if (16 * (wave + kFuseWaves * bi) + 4 * pch < d) pre[bi] = load_global_f4(src + 128 * bi);             \
  }
  ABS_PREFETCH(0, min(TR, B))
  __syncthreads();
  f32x4_ wreg[NB];
#pragma unroll
  for (int bi = 0; bi < NB; ++bi) {
    const int f0 = 16 * (wave + kFuseWaves * bi) + 4 * g4;
#pragma unroll
    for (int v = 0; v < 4; ++v) {         // d % 4 == 0: of the bias row's four only the first exists
      const bool ok = m16 < C && (f0 < d || (f0 == d && v == 0));
      const float x = s_x[ok ? (f0 + v) * C + m16 : 0];
      wreg[bi][v] = ok ? x : 0.f;
    }
  }
  __syncthreads();
  if (t < TR) *(float4*)(s_x + t * dp + d) = make_float4(1.f, 0.f, 0.f, 0.f);   // the 1 of x~; tiles never write here
#pragma unroll
  for (int u = 0; u < NLAB; ++u)
    if (t + u * kFuseThreads < total) s_lab[t + u * kFuseThreads] = lab[u];
  __syncthreads();

  f32x4_ G[NB];
#pragma unroll
  for (int bi = 0; bi < NB; ++bi) G[bi] = f32x4_{0.f, 0.f, 0.f, 0.f};
  float loss = 0.f;
  // off: the tile's first row in the job's stream of rows; base: the same inside its step
  for (int off = 0, base = 0; off < total;) {
    const int nrows = min(TR, B - base);
    const int noff = off + nrows, nbase = base + nrows == B ? 0 : base + nrows;
    // the tile's columns of this wavefront into LDS (its own gradient product of the previous tile
    // was their last reader), then the next tile's loads
    {
      float* xdst = s_x + prow * dp + 16 * wave + 4 * pch;
#pragma unroll
      for (int bi = 0; bi < NB; ++bi)
        if (16 * (wave + kFuseWaves * bi) + 4 * pch < d) *(float4*)(xdst + 128 * bi) = pre[bi];
    }
    // other lanes of this wavefront read what this lane wrote: LDS serves a wavefront's requests in
    // order, the compiler must keep them in order too
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (noff < total) ABS_PREFETCH(noff, min(TR, B - nbase))
    // (1a) this wavefront's share of the logits: lane (m16, g4) feeds row m16 of x~ and its own
    // model elements (class m16) at features 16 blk + 4 g4 .. + 3; two accumulators in turn
    {
      f32x4_ z0 = {0.f, 0.f, 0.f, 0.f}, z1 = {0.f, 0.f, 0.f, 0.f};
      const float* xrow = s_x + m16 * dp;
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        const int kk = 16 * (wave + kFuseWaves * bi) + 4 * g4;
        // no branch but around the last block: a block past d multiplies zeros
        if (bi < NB - 1 || 16 * (wave + kFuseWaves * bi) <= d) {
          float4 av = *(const float4*)(xrow + kk);     // past d + 3: the next row, allocated LDS
          if (kk > d) av = make_float4(0.f, 0.f, 0.f, 0.f);
          f32x4_& z = (bi & 1) ? z1 : z0;
          z = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, wreg[bi][0], z, 0, 0, 0);
          z = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, wreg[bi][1], z, 0, 0, 0);
          z = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, wreg[bi][2], z, 0, 0, 0);
          z = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, wreg[bi][3], z, 0, 0, 0);
        }
      }
      // the lane holds rows 4 g4 .. 4 g4 + 3 of column m16
      float* zp = s_zp + wave * 256 + (4 * g4) * 16 + m16;
      zp[0] = z0[0] + z1[0]; zp[16] = z0[1] + z1[1]; zp[32] = z0[2] + z1[2]; zp[48] = z0[3] + z1[3];
    }
    // the row's label, fetched ahead of the barrier (thread (row t / 16, class t % 16) of (1b))
    const int label = wave < TR / 4 && (t >> 4) < nrows ? s_lab[off + (t >> 4)] : -1;
    __syncthreads();
    // (1b) thread (row t / 16, class t % 16): the logit, softmax over the DPP row, dZ, loss
    if (wave < TR / 4) {
      const int c = m16;
      // the eight partial logits, all requests in flight before the first addition (the compiler
      // would wait for each pair in turn)
      static_assert(kFuseWaves == 8, "eight partial tiles");
      f32x2_ q0, q1, q2, q3;
      asm volatile(
          "ds_read2st64_b32 %0, %4 offset1:4\n\t"
          "ds_read2st64_b32 %1, %4 offset0:8 offset1:12\n\t"
          "ds_read2st64_b32 %2, %4 offset0:16 offset1:20\n\t"
          "ds_read2st64_b32 %3, %4 offset0:24 offset1:28\n\t"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(q0), "=&v"(q1), "=&v"(q2), "=&v"(q3)
          : "v"((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(s_zp + t))
          : "memory");
      float zz = ((((((q0.x + q0.y) + q1.x) + q1.y) + q2.x) + q2.y) + q3.x) + q3.y;
      if (c >= C) zz = -INFINITY;
      const float zmax = row16_max(zz);
      const float e = c < C ? expf(zz - zmax) : 0.f;
      const float ssum = row16_sum(e);
      const float p = e / ssum;
      s_dz[t] = (t >> 4) < nrows && c < C ? w.c * (p - (c == label ? 1.f : 0.f)) : 0.f;
      if (c == label) loss += logf(ssum) - (zz - zmax);
    }
    __syncthreads();
    // (2) G += X~_tile^T dZ: in step j lane (m16, g4) feeds feature f0 + m16 of tile row 4 g4 + j
    // and dZ[4 g4 + j][m16].  Features past d + 3 read on into allocated LDS (at most 16 NB 8 floats
    // past a row's start, less than what follows the tile); their gradient elements are never used.
    {
      float bq[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) bq[j] = s_dz[(4 * g4 + j) * 16 + m16];
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        const int blk = wave + kFuseWaves * bi;
        if (bi < NB - 1 || 16 * blk <= d) {
          const int f = 16 * blk + m16;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int r = 4 * g4 + j;
            float xa = s_x[r * dp + f];
            if (r >= nrows) xa = 0.f;     // rows past the tile hold whatever the last tile left
            G[bi] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa, bq[j], G[bi], 0, 0, 0);
          }
        }
      }
    }
    if (LOCAL && nbase == 0) {
      // end of a local step (Eq. 2): the step's gradient onto the private model; G[bi][i] and
      // wreg[bi][i] are the same element (feature 16 blk + 4 g4 + i, class m16)
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        if (16 * (wave + kFuseWaves * bi) + 4 * g4 <= d) {
#pragma unroll
          for (int i = 0; i < 4; ++i) wreg[bi][i] -= G[bi][i];
        }
        G[bi] = f32x4_{0.f, 0.f, 0.f, 0.f};
      }
    }
    off = noff; base = nbase;
  }
#undef ABS_PREFETCH
  // losses sit in the lanes whose class is the row's label: add them up
  loss = row16_sum(loss);
  __syncthreads();
  if (wave < TR / 4 && m16 == 0) s_zp[t >> 4] = loss;      // TR row sums (s_zp is free now)
  // the upload, staged through LDS in the boundary layout for full-width accesses: the gradient,
  // or (local steps) the model after the U steps
  float* s_G = s_x;
#pragma unroll
  for (int bi = 0; bi < NB; ++bi) {
    const int f0 = 16 * (wave + kFuseWaves * bi) + 4 * g4;
    if (m16 < C) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (f0 < d || (f0 == d && i == 0)) s_G[(f0 + i) * C + m16] = LOCAL ? wreg[bi][i] : G[bi][i];
    }
  }
  __syncthreads();
  float* part = a.delta + (size_t)up * a.slot_stride;
  for (int j = t; j < nP4; j += kFuseThreads) {
    float4 g = ((const float4*)s_G)[j];
    if (LOCAL) {                          // what the U steps changed: w^{t,0} - w^{t,U}
      const float4 w0 = load_global_f4(Wv + 4 * j);
      g = make_float4(w0.x - g.x, w0.y - g.y, w0.z - g.z, w0.w - g.w);
    }
    *(__attribute__((address_space(1))) f32x4_*)(part + 4 * j) = f32x4_{g.x, g.y, g.z, g.w};
  }
  if (4 * nP4 + t < P) part[4 * nP4 + t] = LOCAL ? wtail - s_G[4 * nP4 + t] : s_G[4 * nP4 + t];
  if (t == 0) {
    float l = 0.f;
#pragma unroll
    for (int v = 0; v < TR; ++v) l += s_zp[v];
    a.lossbuf[up] = l / (float)total;
  }
}

// TR == kWreg selects the form with the model in registers
template <int C, int TR, bool LOCAL>
__device__ __forceinline__ void softmax_upload_any(const RegressionArgs& a, const RoundDesc& rd, int up) {
  if constexpr (TR == kWreg) softmax_upload_wreg_body<C, LOCAL>(a, rd, up);
  else softmax_upload_body<C, TR, LOCAL>(a, rd, up);
}

template <int C, int TR>
__global__ __launch_bounds__(kFuseThreads, TR == 16 ? 2 : 4) void softmax_upload_batch_kernel(
    const RegressionArgs* as, const char* rds, size_t stride) {
  const RegressionArgs a = as[blockIdx.y];
  softmax_upload_any<C, TR, false>(a, *(const RoundDesc*)(rds + (size_t)blockIdx.y * stride), blockIdx.x);
}
template <int C, int TR>
__global__ __launch_bounds__(kFuseThreads, TR == 16 ? 2 : 4) void softmax_local_fused_kernel(RegressionArgs a, RoundDesc rd) {
  softmax_upload_any<C, TR, true>(a, rd, blockIdx.x);
}
template <int C, int TR>
__global__ __launch_bounds__(kFuseThreads, TR == 16 ? 2 : 4) void softmax_local_fused_batch_kernel(
    const RegressionArgs* as, const char* rds, size_t stride) {
  const RegressionArgs a = as[blockIdx.y];
  softmax_upload_any<C, TR, true>(a, *(const RoundDesc*)(rds + (size_t)blockIdx.y * stride), blockIdx.x);
}

// Eq. 3 over the uploads' gradients (each already scaled by its c), arrival order
__global__ __launch_bounds__(256) void softmax_combine_batch_kernel(const RegressionArgs* as, const char* rds,
                                                                    size_t stride, int P) {
  __shared__ float s_loss[ABS_MAX_WORKERS];
  const RegressionArgs a = as[blockIdx.y];
  const RoundDesc& rd = *(const RoundDesc*)(rds + (size_t)blockIdx.y * stride);
  const int K = rd.K;
  const float* cur = a.ring + (size_t)rd.slot_cur * a.slot_stride;
  float* nxt = a.ring + (size_t)rd.slot_next * a.slot_stride;
  if (blockIdx.x == 0) {                  // first: the host prepares the next round meanwhile
    for (int up = threadIdx.x; up < K; up += 256) s_loss[up] = a.lossbuf[up];
    __syncthreads();
    publish_losses(a.mailbox, s_loss, K, rd.stamp);
  }
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < P) {
    const float c = load_global(cur + i);
    const float* p = a.delta + i;
    float sum = 0.f;
    int up = 0;
    for (; up + 8 <= K; up += 8) {        // eight loads in flight, added in arrival order
      float g[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) g[u] = load_global(p + (size_t)(up + u) * a.slot_stride);
#pragma unroll
      for (int u = 0; u < 8; ++u) sum += g[u];
    }
    for (; up < K; ++up) sum += load_global(p + (size_t)up * a.slot_stride);
    nxt[i] = c - sum;
  }
}

template <int C, int TR>
static hipError_t launch_softmax_fused_batch(const RegressionArgs* d_args, const char* d_rds, size_t stride, int S,
                                             int d, int B, int Kmax, hipStream_t s) {
  // dynamic LDS the kernel has been cleared for (one device per process; batches may be advanced
  // from several host threads, so the high-water mark is atomic and the call is idempotent)
  static std::atomic<size_t> allowed{0};
  const size_t lds = fuse_lds_bytes(d, C, B, TR);
  if (lds > allowed.load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute((const void*)softmax_upload_batch_kernel<C, TR>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    size_t seen = allowed.load(std::memory_order_relaxed);
    while (seen < lds && !allowed.compare_exchange_weak(seen, lds, std::memory_order_release)) {}
  }
  softmax_upload_batch_kernel<C, TR><<<dim3(Kmax, S), dim3(kFuseThreads), lds, s>>>(d_args, d_rds, stride);
  const int P = (d + 1) * C;
  softmax_combine_batch_kernel<<<dim3((P + 255) / 256, S), dim3(256), 0, s>>>(d_args, d_rds, stride, P);
  return hipGetLastError();
}

// The local steps of the uploads of one simulation (d_args == nullptr: arguments by value) or of S
// simulations; the caller adds the uploads' changes afterwards (Eq. 3).
template <int C, int TR>
static hipError_t launch_softmax_local_fused_c(const RegressionArgs* a1, const RoundDesc* rd1, const RegressionArgs* d_args,
                                               const char* d_rds, size_t stride, int S, int d, int rows, int Kmax,
                                               hipStream_t s) {
  static std::atomic<size_t> allowed1{0}, allowedS{0};
  const size_t lds = fuse_lds_bytes(d, C, rows, TR);
  const bool single = d_args == nullptr;
  std::atomic<size_t>& allowed = single ? allowed1 : allowedS;
  if (lds > allowed.load(std::memory_order_acquire)) {
    const hipError_t e = single ? hipFuncSetAttribute((const void*)softmax_local_fused_kernel<C, TR>,
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                                : hipFuncSetAttribute((const void*)softmax_local_fused_batch_kernel<C, TR>,
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    size_t seen = allowed.load(std::memory_order_relaxed);
    while (seen < lds && !allowed.compare_exchange_weak(seen, lds, std::memory_order_release)) {}
  }
  if (single) softmax_local_fused_kernel<C, TR><<<dim3(Kmax), dim3(kFuseThreads), lds, s>>>(*a1, *rd1);
  else        softmax_local_fused_batch_kernel<C, TR><<<dim3(Kmax, S), dim3(kFuseThreads), lds, s>>>(d_args, d_rds, stride);
  return hipGetLastError();
}

// Which form of the fused kernel: the model in registers where d allows it and two workgroups fit a
// CU; else 8-row tiles if that makes two workgroups fit; else 16-row tiles, one workgroup.
static int fuse_form(int d, int C, int rows) {
  if (d <= kWregMaxD && 2 * fuse_lds_bytes(d, C, rows, kWreg) <= kLdsPerCu) return kWreg;
  return 2 * fuse_lds_bytes(d, C, rows, 8) <= kLdsPerCu ? 8 : 16;
}

bool softmax_local_fused_ok(int B, int U) { return B <= kFuseMaxB && (long)B * U <= kFuseMaxLocalRows; }

hipError_t launch_softmax_local_fused(const RegressionArgs* a1, const RoundDesc* rd1, const RegressionArgs* d_args,
                                      const char* d_rds, size_t stride, int S, int d, int C, int B, int U, int Kmax,
                                      hipStream_t s) {
  const int rows = B * U;
  const int form = fuse_form(d, C, rows);
  switch (C) {
#define ABS_CASE(c)                                                                                              \
  case c:                                                                                                        \
    return form == kWreg ? launch_softmax_local_fused_c<c, kWreg>(a1, rd1, d_args, d_rds, stride, S, d, rows, Kmax, s) \
           : form == 8   ? launch_softmax_local_fused_c<c, 8>(a1, rd1, d_args, d_rds, stride, S, d, rows, Kmax, s)     \
                         : launch_softmax_local_fused_c<c, 16>(a1, rd1, d_args, d_rds, stride, S, d, rows, Kmax, s);
    ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8) ABS_CASE(9)
    ABS_CASE(10) ABS_CASE(11) ABS_CASE(12) ABS_CASE(13) ABS_CASE(14) ABS_CASE(15) ABS_CASE(16)
#undef ABS_CASE
    default: return hipErrorInvalidValue;
  }
}

template <int C>
static hipError_t softmax_round_c(const RegressionArgs& a, const RoundDesc& rd, hipStream_t s,
                                  LaunchHook* hook) {
  const int R = rd.K * a.B;
  const double rows = (double)R;
  hook->begin(KK_SOFTMAX_ROWS, rows * a.d * C * 2.0, rows * (a.d + 1) * 4.0);
  if (R >= kRowsToSpare) softmax_rows_kernel<C, 4><<<dim3(rd.K * ((a.B + 15) / 16)), dim3(256), 0, s>>>(a, rd);
  else                   softmax_rows_kernel<C, 1><<<dim3(rd.K * ((a.B + 3) / 4)), dim3(256), 0, s>>>(a, rd);
  hook->end(KK_SOFTMAX_ROWS);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int nslice = (a.d + kUpdF - 1) / kUpdF;
  hook->begin(KK_SOFTMAX_UPDATE, rows * a.d * C * 2.0, 2.0 * (a.d + 1) * C * 4.0);
  softmax_update_kernel<C><<<dim3(nslice + 1), dim3(1024), 0, s>>>(a, rd);
  hook->end(KK_SOFTMAX_UPDATE);
  return hipGetLastError();
}

hipError_t launch_softmax_round(const RegressionArgs& a, const RoundDesc& rd, hipStream_t s,
                                LaunchHook* hook) {
  switch (a.C) {
#define ABS_CASE(c) case c: return softmax_round_c<c>(a, rd, s, hook);
    ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8) ABS_CASE(9)
    ABS_CASE(10) ABS_CASE(11) ABS_CASE(12) ABS_CASE(13) ABS_CASE(14) ABS_CASE(15) ABS_CASE(16)
#undef ABS_CASE
    default: return hipErrorInvalidValue;
  }
}

bool regression_batch_uses_slots(bool softmax, int B) { return softmax && B <= kFuseMaxB; }

// One round of S simulations of the same shape (model, d, C, B) in one set of launches.
hipError_t launch_regression_round_batch(const RegressionArgs* d_args, const char* d_rds, size_t stride, int S,
                                         bool softmax, int d, int C, int B, int Kmax, bool slots, hipStream_t s) {
  if (!softmax) {
    const dim3 grid(1, S), block(kLinWaves * 64);
    if (d <= 128)       linreg_round_batch_kernel<2><<<grid, block, 0, s>>>(d_args, d_rds, stride);
    else if (d <= 256)  linreg_round_batch_kernel<4><<<grid, block, 0, s>>>(d_args, d_rds, stride);
    else                linreg_round_batch_kernel<8><<<grid, block, 0, s>>>(d_args, d_rds, stride);
    return hipGetLastError();
  }
  if (slots && regression_batch_uses_slots(softmax, B)) {
    const int form = fuse_form(d, C, B);
    switch (C) {
#define ABS_CASE(c)                                                                                          \
  case c:                                                                                                    \
    return form == kWreg ? launch_softmax_fused_batch<c, kWreg>(d_args, d_rds, stride, S, d, B, Kmax, s)     \
           : form == 8   ? launch_softmax_fused_batch<c, 8>(d_args, d_rds, stride, S, d, B, Kmax, s)         \
                         : launch_softmax_fused_batch<c, 16>(d_args, d_rds, stride, S, d, B, Kmax, s);
      ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8) ABS_CASE(9)
      ABS_CASE(10) ABS_CASE(11) ABS_CASE(12) ABS_CASE(13) ABS_CASE(14) ABS_CASE(15) ABS_CASE(16)
#undef ABS_CASE
      default: return hipErrorInvalidValue;
    }
  }
  const int nslice = (d + kUpdF - 1) / kUpdF;
  switch (C) {
#define ABS_CASE(c)                                                                                          \
  case c:                                                                                                    \
    if ((long)S * Kmax * B >= kRowsToSpare)                                                                  \
      softmax_rows_batch_kernel<c, 4><<<dim3(Kmax * ((B + 15) / 16), S), dim3(256), 0, s>>>(d_args, d_rds, stride); \
    else                                                                                                     \
      softmax_rows_batch_kernel<c, 1><<<dim3(Kmax * ((B + 3) / 4), S), dim3(256), 0, s>>>(d_args, d_rds, stride);  \
    softmax_update_batch_kernel<c><<<dim3(nslice + 1, S), dim3(1024), 0, s>>>(d_args, d_rds, stride);        \
    break;
    ABS_CASE(2) ABS_CASE(3) ABS_CASE(4) ABS_CASE(5) ABS_CASE(6) ABS_CASE(7) ABS_CASE(8) ABS_CASE(9)
    ABS_CASE(10) ABS_CASE(11) ABS_CASE(12) ABS_CASE(13) ABS_CASE(14) ABS_CASE(15) ABS_CASE(16)
#undef ABS_CASE
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace abs_impl
