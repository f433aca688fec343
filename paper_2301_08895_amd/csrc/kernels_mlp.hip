// MLP rounds: bf16 operands on the matrix cores (MFMA 16x16x32 in the large-tile kernel, 32x32x16
// in the others), fp32 accumulation,
// fp32 master weights.
//
// The K^t uploads of a round are stacked into one batch of K^t * Bp rows (Bp = B padded
// to the 128-row tile, so a row tile never straddles two uploads).  Forward and
// input-gradient products are grouped GEMMs: each 128-row tile multiplies with the bf16
// copy of the model version its upload computed at (Eq. 2 at the stale model
// w^{t - tau_k}).  The weight gradient and the K-of-N reduction of Eq. 3 are ONE
// contraction over all stacked rows, G_l = H_{l-1}^T dZ_l: rows of dZ already carry their
// upload's coefficient c_k = eta_k / (K^t B), so per-upload gradients are never
// materialised.  The contraction is split along the rows into partial sums that are
// combined in a fixed order by the update kernel, which also writes w^{t+1} = w^t - G
// into the next ring slot together with its two bf16 copies.
//
// All three products have the form  C[m][n] = sum_k A[m][k] * Bt[n][k]  with both
// operands contiguous along k, so one main loop serves them:
//   forward    A = H_{l}      [rows][dp_l]      Bt = W_l^T  [dp_{l+1}][dp_l]   (per upload)
//   dgrad      A = dZ_{l+1}   [rows][dp_{l+1}]  Bt = W_l    [dp_l][dp_{l+1}]   (per upload)
//   wgrad      A = H_l^T      [dp_l][rows]      Bt = dZ_{l+1}^T [dp_{l+1}][rows]
// which is why activations and output gradients are stored in both orientations and
// the weights' bf16 copies in both orientations.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <string>

#include "kernels.h"

namespace abs_impl {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int TM = 128;   // rows of C per workgroup
constexpr int BK = 64;    // contraction elements per main-loop step
constexpr int kMaxSplit = 16;
// Row pitches of the bf16 operand arrays are the padded width plus this many elements (128 B):
// with a pitch that is a multiple of 4 KB the same 128-byte column of every row of a tile maps
// to one L2 channel, and all workgroups walk the k dimension in step.
#ifndef ABS_PITCH_PAD
#define ABS_PITCH_PAD 64
#endif
constexpr int kPitchPad = ABS_PITCH_PAD;
constexpr int kPartialPad = 32;         // the same for the fp32 weight-gradient partials (floats)

size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  // round to nearest, ties to even (finite values)
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// 16-byte store that, on request, does not keep its line in the cache.  The activations and
// gradients of a large round are hundreds of megabytes that another kernel reads next; kept out of
// the L2 they no longer evict the operand panels the other workgroups of the XCD still share
// (a 32768 x 2048 x 2048 forward product 250 -> 230 us).  A small round's outputs fit the caches and
// are better left there for their reader (8192 rows: the products that follow got 4 % slower).
#ifndef ABS_STREAM_MIN_BYTES
#define ABS_STREAM_MIN_BYTES (64u << 20)
#endif
__device__ __forceinline__ void store16_stream(uint16_t* p, const uint4& v, bool stream) {
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  // (written out by hand: when both forms of the store sit in the two arms of a branch the optimiser
  // merges them into one plain store)
  if (stream) asm volatile("global_store_dwordx4 %0, %1, off nt" : : "v"(p), "v"(u32x4_t{v.x, v.y, v.z, v.w}) : "memory");
  else        *(uint4*)p = v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// ------------------------------------------------------------------ gather + transpose of X
// XgT[k][m] = X[rowidx[m]][k]  (zero for k >= d0): the A operand of the first layer's
// weight-gradient contraction.  64 x 64 tiles through LDS.
__global__ __launch_bounds__(256) void mlp_gather_t_kernel(const uint16_t* X, int d0, const uint32_t* rowidx,
                                                          uint16_t* XgT, size_t ldt) {
  __shared__ uint16_t tile[64][72];
  const int m0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = t + 256 * i;
    const int r = q >> 3, c = q & 7;
    const int k = k0 + c * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (k < d0) v = *(const uint4*)(X + (size_t)rowidx[m0 + r] * d0 + k);
    *(uint4*)&tile[r][c * 8] = v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = t + 256 * i;
    const int kk = q >> 3, c = q & 7;      // output row kk, 8 consecutive m
    uint16_t v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = tile[c * 8 + j][kk];
    uint4 o;
    o.x = v[0] | ((uint32_t)v[1] << 16); o.y = v[2] | ((uint32_t)v[3] << 16);
    o.z = v[4] | ((uint32_t)v[5] << 16); o.w = v[6] | ((uint32_t)v[7] << 16);
    *(uint4*)(XgT + (size_t)(k0 + kk) * ldt + m0 + c * 8) = o;
  }
}

// ------------------------------------------------------------------ Eq. 3 on a block of a weight matrix
// w^{t+1} = w^t - sum_z partial[z] (fixed order) for one weight matrix, written as fp32 into the next
// ring slot and as bf16 in both orientations into the next shadow slot.
struct TileUpdate {
  const float* partial; size_t split_stride; size_t ldp; int nsplit;
  const float* w_cur; float* w_next;   // [d_in][d_out] fp32, pitch d_out
  int d_in, d_out;
  uint16_t* wn; size_t ldwn;           // bf16 [dp_in][dp_out] (may be null)
  uint16_t* wt; size_t ldwt;           // bf16 [dp_out][dp_in]
  // sk_q > 0: the partials come from a weight-gradient launch that cut the contraction into equal
  // runs of sk_q k-steps across the 256 x 256 output tiles (see GemmArgs::sk_q); tile T then has as
  // many partials as runs touch its sk_ksteps k-steps, in slots 0 .. count - 1.
  int sk_q, sk_ksteps, sk_nt;
};
__device__ __forceinline__ int partial_count(const TileUpdate& u, int i0, int j0) {
  if (!u.sk_q) return u.nsplit;
  const int tile = (i0 >> 8) * u.sk_nt + (j0 >> 8);
  return ((tile + 1) * u.sk_ksteps - 1) / u.sk_q - tile * u.sk_ksteps / u.sk_q + 1;
}
// Tiled version for 16-byte aligned rows (d_out % 4 == 0).  One block of 64 rows x TJ columns at
// (i0, j0), by all NT threads of the workgroup (uniform call): a thread moves 4 consecutive columns at
// a time, TJ / 4 threads cover a row (TJ = 256: 1 KB of a model row per row of the tile, so that the
// rows of a tile - a whole number of 4 KB apart for the usual widths - do not all fall on one memory
// channel).  `tile` is 64 x (TJ + 2) bf16 of LDS: with a row pitch of 129 / 33 words the transposed
// copy's 8 blocks of 8 rows start 8 banks apart and no two lanes of a wavefront collide.
template <int NT, int TJ>
__device__ __forceinline__ void update_block64(const TileUpdate& u, int i0, int j0, uint16_t* tile) {
  constexpr int TPR = TJ / 4;            // threads per row
  constexpr int RPP = NT / TPR;          // rows per pass
  constexpr int NPASS = 64 / RPP;        // passes
  constexpr int PT = TJ + 2;             // pitch of the LDS tile
  static_assert(NPASS >= 2 && NPASS % 2 == 0, "two rows of a thread at a time");
  const int jq = ((int)threadIdx.x % TPR) * 4, ir = (int)threadIdx.x / TPR;
  const int nsplit = partial_count(u, i0, j0);
  // two of the thread's rows at a time, with the model row and up to 8 partials of both in
  // flight together (a partial beyond the 8th, rare, is fetched afterwards); summed in split order
#pragma unroll 1
  for (int r2 = 0; r2 < NPASS / 2; ++r2) {
    float4 wc[2], v[2][8];
    bool ok[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int i = i0 + ir + RPP * (2 * r2 + h), j = j0 + jq;
      ok[h] = i < u.d_in && j < u.d_out;
      if (ok[h]) {
        const float* pp = u.partial + (size_t)i * u.ldp + j;
        wc[h] = *(const float4*)(u.w_cur + (size_t)i * u.d_out + j);
#pragma unroll
        for (int z = 0; z < 8; ++z)
          if (z < nsplit) v[h][z] = *(const float4*)(pp + (size_t)z * u.split_stride);
      }
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int il = ir + RPP * (2 * r2 + h), i = i0 + il, j = j0 + jq;
      uint2 hh = make_uint2(0, 0);
      if (ok[h]) {
        float4 G = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int z = 0; z < 8; ++z)
          if (z < nsplit) { G.x += v[h][z].x; G.y += v[h][z].y; G.z += v[h][z].z; G.w += v[h][z].w; }
        for (int z = 8; z < nsplit; ++z) {
          const float4 t = *(const float4*)(u.partial + (size_t)i * u.ldp + j + (size_t)z * u.split_stride);
          G.x += t.x; G.y += t.y; G.z += t.z; G.w += t.w;
        }
        float4 w = wc[h];
        w.x -= G.x; w.y -= G.y; w.z -= G.z; w.w -= G.w;
        *(float4*)(u.w_next + (size_t)i * u.d_out + j) = w;
        hh.x = f32_to_bf16(w.x) | ((uint32_t)f32_to_bf16(w.y) << 16);
        hh.y = f32_to_bf16(w.z) | ((uint32_t)f32_to_bf16(w.w) << 16);
        if (u.wn) *(uint2*)(u.wn + (size_t)i * u.ldwn + j) = hh;
      }
      *(uint32_t*)&tile[il * PT + jq] = hh.x;
      *(uint32_t*)&tile[il * PT + jq + 2] = hh.y;
    }
  }
  __syncthreads();
  // transposed bf16 copy: thread -> column j, 8 consecutive rows i (the padded pitch of wt makes
  // the 16-byte store safe; rows beyond d_in hold zeros, which is what the padding must be)
  for (int q = threadIdx.x; q < TJ * 8; q += NT) {
    const int jl = q >> 3, ib = (q & 7) * 8;
    const int j = j0 + jl;
    if (j < u.d_out) {
      uint16_t v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = tile[(ib + e) * PT + jl];
      uint4 o;
      o.x = v[0] | ((uint32_t)v[1] << 16); o.y = v[2] | ((uint32_t)v[3] << 16);
      o.z = v[4] | ((uint32_t)v[5] << 16); o.w = v[6] | ((uint32_t)v[7] << 16);
      *(uint4*)(u.wt + (size_t)j * u.ldwt + i0 + ib) = o;
    }
  }
}

// ------------------------------------------------------------------ the GEMM
enum { EPI_RELU = 0, EPI_LOGITS = 1, EPI_DGRAD = 2, EPI_WGRAD = 3 };

// ------------------------------------------------------------------ bias update
// b_j <- b_j - sum over the rows of dZ_l[.][j] (Eq. 2 / Eq. 3 for the biases).  The producers of
// dZ_l leave the column sums of every block of 64 rows (128 for the output layer); 16 threads per entry
// add them (partial row g, g + 16, ... each, then the 16 shares in order).  A block of 256 threads
// takes 16 consecutive entries of the concatenated bias vectors.
struct BiasCore {
  int L;
  int col_begin[ABS_MAX_LAYERS + 1];       // prefix of valid columns over the layers
  const float* colsum[ABS_MAX_LAYERS]; size_t ldcs[ABS_MAX_LAYERS];
  size_t b_off[ABS_MAX_LAYERS];
  const float* w_cur; float* w_next;
  int prow[ABS_MAX_LAYERS];                // row blocks of colsum[l] (per upload in the per-upload form)
};
// blk: which 16 entries; first_row_block(l): where the sum over layer l's row blocks starts; cur / nxt:
// the model read and written.  Threads 0 .. 255 of the workgroup work, all of them meet the barrier.
template <typename FirstRow>
__device__ __forceinline__ void bias_block(const BiasCore& a, int blk, FirstRow first_row_block, const float* cur,
                                           float* nxt, float* lds) {
  float (*s_part)[17] = (float (*)[17])lds;
  const int t = threadIdx.x, cl = t & 15, grp = (t >> 4) & 15;
  const int w = blk * 16 + cl;
  const int ncol = a.col_begin[a.L];
  float s = 0.f;
  int l = 0, j = 0;
  if (w < ncol && t < 256) {
    while (w >= a.col_begin[l + 1]) ++l;
    j = w - a.col_begin[l];
    const int prow = a.prow[l];
    const float* src = a.colsum[l] + (size_t)first_row_block(l) * a.ldcs[l] + j;
    int r = grp;
    for (; r + 48 < prow; r += 64) {         // four loads in flight
      const float v0 = src[(size_t)r * a.ldcs[l]], v1 = src[(size_t)(r + 16) * a.ldcs[l]];
      const float v2 = src[(size_t)(r + 32) * a.ldcs[l]], v3 = src[(size_t)(r + 48) * a.ldcs[l]];
      s += v0; s += v1; s += v2; s += v3;
    }
    for (; r < prow; r += 16) s += src[(size_t)r * a.ldcs[l]];
  }
  if (t < 256) s_part[grp][cl] = s;
  __syncthreads();
  if (t < 16 && w < ncol) {
    float sum = 0.f;
#pragma unroll
    for (int g = 0; g < 16; ++g) sum += s_part[g][cl];
    nxt[a.b_off[l] + j] = cur[a.b_off[l] + j] - sum;
  }
}

struct GemmArgs {
  const uint16_t* A;  size_t lda;     // [Mdim][lda], k contiguous
  const uint32_t* a_rowidx;           // GATHER: row m of A is A + a_rowidx[m] * lda
  int a_kvalid;                       // GATHER: k >= a_kvalid reads as zero
  const uint16_t* Bt; size_t ldb;     // [Ndim][ldb], k contiguous
  size_t bt_slot_stride;              // PER_UPLOAD: Bt += slot(upload of the row tile) * stride
  int rows_per_upload;                // Bp
  int by_upload;                      // PER_UPLOAD: the slot is the upload's position (private models) instead of its ring slot
  int ksteps_total;                   // BK-steps of the whole contraction
  int ksteps_per_split;               // BK-steps per blockIdx.z
  const float* bias; size_t bias_slot_stride; int n_valid;   // EPI_RELU / EPI_LOGITS
  uint16_t* out;  size_t ldo;         // bf16 [Mdim][ldo]   (may be null)
  uint16_t* outT; size_t ldoT;        // bf16 [Ndim][ldoT]  (may be null)
  float* outf;    size_t ldof;        // fp32 [Mdim][ldof]; EPI_WGRAD: + z * split_stride
  size_t split_stride;
  int mt, nt, nsplit, rows_per_xcd;   // tile grid (see the block -> tile mapping in the kernel)
  const uint16_t* maskT; size_t ldmaskT; // EPI_DGRAD: H_l^T [Ndim][ldmaskT]; the gradient passes where H_l > 0
  float* colsum; size_t ldcs;         // EPI_DGRAD: column sums of the bf16 results per block of 64 rows, [Mdim / 64][ldcs]
  // 256 x 256 tile kernel only: the ReLU mask as one bit per element in the kernel's own accumulator
  // order (16 bytes per lane and tile: [tile][wavefront][lane][4 words], word a / 2, bit (a & 1) 16 + 4 b + r
  // for the 16 x 16 block (a, b) of the wavefront's sub-tile and accumulator register r).
  // EPI_RELU writes it when set; EPI_DGRAD reads it instead of maskT when set.
  uint32_t* maskbits;
  // 256 x 256 tile kernel, bf16 outputs: store them without keeping their lines in the L2 (set by the
  // launcher for outputs much larger than the L2s: see store16_stream)
  int stream_out;
  // GATHER with gen_rows set: the kernel draws the minibatch rows itself (stacked row m = upload
  // m / rows_per_upload, sample m % rows_per_upload; Section II-A: independent uniform draws from the
  // worker's shard) instead of reading a_rowidx, and the workgroups of the first column tile leave
  // them, with their labels, in gen_rowidx / gen_label for the kernels that follow.
  int gen_rows;
  int gen_B;                          // samples per upload (rows beyond are padding: label -1)
  uint64_t gen_shard_rows, gen_batch_key;
  uint32_t gen_draw0;                 // first draw index of this step (local step u: u B)
  const int32_t* gen_y;
  uint32_t* gen_rowidx; int32_t* gen_label;
  // EPI_WGRAD on the 256 x 256 tile kernel with sk_q > 0: instead of nsplit equal row ranges per
  // output tile, the mt nt ksteps_total (tile, k-step) pairs, tile after tile, are cut into runs of
  // sk_q and workgroup w takes run w - a run may end in one tile and begin the next.  Every workgroup
  // then does the same number of k-steps whatever the tile count (96 tiles on 256 CUs: two splits
  // each leave a quarter of the CUs idle, runs of 48 k-steps none); a tile's partials are the pieces
  // of the runs that touch it, in order, slot = piece number.
  int sk_q;
  // EPI_WGRAD with pig_blocks > 0: the launch's first pig_blocks workgroups do not belong to this
  // product at all - each applies Eq. 3 to one 64 x pig_tj block of ANOTHER layer's weight matrix,
  // whose split partials the previous launch completed (pig_upd).  The update is bound by memory, the
  // product by the matrix cores, and a weight-gradient launch rarely has a whole number of waves of
  // tiles: sharing a launch lets the two overlap without streams, events or fences.
  int pig_blocks, pig_tj;
  TileUpdate pig_upd;
  // ... and its very last bias_blocks workgroups the round's bias update (every dZ_l and its column
  // sums are complete before the first weight-gradient launch).
  int bias_blocks;
  BiasCore bias_upd;
  // EPI_DGRAD with pub_mailbox set: the first workgroup publishes the uploads' mean minibatch losses
  // (sums of pub_nb row blocks each, left by the output-layer kernel) before it starts on its tile.
  LossMailbox* pub_mailbox; const float* pub_rowloss; int pub_nb; int pub_B;
};

// Dataset row of stacked row m (and whether it carries a sample).
__device__ __forceinline__ uint32_t gen_row_of(const GemmArgs& g, const RoundDesc& rd, int m, bool* real) {
  const int up = m / g.rows_per_upload, b = m - up * g.rows_per_upload;
  const WorkerDesc w = rd.w[up];
  uint64_t row = (uint64_t)w.id * g.gen_shard_rows;
  *real = b < g.gen_B;
  if (b < g.gen_B) row += draw(job_key(g.gen_batch_key, w.id, w.job), g.gen_draw0 + (uint32_t)b) % g.gen_shard_rows;
  return (uint32_t)row;
}
__device__ __forceinline__ void gen_row_store(const GemmArgs& g, int m, uint32_t row, bool real) {
  g.gen_rowidx[m] = row;
  g.gen_label[m] = real ? g.gen_y[row] : -1;
}

// The uploads' mean minibatch losses (what each worker reports next to its gradient) into the
// mailbox, then the stamp: thread a < K adds the loss sums of upload a's row blocks in order.  Every
// wavefront that wrote fences at system scope before the barrier, so the host that sees the stamp
// sees the losses.  Whole workgroup, uniform call.
__device__ __forceinline__ void publish_upload_losses(LossMailbox* box, const float* rowloss, int nb, int B,
                                                      int K, uint32_t stamp) {
  const int up = threadIdx.x;
  if (up < K) {
    float sum = 0.f;
    for (int q = 0; q < nb; ++q) sum += rowloss[(size_t)up * nb + q];
    box->loss[up] = sum / (float)B;
  }
  if (threadIdx.x < ABS_MAX_WORKERS) __threadfence_system();
  __syncthreads();
  if (threadIdx.x == 0) box->stamp = stamp;
}

// A piggybacked update block (see GemmArgs::pig_blocks): block b of the other layer's matrix, 64 rows
// x pig_tj columns, by the NT threads of this workgroup.  Blocks beyond the matrix (the count is
// rounded up to a multiple of 8 to keep the product's block -> XCD mapping) do nothing.
template <int NT, bool WIDE_OK>
__device__ __forceinline__ void piggy_update(const GemmArgs& g, int b, uint16_t* lds) {
  const TileUpdate& u = g.pig_upd;
  const int rows = (u.d_in + 63) / 64;
  if (WIDE_OK && g.pig_tj == 256) {
    const int nbx = (u.d_out + 255) / 256;
    if (b < nbx * rows) update_block64<NT, 256>(u, (b / nbx) * 64, (b % nbx) * 256, lds);
  } else {
    const int nbx = (u.d_out + 63) / 64;
    if (b < nbx * rows) update_block64<NT, 64>(u, (b / nbx) * 64, (b % nbx) * 64, lds);
  }
}

__device__ __forceinline__ void lds_dma16(const uint16_t* gsrc, uint16_t* lds_block) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_block, 16, 0, 0);
}

// 256 threads = 2 x 2 wavefronts; a wavefront owns a 64 x (TN/2) sub-tile made of
// 32x32x16 MFMA blocks (TN = 256: 2 x 4 blocks, 128 accumulator registers).  A and B
// tiles of BK = 64 are staged in LDS (one stage; the next tile's global loads are in
// flight in registers while the current one is multiplied, and two workgroups per CU
// cover each other's barriers).  A tile row is 128 bytes; its 16-byte chunk c is stored at
// position c ^ ((row >> 1) & 7): the 16 lanes that one cycle of a 128-bit LDS read serves
// (16 consecutive rows of a fragment) then cover all 64 banks.
#ifndef ABS_RING64
#define ABS_RING64 3
#endif
#ifndef ABS_RING128
#define ABS_RING128 2
#endif
template <int TN>
struct GemmCfg {
  static constexpr int WN = TN / 2;            // columns per wavefront
  static constexpr int NI = WN / 32;           // MFMA blocks along n per wavefront
  static constexpr int BCH = TN / 32;          // 16-byte chunks of the B tile per thread
  static constexpr int kMainElems = (TM + TN) * BK;
  static constexpr int kEpiPitch = 64 + 8;     // transposed staging: [WN][64 + 8] per wavefront
  static constexpr int kEpiElems = 4 * WN * kEpiPitch;
};

// TAG only separates kernel symbols (first layer / other layers) for profilers.
//
// RING > 0: the tiles travel global -> LDS by DMA through a ring of RING stages with RING - 1
// tiles in flight and one barrier per k-step (as in the 256 x 256 kernel, swizzle on the global
// side).  For products with few tiles per CU, where one tile in flight per workgroup leaves the
// k-steps waiting for memory latency one after the other.  Needs whole 64-wide k-steps of A
// (a_kvalid a multiple of BK covering the contraction).  KPS > 1: a stage holds KPS consecutive
// k-steps, requested, awaited and released together (one barrier per KPS k-steps).
template <int TN, int EPI, bool GATHER, bool PER_UPLOAD, int TAG, int RING = 0, int KPS = 1>
__global__ __launch_bounds__(256, (RING * KPS * GemmCfg<TN>::kMainElems * 2 > 80 * 1024) ? 1 : 2)
void mlp_gemm_kernel(GemmArgs g, RoundDesc rd) {
  using Cfg = GemmCfg<TN>;
  constexpr int WN = Cfg::WN, NI = Cfg::NI, BCH = Cfg::BCH;
  constexpr bool kStageT = (EPI == EPI_RELU || EPI == EPI_DGRAD);
  static_assert(KPS == 1 || RING > 0, "several k-steps per stage: ring only");
  constexpr int kStageElems = KPS * Cfg::kMainElems;       // a ring stage holds KPS consecutive k-steps
  constexpr int kMain = (RING ? RING : 1) * kStageElems;
  constexpr int kSmem = kStageT && Cfg::kEpiElems > kMain ? Cfg::kEpiElems : kMain;
  static_assert(kSmem * 2 <= 160 * 1024, "LDS budget");
  __shared__ __attribute__((aligned(16))) uint16_t smem[kSmem];

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int bx = blockIdx.x;
  if (EPI == EPI_WGRAD && (g.pig_blocks | g.bias_blocks)) {
    // The update's blocks come last in the grid: they take the CUs that the product's last wave of
    // tiles leaves idle and the tail.  (Dealt out evenly between the tiles they slowed every tile
    // down: 260 -> 400 us for the hidden layer's product at K = 128.)  Behind them the bias blocks.
    const int own = (int)gridDim.x - g.pig_blocks - g.bias_blocks;
    if (bx >= own + g.pig_blocks) {
      bias_block(g.bias_upd, bx - own - g.pig_blocks, [](int) { return 0; }, g.bias_upd.w_cur, g.bias_upd.w_next, (float*)smem);
      return;
    }
    if (bx >= own) { piggy_update<256, false>(g, bx - own, smem); return; }
  }
  // Block -> tile mapping.  Workgroups are handed to the 8 XCDs round-robin and every XCD has
  // its own L2, so block b works for XCD b % 8.  The (split, row-tile) pairs are cut into 8
  // contiguous ranges, one per XCD, and inside a range consecutive blocks sweep the column
  // tiles of one row tile: the blocks resident on an XCD then share their A rows (and, for
  // neighbouring row tiles of the same upload, their B rows) through that XCD's L2.
  const int xcd = bx & 7, jx = bx >> 3;
  const int trow = xcd * g.rows_per_xcd + jx / g.nt;
  if (trow >= g.mt * g.nsplit) return;
  const int zsplit = trow / g.mt;
  const int m0 = (trow - zsplit * g.mt) * TM, n0 = (jx % g.nt) * TN;
  const int ks0 = zsplit * g.ksteps_per_split;
  const int ks1 = min(g.ksteps_total, ks0 + g.ksteps_per_split);

  if (EPI == EPI_DGRAD && g.pub_mailbox && blockIdx.x == 0)
    publish_upload_losses(g.pub_mailbox, g.pub_rowloss, g.pub_nb, g.pub_B, rd.K, rd.stamp);

  const uint16_t* Bt = g.Bt;
  uint32_t slot = 0;
  if (PER_UPLOAD) {
    slot = g.by_upload ? (uint32_t)(m0 / g.rows_per_upload) : rd.w[m0 / g.rows_per_upload].slot;
    Bt += (size_t)slot * g.bt_slot_stride;
  }

  // staging.  Register path: thread t moves chunk (row r0 + 32 i, 16-byte column c) of each tile.
  // DMA path: instruction i of wavefront w fills 8 rows of 128 bytes, lane l row (l >> 3) of them at
  // chunk position l & 7, fetching logical chunk (l & 7) ^ ((row >> 1) & 7): A rows 32 w + 8 i
  // (i < 4), B rows (TN / 4) w + 8 i (i < TN / 32); (row >> 1) & 7 is (l >> 4) + 4 (i & 1) for both.
  constexpr int kRowStep = RING ? 8 : 32;
  const int r0 = RING ? wave * 32 + (lane >> 3) : t >> 3;
  const int c8 = (t & 7) * 8;
  const int c_even = ((t & 7) ^ ((lane >> 4) & 7)) * 8, c_odd = ((t & 7) ^ ((4 + (lane >> 4)) & 7)) * 8;
  const int st_off = r0 * BK + (((t & 7) ^ ((r0 >> 1) & 7)) << 3);   // swizzled LDS offset of chunk i = 0
  const uint16_t* pa0; const uint16_t* pa1; const uint16_t* pa2; const uint16_t* pa3;
  if (GATHER) {
    uint32_t ri[4];
    if (g.gen_rows) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bool real;
        ri[i] = gen_row_of(g, rd, m0 + r0 + kRowStep * i, &real);
        if (n0 == 0 && (t & 7) == 0) gen_row_store(g, m0 + r0 + kRowStep * i, ri[i], real);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) ri[i] = g.a_rowidx[m0 + r0 + kRowStep * i];
    }
    pa0 = g.A + (size_t)ri[0] * g.lda + (RING ? c_even : c8);
    pa1 = g.A + (size_t)ri[1] * g.lda + (RING ? c_odd : c8);
    pa2 = g.A + (size_t)ri[2] * g.lda + (RING ? c_even : c8);
    pa3 = g.A + (size_t)ri[3] * g.lda + (RING ? c_odd : c8);
  } else if (RING) {
    const uint16_t* base = g.A + (size_t)(m0 + r0) * g.lda;
    pa0 = base + c_even; pa1 = base + 8 * g.lda + c_odd;
    pa2 = base + 16 * g.lda + c_even; pa3 = base + 24 * g.lda + c_odd;
  } else {
    pa0 = g.A + (size_t)(m0 + r0) * g.lda + c8;
    pa1 = pa0 + 32 * g.lda; pa2 = pa0 + 64 * g.lda; pa3 = pa0 + 96 * g.lda;
  }
  const uint16_t* pb0 = RING ? Bt + (size_t)(n0 + wave * (TN / 4) + (lane >> 3)) * g.ldb
                             : Bt + (size_t)(n0 + r0) * g.ldb + c8;
  const size_t b_step = (RING ? 8 : 32) * g.ldb;
  const bool a_ok = !GATHER || c8 < g.a_kvalid;       // refined per k-step below

  f32x16_t acc[2][NI];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  uint4 ra0, ra1, ra2, ra3, rb0, rb1, rb2, rb3, rb4, rb5, rb6, rb7;
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  rb2 = rb3 = rb4 = rb5 = rb6 = rb7 = zero4;
#define ABS_FETCH(ks)                                                                     \
  {                                                                                       \
    const int k0_ = (ks) * BK;                                                            \
    if (GATHER && (!a_ok || k0_ + c8 >= g.a_kvalid)) {                                    \
      ra0 = zero4; ra1 = zero4; ra2 = zero4; ra3 = zero4;                                 \
    } else {                                                                              \
      ra0 = *(const uint4*)(pa0 + k0_); ra1 = *(const uint4*)(pa1 + k0_);                 \
      ra2 = *(const uint4*)(pa2 + k0_); ra3 = *(const uint4*)(pa3 + k0_);                 \
    }                                                                                     \
    const uint16_t* pb_ = pb0 + k0_;                                                      \
    rb0 = *(const uint4*)(pb_); rb1 = *(const uint4*)(pb_ + b_step);                      \
    if (BCH > 2) { rb2 = *(const uint4*)(pb_ + 2 * b_step); rb3 = *(const uint4*)(pb_ + 3 * b_step); } \
    if (BCH > 4) { rb4 = *(const uint4*)(pb_ + 4 * b_step); rb5 = *(const uint4*)(pb_ + 5 * b_step);   \
                   rb6 = *(const uint4*)(pb_ + 6 * b_step); rb7 = *(const uint4*)(pb_ + 7 * b_step); } \
  }
#define ABS_STAGE()                                                                       \
  {                                                                                       \
    *(uint4*)&smem[st_off] = ra0;            *(uint4*)&smem[st_off + 32 * BK] = ra1;          \
    *(uint4*)&smem[st_off + 64 * BK] = ra2;  *(uint4*)&smem[st_off + 96 * BK] = ra3;          \
    *(uint4*)&smem[TM * BK + st_off] = rb0;            *(uint4*)&smem[TM * BK + st_off + 32 * BK] = rb1;          \
    if (BCH > 2) { *(uint4*)&smem[TM * BK + st_off + 64 * BK] = rb2; *(uint4*)&smem[TM * BK + st_off + 96 * BK] = rb3; }   \
    if (BCH > 4) { *(uint4*)&smem[TM * BK + st_off + 128 * BK] = rb4; *(uint4*)&smem[TM * BK + st_off + 160 * BK] = rb5;   \
                   *(uint4*)&smem[TM * BK + st_off + 192 * BK] = rb6; *(uint4*)&smem[TM * BK + st_off + 224 * BK] = rb7; } \
  }

  const int lr = lane & 31, lk = lane >> 5;
  const int fa_row = (wm * 64 + lr) * BK, fb_row = (wn * WN + lr) * BK;
  const int sw = (lr >> 1) & 7;
  // one request per 8 rows: stage `st_` receives tile `ks_`
#define ABS_RING_DMA(ks_, st_)                                                            \
  _Pragma("unroll") for (int p_ = 0; p_ < KPS; ++p_) {                                    \
    const int k0_ = ((ks_) + p_) * BK;                                                    \
    uint16_t* a_ = smem + (st_) * kStageElems + p_ * Cfg::kMainElems + wave * 32 * BK;    \
    uint16_t* b_ = smem + (st_) * kStageElems + p_ * Cfg::kMainElems + TM * BK + wave * (TN / 4) * BK; \
    lds_dma16(pa0 + k0_, a_);            lds_dma16(pa1 + k0_, a_ + 8 * BK);               \
    lds_dma16(pa2 + k0_, a_ + 16 * BK);  lds_dma16(pa3 + k0_, a_ + 24 * BK);              \
    _Pragma("unroll") for (int i = 0; i < TN / 32; ++i)                                   \
      lds_dma16(pb0 + i * b_step + ((i & 1) ? c_odd : c_even) + k0_, b_ + i * 8 * BK);    \
  }
  constexpr int kDmaPerWave = KPS * (4 + TN / 32);        // requests per wavefront and stage
  if (ks0 < ks1) {
    if (RING) {
#pragma unroll
      for (int j = 0; j < RING - 1; ++j)
        if (ks0 + j * KPS < ks1) ABS_RING_DMA(ks0 + j * KPS, j);
    } else {
      ABS_FETCH(ks0);
    }
    int stage = 0;
    for (int ks = ks0; ks < ks1; ++ks) {
      const uint16_t* sA = smem;
      if (RING) {
        // (KPS > 1: the launcher hands over whole stages, ks1 - ks0 a multiple of KPS; wait, barrier and
        // requests happen once per stage, at its first k-step)
        const int pnl = KPS > 1 ? (ks - ks0) % KPS : 0;
        if (pnl == 0) {
          // stage ks has landed when at most the RING - 2 stages behind it are outstanding
          constexpr int kOut = RING > 2 ? (RING - 2) * kDmaPerWave : 0;
          if (ks + (RING - 2) * KPS < ks1) __builtin_amdgcn_s_waitcnt(0x0F70 | (kOut & 15) | ((kOut >> 4) << 14));
          else                             __builtin_amdgcn_s_waitcnt(0x0F70);
          __syncthreads();      // ... for every wavefront; and everybody is done with stage ks - KPS
          if (ks + (RING - 1) * KPS < ks1) ABS_RING_DMA(ks + (RING - 1) * KPS, stage == 0 ? RING - 1 : stage - 1);
        }
        sA = smem + stage * kStageElems + pnl * Cfg::kMainElems;
        if (pnl == KPS - 1) stage = stage + 1 == RING ? 0 : stage + 1;
      } else {
        ABS_STAGE();
        __syncthreads();
        if (ks + 1 < ks1) ABS_FETCH(ks + 1);
      }
      const uint16_t* sB = sA + TM * BK;
      // fragments of sub-step s+1 are read while the MFMAs of sub-step s run
      bf16x8_t fa[2][2], fb[2][NI];
#define ABS_FRAGS(set, s_)                                                                        \
  {                                                                                               \
    const int ch_ = ((((s_) << 1) | lk) ^ sw) << 3;                                               \
    _Pragma("unroll") for (int mi = 0; mi < 2; ++mi)                                              \
      fa[set][mi] = *(const bf16x8_t*)&sA[fa_row + mi * 32 * BK + ch_];                           \
    _Pragma("unroll") for (int ni = 0; ni < NI; ++ni)                                             \
      fb[set][ni] = *(const bf16x8_t*)&sB[fb_row + ni * 32 * BK + ch_];                           \
  }
      ABS_FRAGS(0, 0);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        if (s < 3) ABS_FRAGS((s + 1) & 1, s + 1);
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s & 1][mi], fb[s & 1][ni], acc[mi][ni], 0, 0, 0);
      }
#undef ABS_FRAGS
      // pin the interleaving: first fragment set, then one LDS read behind each MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 2 + NI, 0);
#pragma unroll
      for (int s = 0; s < 3; ++s) {
#pragma unroll
        for (int i = 0; i < 2 + NI; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (2 * NI > 2 + NI) __builtin_amdgcn_sched_group_barrier(0x008, 2 * NI - (2 + NI), 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * NI, 0);
      if (!RING) __syncthreads();
    }
  }
  if (RING) __syncthreads();      // all fragment reads done before the staging area is reused

#undef ABS_RING_DMA
#undef ABS_FETCH
#undef ABS_STAGE

  // ---- epilogue.  Accumulator register r of lane l holds C[8 (r/4) + 4 (l/32) + r%4][l%32]
  // of its 32 x 32 block.
  const int lcol = lane & 31, lrow4 = (lane >> 5) * 4;
  const float* bias = nullptr;
  if (EPI == EPI_RELU || EPI == EPI_LOGITS) bias = g.bias + (size_t)slot * g.bias_slot_stride;
  float* outf = g.outf;
  if (EPI == EPI_WGRAD) outf += (size_t)zsplit * g.split_stride;
  uint16_t* const sE = smem + wave * (WN * Cfg::kEpiPitch);     // this wavefront's [WN][72] staging
  float cs[NI];                           // EPI_DGRAD: column sums over this wavefront's 64 rows
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) cs[ni] = 0.f;
  if (EPI == EPI_DGRAD) {
    // the ReLU mask of this wavefront's tile, H_l^T [n][m], fetched as whole 128-byte rows into
    // the staging area; every lane later replaces the 4 entries it read by its 4 results
    const int mrow = m0 + wm * 64;
#pragma unroll
    for (int i = 0; i < WN / 8; ++i) {
      const int q = lane + 64 * i, nl = q >> 3, ch = (q & 7) * 8;
      *(uint4*)&sE[nl * Cfg::kEpiPitch + ch] =
          *(const uint4*)(g.maskT + (size_t)(n0 + wn * WN + nl) * g.ldmaskT + mrow + ch);
    }
  }
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int nl = ni * 32 + lcol;
      const int n = n0 + wn * WN + nl;
      float bv = 0.f;
      if (EPI == EPI_RELU || EPI == EPI_LOGITS) bv = n < g.n_valid ? bias[n] : 0.f;
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int ml = mi * 32 + rg * 8 + lrow4;
        const int mbase = m0 + wm * 64 + ml;
        uint16_t h[4];
        uint2 hm = make_uint2(0, 0);     // H_l of the 4 consecutive rows this lane holds
        if (EPI == EPI_DGRAD) hm = *(const uint2*)&sE[nl * Cfg::kEpiPitch + ml];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const int m = mbase + rr;
          float v = acc[mi][ni][rg * 4 + rr];
          if (EPI == EPI_RELU) {
            v = fmaxf(v + bv, 0.f);
          } else if (EPI == EPI_LOGITS) {
            v += bv;
            outf[(size_t)m * g.ldof + n] = v;
          } else if (EPI == EPI_DGRAD) {
            const uint32_t pair = rr < 2 ? hm.x : hm.y;
            v = ((pair >> ((rr & 1) * 16)) & 0x7FFFu) ? v : 0.f;
          } else {
            outf[(size_t)m * g.ldof + n] = v;
          }
          if (kStageT) {
            h[rr] = f32_to_bf16(v);
            if (EPI == EPI_DGRAD) cs[ni] += __uint_as_float((uint32_t)h[rr] << 16);
            if (g.out) g.out[(size_t)m * g.ldo + n] = h[rr];
          }
        }
        if (kStageT) {
          uint2 o;
          o.x = h[0] | ((uint32_t)h[1] << 16);
          o.y = h[2] | ((uint32_t)h[3] << 16);
          *(uint2*)&sE[nl * Cfg::kEpiPitch + ml] = o;
        }
      }
    }
  }
  if (EPI == EPI_DGRAD) {
    // the bias gradient's share of these 64 rows (the two half-wavefronts hold alternate rows)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const float c = cs[ni] + __shfl_xor(cs[ni], 32, 64);
      if (lane < 32) g.colsum[(size_t)((m0 + wm * 64) >> 6) * g.ldcs + n0 + wn * WN + ni * 32 + lcol] = c;
    }
  }
  if (kStageT) {
    // transposed copy: each staged row is 64 consecutive m of one n -> 16-byte stores
    __syncthreads();
    const int mrow = m0 + wm * 64;
#pragma unroll
    for (int i = 0; i < WN / 8; ++i) {
      const int q = lane + 64 * i, nl = q >> 3, ch = (q & 7) * 8;
      const uint4 v = *(const uint4*)&sE[nl * Cfg::kEpiPitch + ch];
      *(uint4*)(g.outT + (size_t)(n0 + wn * WN + nl) * g.ldoT + mrow + ch) = v;
    }
  }
}

// ------------------------------------------------------------------ the large-tile GEMM
// 256 x 256 tile, 512 threads = 2 x 4 wavefronts of 128 x 64 (8 x 4 blocks of MFMA 16x16x32, 128
// accumulator registers), BK = 64.  On gfx950 the LDS accepts about 64 B/clk of writes
// against 256 B/clk of reads and the L1 delivers 64 B/clk, so what bounds a bf16 GEMM
// tile is the bytes staged per flop: a 256 x 256 tile stages 64 KB per 8.4 MFLOP, two
// thirds of what the 128 x 256 tile needs.  Tiles go from global memory straight into
// LDS (global_load_lds_dwordx4: lane l of a wavefront fills bytes [16 l, 16 l + 16) of a
// 1 KB LDS block, i.e. 8 rows of 128 B), two stages, so the loads of step k+1 are in
// flight during all of step k and there is one barrier per step.  The XOR swizzle is
// applied on the global side: the lane that fills chunk position p of row r fetches
// logical chunk p ^ ((r >> 1) & 7).
// Needs: row count and column count multiples of 256, GATHER with d_0 equal to the padded
// k extent (d_0 % 128 == 0: a gathered row is read over the whole k range).
constexpr int TM3 = 256, TN3 = 256;
constexpr int kStage3 = (TM3 + TN3) * BK;            // elements per LDS stage (64 KB)
constexpr int kEpiPitch3 = 64 + 8;                   // per wavefront: staging [64 n][72] and [64 m][72]
constexpr int kEpiElems3 = 8 * 2 * 64 * kEpiPitch3;   // 147456 B
constexpr int kSmem3 = 2 * kStage3 > kEpiElems3 ? 2 * kStage3 : kEpiElems3;
static_assert(kSmem3 * 2 <= 160 * 1024, "LDS budget");

// The same request written out by hand.  The compiler makes every LDS read that it cannot tell
// apart from a pending global->LDS request wait for all of them, and it cannot for the
// transposing read: a k-step would then start by waiting for the tile it has just requested.
// Requests issued this way are invisible to that bookkeeping; the loop's own vmcnt(0) and
// barrier order them against the reads.  The LDS base travels in m0, which the register
// allocator hands over through the "{m0}" constraint (it knows the register is written).
__device__ __forceinline__ void lds_dma16_raw(const uint16_t* gsrc, uint16_t* lds_block) {
  const uint32_t lds = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_block);
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(gsrc), "{m0}"(lds)
               : "memory");
}

template <int EPI, bool GATHER, bool PER_UPLOAD, int TAG>
__global__ __launch_bounds__(512, 1) void mlp_gemm256_kernel(GemmArgs g, RoundDesc rd) {
  // TAG 2 (first-layer weight gradient): the A operand is the dataset itself, rows gathered by
  // a_rowidx and the contraction running over those rows, i.e. A arrives as [k][m] instead of
  // [m][k]; its fragments are read with the transposing LDS read, so no transposed copy of
  // the minibatch is ever written.
  // TAG 3 (forward / input gradient of a hidden layer): the A operand is the TRANSPOSED copy of the
  // activations / output gradients, [k = features][m = stacked rows], read the same way - the layer
  // that produced it then writes no row-major copy at all.
  constexpr bool kATR = (EPI == EPI_WGRAD && TAG == 2) || ((EPI == EPI_RELU || EPI == EPI_DGRAD) && TAG == 3);
  constexpr bool kARows = kATR && EPI == EPI_WGRAD;      // the k rows of A are gathered through a_rowidx
  __shared__ __attribute__((aligned(16))) uint16_t smem[kSmem3];

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int bx = blockIdx.x;
  if (EPI == EPI_WGRAD && (g.pig_blocks | g.bias_blocks)) {
    // The update's blocks come last in the grid: they take the CUs that the product's last wave of
    // tiles leaves idle and the tail.  (Dealt out evenly between the tiles they slowed every tile
    // down: 260 -> 400 us for the hidden layer's product at K = 128.)  Behind them the bias blocks.
    const int own = (int)gridDim.x - g.pig_blocks - g.bias_blocks;
    if (bx >= own + g.pig_blocks) {
      bias_block(g.bias_upd, bx - own - g.pig_blocks, [](int) { return 0; }, g.bias_upd.w_cur, g.bias_upd.w_next, (float*)smem);
      return;
    }
    if (bx >= own) { piggy_update<512, true>(g, bx - own, smem); return; }
  }
  int m0, n0, zsplit, ks0, ks1;
  // runs of k-steps across tiles (sk_q > 0): this workgroup's next (tile, k-step) pair and the end of
  // its run.
  const bool kRuns = EPI == EPI_WGRAD && g.sk_q > 0;
  int sk_u = 0, sk_end = 0;
  if (kRuns) {
    const int own = (int)gridDim.x - g.pig_blocks - g.bias_blocks;
    // Block b runs on XCD b % 8.  When eight runs span a whole number of tiles' k ranges
    // (8 q = 0 mod k-steps), runs b, b + 8, b + 16, ... start at the same k-step of their tiles: handing
    // run b to block b puts workgroups on one XCD that walk the same k range in step and share their
    // A and B panels in that XCD's L2.  Otherwise an XCD takes neighbouring runs (neighbouring tiles).
    const int lw = (8 * g.sk_q) % g.ksteps_total == 0 ? bx : (bx & 7) * (own >> 3) + (bx >> 3);
    sk_u = lw * g.sk_q;
    sk_end = min(sk_u + g.sk_q, g.mt * g.nt * g.ksteps_total);
    if (sk_u >= sk_end) return;
  } else {
    const int xcd = bx & 7, jx = bx >> 3;
    const int trow = xcd * g.rows_per_xcd + jx / g.nt;
    if (trow >= g.mt * g.nsplit) return;
    zsplit = trow / g.mt;
    m0 = (trow - zsplit * g.mt) * TM3; n0 = (jx % g.nt) * TN3;
    ks0 = zsplit * g.ksteps_per_split;
    ks1 = min(g.ksteps_total, ks0 + g.ksteps_per_split);
  }

  if (EPI == EPI_DGRAD && g.pub_mailbox && blockIdx.x == 0)
    publish_upload_losses(g.pub_mailbox, g.pub_rowloss, g.pub_nb, g.pub_B, rd.K, rd.stamp);

  for (;;) {       // one pass per piece of the run (a single pass without runs)
  if (kRuns) {
    const int tile = sk_u / g.ksteps_total;
    ks0 = sk_u - tile * g.ksteps_total;
    ks1 = min(g.ksteps_total, ks0 + (sk_end - sk_u));
    m0 = (tile / g.nt) * TM3; n0 = (tile % g.nt) * TN3;
    zsplit = sk_u / g.sk_q - tile * g.ksteps_total / g.sk_q;     // pieces of earlier runs in this tile
    sk_u += ks1 - ks0;
  }

  const uint16_t* Bt = g.Bt;
  uint32_t slot = 0;
  if (PER_UPLOAD) {
    slot = g.by_upload ? (uint32_t)(m0 / g.rows_per_upload) : rd.w[m0 / g.rows_per_upload].slot;
    Bt += (size_t)slot * g.bt_slot_stride;
  }

  // DMA assignment: wavefront w, instruction i fills rows (4 w + i) 8 .. + 8 of a tile;
  // lane l handles row + (l >> 3), chunk position l & 7.
  const int dr = wave * 32 + (lane >> 3);                  // row for i = 0; + 8 i
  const int pc = lane & 7;
  const int c_even = (pc ^ (((lane >> 4)) & 7)) * 8;        // (r >> 1) & 7 for i even
  const int c_odd = (pc ^ ((4 + (lane >> 4)) & 7)) * 8;     //               for i odd
  const uint16_t *pa0 = nullptr, *pa1 = nullptr, *pa2 = nullptr, *pa3 = nullptr;
  // kATR: a k-step's A tile is 64 gathered rows x 256 columns (512 B per row); a DMA instruction
  // fills two rows, wavefront w takes rows 8 w .. 8 w + 7.  Lane l of instruction q handles row
  // 8 w + 2 q + (l >> 5) and chunk position l & 31; the 64-byte blocks of a row are stored at block
  // position b ^ (row & 3), so that the four rows one transposing read touches cover all banks.
  const int atr_row = wave * 8 + (lane >> 5);                 // + 2 q
  const int atr_c = lane & 31;
  const int atr_col_even = m0 + (((((atr_c >> 2) ^ (lane >> 5)) << 2) | (atr_c & 3)) << 3);          // q even
  const int atr_col_odd = m0 + (((((atr_c >> 2) ^ (2 + (lane >> 5))) << 2) | (atr_c & 3)) << 3);     // q odd
  uint32_t aidx0 = 0, aidx1 = 0, aidx2 = 0, aidx3 = 0;       // dataset rows of the next tile to request
  if (kATR) {
  } else if (GATHER) {
    uint32_t ri[4];
    if (g.gen_rows) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bool real;
        ri[i] = gen_row_of(g, rd, m0 + dr + 8 * i, &real);
        if (n0 == 0 && pc == 0) gen_row_store(g, m0 + dr + 8 * i, ri[i], real);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) ri[i] = g.a_rowidx[m0 + dr + 8 * i];
    }
    pa0 = g.A + (size_t)ri[0] * g.lda + c_even;
    pa1 = g.A + (size_t)ri[1] * g.lda + c_odd;
    pa2 = g.A + (size_t)ri[2] * g.lda + c_even;
    pa3 = g.A + (size_t)ri[3] * g.lda + c_odd;
  } else {
    const uint16_t* base = g.A + (size_t)(m0 + dr) * g.lda;
    pa0 = base + c_even; pa1 = base + 8 * g.lda + c_odd;
    pa2 = base + 16 * g.lda + c_even; pa3 = base + 24 * g.lda + c_odd;
  }
  const uint16_t* bbase = Bt + (size_t)(n0 + dr) * g.ldb;
  const uint16_t* pb0 = bbase + c_even;
  const uint16_t* pb1 = bbase + 8 * g.ldb + c_odd;
  const uint16_t* pb2 = bbase + 16 * g.ldb + c_even;
  const uint16_t* pb3 = bbase + 24 * g.ldb + c_odd;
  uint16_t* const dmaA = smem + wave * 4 * 512;              // 512 elements = 1 KB per instruction
  uint16_t* const dmaB = smem + TM3 * BK + wave * 4 * 512;

  // (kATR) the four dataset rows this lane requests for k-step ks
#define ABS_AIDX(ks)                                                              \
  if (kARows) {                                                                   \
    const uint32_t* ri_ = g.a_rowidx + (size_t)(ks) * BK + atr_row;               \
    aidx0 = ri_[0]; aidx1 = ri_[2]; aidx2 = ri_[4]; aidx3 = ri_[6];               \
  } else {                                                                        \
    aidx0 = (uint32_t)((ks) * BK + atr_row);                                      \
    aidx1 = aidx0 + 2; aidx2 = aidx0 + 4; aidx3 = aidx0 + 6;                      \
  }
#define ABS_DMA(ks, stage)                                                        \
  {                                                                               \
    const int k0_ = (ks) * BK;                                                    \
    uint16_t* a_ = dmaA + (stage) * kStage3;                                      \
    uint16_t* b_ = dmaB + (stage) * kStage3;                                      \
    if (kATR) {                                                                   \
      lds_dma16_raw(g.A + (size_t)aidx0 * g.lda + atr_col_even, a_);              \
      lds_dma16_raw(g.A + (size_t)aidx1 * g.lda + atr_col_odd, a_ + 512);         \
      lds_dma16_raw(g.A + (size_t)aidx2 * g.lda + atr_col_even, a_ + 1024);       \
      lds_dma16_raw(g.A + (size_t)aidx3 * g.lda + atr_col_odd, a_ + 1536);        \
      lds_dma16_raw(pb0 + k0_, b_);        lds_dma16_raw(pb1 + k0_, b_ + 512);    \
      lds_dma16_raw(pb2 + k0_, b_ + 1024); lds_dma16_raw(pb3 + k0_, b_ + 1536);   \
    } else {                                                                      \
      lds_dma16(pa0 + k0_, a_);        lds_dma16(pa1 + k0_, a_ + 512);            \
      lds_dma16(pa2 + k0_, a_ + 1024); lds_dma16(pa3 + k0_, a_ + 1536);           \
      lds_dma16(pb0 + k0_, b_);        lds_dma16(pb1 + k0_, b_ + 512);            \
      lds_dma16(pb2 + k0_, b_ + 1024); lds_dma16(pb3 + k0_, b_ + 1536);           \
    }                                                                             \
  }

  // ---- main loop on MFMA 16x16x32.  A wavefront's 128 x 64 sub-tile is 8 x 4 blocks of 16 x 16
  // (128 accumulator registers); lane l holds row l & 15 and the 8 k values 8 (l >> 4) .. of an
  // operand block, and accumulator register r of a block is row 4 (l >> 4) + r, column l & 15.
  // Per flop this form moves a quarter of the accumulator registers in and out of the matrix pipe
  // that the 32x32x16 form does: on random operands the pipes alone sustain 2.18 instead of
  // 1.86 PFLOP/s before the chip lowers its clock, and the products got 3-7 % faster.  The
  // fragments of a 32-wide sub-step are read in halves (rows 0-63, rows 64-127 of A; B once per
  // sub-step) one half ahead of the MFMAs that use them, pinned there with sched_group_barrier.
  f32x4_t acc[8][4];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[a][b][r] = 0.f;
  const int lr = lane & 15, lk = lane >> 4;
  const int fa_row = (wm * 128 + lr) * BK, fb_row = TM3 * BK + (wn * 64 + lr) * BK;
  const int sw = (lr >> 1) & 7;
  const int ch0 = (lk ^ sw) << 3, ch1 = ((4 | lk) ^ sw) << 3;
  // kATR (A stored [k][m]): a block's fragment is two transposing reads.  Such a read works on groups
  // of 16 lanes: lane s of a group points at 4 consecutive columns of row s / 4 of a 4 x 16 piece and
  // receives column s of its 4 rows.  Quarter-wavefront q takes k rows 8 q .. 8 q + 7 of the 32-row
  // sub-step (pieces at rows + 0 and + 4), all quarters the same 16 columns; the block position is
  // XORed with the row's low bits (= s / 4) as stored.
  const int t16s = lane & 15, t16r = t16s >> 2;
  int fa_tr[8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
    fa_tr[a] = (t16r + 8 * lk) * TM3 + (wm * 4 + ((a >> 1) ^ t16r)) * 32 + 16 * (a & 1) + 4 * (t16s & 3);
  if (ks0 < ks1) {
    if (kATR) ABS_AIDX(ks0);
    ABS_DMA(ks0, 0);
    if (kATR) ABS_AIDX(min(ks0 + 1, ks1 - 1));
    for (int ks = ks0; ks < ks1; ++ks) {
      const int stage = (ks - ks0) & 1;
      __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): this wavefront's part of tile ks is in LDS
      __syncthreads();                         // ... and everybody's; everybody is done with tile ks-1
      if (ks + 1 < ks1) ABS_DMA(ks + 1, stage ^ 1);
      if (kATR) ABS_AIDX(min(ks + 2, ks1 - 1));
      const uint16_t* sS = smem + stage * kStage3;
      bf16x8_t fa[2][4], fb[2][4];
#define ABS_LOAD_A(set, s_, h_)                                                                                    \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                                  \
    if (kATR) {                                                                                                    \
      typedef short s16x4_ __attribute__((ext_vector_type(4)));                                                    \
      const uint16_t* q_ = sS + fa_tr[(h_) * 4 + i] + (s_) * 32 * TM3;                                             \
      union { s16x4_ h[2]; bf16x8_t v; } u_;                                                                       \
      u_.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_*)(q_));          \
      u_.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_*)(q_ + 4 * TM3)); \
      fa[set][i] = u_.v;                                                                                           \
    } else {                                                                                                       \
      fa[set][i] = *(const bf16x8_t*)&sS[fa_row + ((h_) * 4 + i) * 16 * BK + ((s_) ? ch1 : ch0)];                  \
    }                                                                                                              \
  }
#define ABS_LOAD_B(set, s_)     _Pragma("unroll") for (int i = 0; i < 4; ++i) fb[set][i] = *(const bf16x8_t*)&sS[fb_row + i * 16 * BK + ((s_) ? ch1 : ch0)];
#define ABS_MMA(h_, aset, bset)                                                          \
  _Pragma("unroll") for (int i = 0; i < 4; ++i)                                          \
    _Pragma("unroll") for (int b = 0; b < 4; ++b)                                        \
      acc[(h_) * 4 + i][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[aset][i], fb[bset][b], acc[(h_) * 4 + i][b], 0, 0, 0);
      ABS_LOAD_B(0, 0); ABS_LOAD_A(0, 0, 0);
      ABS_LOAD_A(1, 0, 1);                       ABS_MMA(0, 0, 0);
      ABS_LOAD_B(1, 1); ABS_LOAD_A(0, 1, 0);     ABS_MMA(1, 1, 0);
      ABS_LOAD_A(1, 1, 1);                       ABS_MMA(0, 0, 1);
                                                 ABS_MMA(1, 1, 1);
#undef ABS_LOAD_A
#undef ABS_LOAD_B
#undef ABS_MMA
      // issue order: the first fragments, then the reads of the next half spread between the
      // 16 MFMAs of the current one (a transposed A block takes two reads)
      if (kATR) {
        __builtin_amdgcn_sched_group_barrier(0x100, 12, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
#pragma unroll
        for (int i = 0; i < 12; ++i) { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
      } else {
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) { __builtin_amdgcn_sched_group_barrier(0x008, 2, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) { __builtin_amdgcn_sched_group_barrier(0x008, 2, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
    }
  }
#undef ABS_DMA
#undef ABS_AIDX
  __syncthreads();      // all fragment reads done before the staging area is reused

  // ---- epilogue: bf16 outputs leave through this wavefront's private LDS staging, half of the
  // wavefront's tile (64 x 64) at a time, staged as [n][m] for the transposed copy and as [m][n]
  // for the row-major one, so that every global store is 16 bytes per lane and 128 contiguous
  // bytes per row.  The ReLU mask of the tile is one bit per element in accumulator order:
  // word a / 2 of a lane, bit (a & 1) 16 + 4 b + r for block (a, b), register r.
  const int lcol = lane & 15, lrow4 = (lane >> 4) * 4;
  if constexpr (EPI == EPI_WGRAD || EPI == EPI_LOGITS) {
    // fp32 results straight from the accumulators (64 contiguous bytes per row and quarter-wavefront):
    // this piece's partial of the tile, or the logits with their bias
    float* const outf = g.outf + (EPI == EPI_WGRAD ? (size_t)zsplit * g.split_stride : (size_t)0) +
                        (size_t)(m0 + wm * 128 + lrow4) * g.ldof + n0 + wn * 64 + lcol;
    float bv[4] = {0.f, 0.f, 0.f, 0.f};
    if (EPI == EPI_LOGITS) {
      const float* bias = g.bias + (size_t)slot * g.bias_slot_stride;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int n = n0 + wn * 64 + b * 16 + lcol;
        bv[b] = n < g.n_valid ? bias[n] : 0.f;
      }
    }
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr)
#pragma unroll
        for (int b = 0; b < 4; ++b) outf[(size_t)(a * 16 + rr) * g.ldof + b * 16] = acc[a][b][rr] + bv[b];
    if (!kRuns || sk_u >= sk_end) break;
    continue;
  }
  const float* bias = nullptr;
  if (EPI == EPI_RELU) bias = g.bias + (size_t)slot * g.bias_slot_stride;
  uint32_t mbits[4] = {0u, 0u, 0u, 0u};
  uint32_t* const mbits_at =
      g.maskbits ? g.maskbits + ((((size_t)(m0 / TM3) * g.nt + n0 / TN3) * 8 + wave) * 64 + lane) * 4 : nullptr;
  if (EPI == EPI_DGRAD && mbits_at) {
    const uint4 q = *(const uint4*)mbits_at;
    mbits[0] = q.x; mbits[1] = q.y; mbits[2] = q.z; mbits[3] = q.w;
  }
  uint16_t* const sT = smem + wave * (2 * 64 * kEpiPitch3);     // [64 n][72]
  uint16_t* const sN = sT + 64 * kEpiPitch3;                    // [64 m][72]
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    float cs[4] = {0.f, 0.f, 0.f, 0.f};   // EPI_DGRAD: column sums over this half's 64 rows
    if (EPI == EPI_DGRAD && !mbits_at) {
      // the ReLU mask of this half, H_l^T [64 n][64 m], fetched as whole 128-byte rows into sT;
      // every lane later replaces the 4 entries it read by its 4 results
      const int mrow = m0 + wm * 128 + half * 64, ncol = n0 + wn * 64;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int q = lane + 64 * i, r = q >> 3, ch = (q & 7) * 8;
        *(uint4*)&sT[r * kEpiPitch3 + ch] = *(const uint4*)(g.maskT + (size_t)(ncol + r) * g.ldmaskT + mrow + ch);
      }
    }
#pragma unroll
    for (int ah = 0; ah < 4; ++ah) {
      const int a = half * 4 + ah;
      const int ml = ah * 16 + lrow4;                           // first of this lane's 4 rows inside the half
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int nl = b * 16 + lcol;
        const int n = n0 + wn * 64 + nl;
        float bv = 0.f;
        if (EPI == EPI_RELU) bv = n < g.n_valid ? bias[n] : 0.f;
        uint2 hm = make_uint2(0, 0);
        if (EPI == EPI_DGRAD && !mbits_at) hm = *(const uint2*)&sT[nl * kEpiPitch3 + ml];
        uint16_t h[4];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const int bit = (a & 1) * 16 + b * 4 + rr;
          float v = acc[a][b][rr];
          if (EPI == EPI_RELU) {
            v = fmaxf(v + bv, 0.f);
            // (the mask is taken from the narrowed value, as the transposed copy would give it)
            if ((f32_to_bf16(v) & 0x7FFFu) != 0) mbits[a >> 1] |= 1u << bit;
          } else {
            const uint32_t pair = rr < 2 ? hm.x : hm.y;
            const bool pass = mbits_at ? ((mbits[a >> 1] >> bit) & 1u) != 0
                                       : ((pair >> ((rr & 1) * 16)) & 0x7FFFu) != 0;
            v = pass ? v : 0.f;
          }
          h[rr] = f32_to_bf16(v);
          if (EPI == EPI_DGRAD) cs[b] += __uint_as_float((uint32_t)h[rr] << 16);
        }
        uint2 o;
        o.x = h[0] | ((uint32_t)h[1] << 16);
        o.y = h[2] | ((uint32_t)h[3] << 16);
        *(uint2*)&sT[nl * kEpiPitch3 + ml] = o;
        if (g.out) {
          // row-major staging in 4-byte pieces: neighbouring lanes hold neighbouring columns of the same
          // 4 rows; the even lane takes rows 0-1 of the pair of columns, the odd lane rows 2-3 (half the
          // LDS writes of one 2-byte write per element: a round 0.7 % faster)
          const bool odd = lane & 1;
          const uint32_t send = odd ? o.x : o.y;
          const uint32_t recv = (uint32_t)__builtin_amdgcn_mov_dpp((int)send, 0xB1, 0xF, 0xF, true);   // lane ^ 1
          const uint32_t w0 = odd ? ((recv & 0xFFFFu) | (o.y << 16)) : ((o.x & 0xFFFFu) | (recv << 16));
          const uint32_t w1 = odd ? ((recv >> 16) | (o.y & 0xFFFF0000u)) : ((o.x >> 16) | (recv & 0xFFFF0000u));
          uint16_t* const q = &sN[(ml + (odd ? 2 : 0)) * kEpiPitch3 + (nl & ~1)];
          *(uint32_t*)q = w0;
          *(uint32_t*)(q + kEpiPitch3) = w1;
        }
      }
    }
    if (EPI == EPI_DGRAD) {
      // the bias gradient's share of these 64 rows (the four quarter-wavefronts hold rows 4 q .. 4 q + 3 of every 16)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        float c = cs[b] + __shfl_xor(cs[b], 16, 64);
        c += __shfl_xor(c, 32, 64);
        if (lane < 16)
          g.colsum[(size_t)((m0 + wm * 128 + half * 64) >> 6) * g.ldcs + n0 + wn * 64 + b * 16 + lcol] = c;
      }
    }
    {
      const int mrow = m0 + wm * 128 + half * 64, ncol = n0 + wn * 64;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int q = lane + 64 * i, r = q >> 3, ch = (q & 7) * 8;
        const uint4 vt = *(const uint4*)&sT[r * kEpiPitch3 + ch];
        store16_stream(g.outT + (size_t)(ncol + r) * g.ldoT + mrow + ch, vt, g.stream_out != 0);
        if (g.out) {
          const uint4 vn = *(const uint4*)&sN[r * kEpiPitch3 + ch];
          store16_stream(g.out + (size_t)(mrow + r) * g.ldo + ncol + ch, vn, g.stream_out != 0);
        }
      }
    }
  }
  if (EPI == EPI_RELU && mbits_at) *(uint4*)mbits_at = make_uint4(mbits[0], mbits[1], mbits[2], mbits[3]);
  break;
  }
}

// ------------------------------------------------------------------ output layer: logits, loss, dZ_L
// The last layer's product, the softmax cross-entropy and the output gradient in one kernel: the
// class count is at most 256, so a workgroup that owns 128 stacked rows owns their whole logit rows
// and nothing of Z_L ever goes to memory.  The product is narrow (few classes) and long (the last
// hidden width): what bounds it is how many bytes a CU keeps in flight, so the 64-wide k-steps of
// the A tile (128 rows of H_{L-1}) and the B tile (all classes of W_L^T) go from global memory
// straight into a ring of LDS stages (global_load_lds_dwordx4, swizzled on the global side as in the
// large-tile GEMM), kStages - 1 steps ahead of their use, one barrier per step.  Wavefront w owns
// rows 32 w .. 32 w + 31 and all classes, and multiplies the other way round - W_L^T is the
// MFMA's row operand, the activations its column operand - so that the 32x32 blocks hold Z_L^T:
// accumulator register r of lane l is class 32 b + 8 (r / 4) + 4 (l / 32) + r % 4 of row l % 32.
// All classes of a row then sit in the registers of two lanes (l and l + 32), and its softmax is
// arithmetic inside a lane plus one exchange, instead of a 32-lane reduction per row and class.
// Outputs: dZ_L = c_k (softmax - onehot) narrowed to bf16 (zero in padding rows and classes) in
// both orientations, the 128 rows' loss sum, and the column sums of the narrowed dZ_L (the bias
// gradient's share of these rows).
constexpr int kCeRows = 128;             // stacked rows per workgroup of the output-layer kernel

struct LogitsCeArgs {
  const uint16_t* H; size_t ldh;         // H_{L-1} [rows][ldh]
  int ksteps;                            // dp_{L-1} / 64
  const uint16_t* Wt; size_t ldw;        // W_L^T [dp_L][ldw] inside a shadow slot
  size_t w_slot_stride;
  const float* bias; size_t bias_slot_stride;
  int C;                                 // classes (columns >= C are padding)
  int rows_per_upload, by_upload;
  const int32_t* label;                  // -1: padding row
  uint16_t* dZ; size_t lddz;             // [rows][lddz]
  uint16_t* dZT; size_t lddzt;           // [dp_L][lddzt]
  float* rowloss;                        // [rows / 128]
  float* colsum; size_t ldcs;            // [rows / 128][ldcs]
};

__device__ __forceinline__ void lds_dma16_raw(const uint16_t* gsrc, uint16_t* lds_block);

template <int NB>                        // dp_L = 32 NB: 2, 4 or 8
__global__ __launch_bounds__(256, 1) void mlp_logits_ce_kernel(LogitsCeArgs a, RoundDesc rd) {
  constexpr int NP = 32 * NB;            // padded class count
  constexpr int kStageElems = (kCeRows + NP) * BK;
  constexpr int kStages = NB == 8 ? 3 : 4;
  constexpr int kPitchD = NP + 8;        // narrowed dZ tile, bf16 [128][kPitchD], after the main loop ...
  constexpr int kPitchT = kCeRows + 8;   // ... and its transpose, bf16 [NP][kPitchT], behind it
  static_assert(kStages * kStageElems >= kCeRows * kPitchD + NP * kPitchT, "staging fits the ring");
  static_assert(kStages * kStageElems * 2 <= 150 * 1024, "LDS budget");
  constexpr int kDmaPerWave = 4 + NB;    // requests per wavefront and stage (8 rows of 128 bytes each)
  __shared__ __attribute__((aligned(16))) uint16_t smem[kStages * kStageElems];
  __shared__ float s_l[4];
  __shared__ __attribute__((aligned(16))) float s_bias[NP];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int m0 = blockIdx.x * kCeRows;
  const int up = m0 / a.rows_per_upload;
  const uint32_t slot = a.by_upload ? (uint32_t)up : rd.w[up].slot;
  const float coef = rd.w[up].c;
  const uint16_t* Wt = a.Wt + (size_t)slot * a.w_slot_stride;

  // requests of this wavefront: its own 32 rows of A (4 requests) and NP / 4 rows of B (NB requests);
  // lane l of a request fills position l & 7 of row r8 + (l >> 3) with chunk (l & 7) ^ ((row >> 1) & 7)
  const int lr = lane >> 3, lp = lane & 7;
  const uint16_t* ga[4]; const uint16_t* gb[NB];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = wave * 32 + 8 * i + lr;
    ga[i] = a.H + (size_t)(m0 + row) * a.ldh + ((lp ^ ((row >> 1) & 7)) << 3);
  }
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int row = wave * (NP / 4) + 8 * i + lr;
    gb[i] = Wt + (size_t)row * a.ldw + ((lp ^ ((row >> 1) & 7)) << 3);
  }
  uint16_t* const dmaA = smem + (wave * 32) * BK;
  uint16_t* const dmaB = smem + kCeRows * BK + (wave * (NP / 4)) * BK;
#define ABS_CE_DMA(ks_)                                                            \
  {                                                                                \
    const int k0_ = (ks_) * BK;                                                    \
    uint16_t* st_ = smem + ((ks_) % kStages) * kStageElems;                        \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                  \
      lds_dma16_raw(ga[i] + k0_, st_ + (dmaA - smem) + i * 512);                   \
    _Pragma("unroll") for (int i = 0; i < NB; ++i)                                 \
      lds_dma16_raw(gb[i] + k0_, st_ + (dmaB - smem) + i * 512);                   \
  }
  f32x16_t acc[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
  const int l32 = lane & 31, lk = lane >> 5;
  const int sw = (l32 >> 1) & 7;
  const int fa_row = (wave * 32 + l32) * BK, fb_row = kCeRows * BK + l32 * BK;
  const int nk = a.ksteps;
  // what the epilogue needs from memory is requested before the main loop: the label of the lane's
  // row, and the biases, which wait in LDS (padding classes: -inf, so they drop out of max and sum)
  const int lab = a.label[m0 + wave * 32 + l32];
  if (t < NP) s_bias[t] = t < a.C ? (a.bias + (size_t)slot * a.bias_slot_stride)[t] : -INFINITY;
#pragma unroll
  for (int st = 0; st < kStages - 1; ++st)
    if (st < nk) ABS_CE_DMA(st);
  for (int ks = 0; ks < nk; ++ks) {
    // this wavefront's requests of step ks have landed once at most those of the steps behind it
    // (kStages - 2 of them, kDmaPerWave requests each) are still in flight; near the end: all
    if (ks + kStages - 2 < nk) __builtin_amdgcn_s_waitcnt(0x0F70 | (((kStages - 2) * kDmaPerWave) & 15) |
                                                          ((((kStages - 2) * kDmaPerWave) >> 4) << 14));
    else                       __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();                     // everybody's part of step ks is in LDS; everybody is done with step ks - 1
    if (ks + kStages - 1 < nk) ABS_CE_DMA(ks + kStages - 1);
    const uint16_t* sS = smem + (ks % kStages) * kStageElems;
    // fragments of sub-step s + 1 are read while the MFMAs of sub-step s run
    bf16x8_t fa[2], fb[2][NB];
#define ABS_CE_FRAGS(set, s_)                                                      \
  {                                                                                \
    const int ch_ = ((((s_) << 1) | lk) ^ sw) << 3;                                \
    fa[set] = *(const bf16x8_t*)&sS[fa_row + ch_];                                 \
    _Pragma("unroll") for (int b = 0; b < NB; ++b)                                 \
      fb[set][b] = *(const bf16x8_t*)&sS[fb_row + b * 32 * BK + ch_];              \
  }
    ABS_CE_FRAGS(0, 0);
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      if (sub < 3) ABS_CE_FRAGS((sub + 1) & 1, sub + 1);
#pragma unroll
      for (int b = 0; b < NB; ++b)
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[sub & 1][b], fa[sub & 1], acc[b], 0, 0, 0);
    }
#undef ABS_CE_FRAGS
    // issue order: the first fragment set, then per sub-step one read ahead and one read behind each MFMA
    __builtin_amdgcn_sched_group_barrier(0x100, 1 + NB, 0);
#pragma unroll
    for (int sub = 0; sub < 3; ++sub) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    }
    __builtin_amdgcn_sched_group_barrier(0x008, NB, 0);
  }
#undef ABS_CE_DMA
  __syncthreads();                       // all fragment reads done before the ring is reused for staging

  // ---- softmax cross-entropy: the lane's 16 NB classes of row l % 32, its partner holds the rest
  uint16_t* const sD = smem;             // [128][kPitchD]
  uint16_t* const sT = smem + kCeRows * kPitchD;       // [NP][kPitchT]
  const int ml = wave * 32 + l32;
  float zmax = -INFINITY;
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 bq = *(const float4*)&s_bias[b * 32 + q * 8 + lk * 4];
      acc[b][q * 4 + 0] += bq.x; acc[b][q * 4 + 1] += bq.y; acc[b][q * 4 + 2] += bq.z; acc[b][q * 4 + 3] += bq.w;
#pragma unroll
      for (int e = 0; e < 4; ++e) zmax = fmaxf(zmax, acc[b][q * 4 + e]);
    }
  zmax = fmaxf(zmax, __shfl_xor(zmax, 32, 64));
  const int lrel = lab - lk * 4;         // the label relative to this half's class offset
  float ssum = 0.f, zy = 0.f;
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float dz = acc[b][r] - zmax;
      zy = (b * 32 + (r >> 2) * 8 + (r & 3) == lrel) ? dz : zy;
      acc[b][r] = __expf(dz);
      ssum += acc[b][r];
    }
  ssum += __shfl_xor(ssum, 32, 64);
  zy += __shfl_xor(zy, 32, 64);
  float lsum = lab >= 0 ? logf(ssum) - zy : 0.f;       // this row's loss (same in both of its lanes)
  const float cr = lab >= 0 ? coef : 0.f;              // c_k (softmax - onehot), zero for padding rows
  const float scale = cr / ssum;
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      uint16_t h[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float v = acc[b][q * 4 + e] * scale - ((b * 32 + q * 8 + e == lrel) ? cr : 0.f);
        h[e] = __builtin_bit_cast(uint16_t, (__bf16)v);
        sT[(b * 32 + q * 8 + lk * 4 + e) * kPitchT + ml] = h[e];       // (32 lanes: 64 contiguous bytes)
      }
      uint2 o;
      o.x = h[0] | ((uint32_t)h[1] << 16);
      o.y = h[2] | ((uint32_t)h[3] << 16);
      *(uint2*)&sD[ml * kPitchD + b * 32 + q * 8 + lk * 4] = o;
    }
  // the 32 rows of the wavefront (lanes of a half), then the four wavefronts, always in this order
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) lsum += __shfl_xor(lsum, o, 64);
  if (lane == 0) s_l[wave] = lsum;
  __syncthreads();
  if (t == 0) a.rowloss[blockIdx.x] = (s_l[0] + s_l[1]) + (s_l[2] + s_l[3]);
  // row-major copy: 16-byte pieces, NP / 8 per row
  for (int q = t; q < kCeRows * (NP / 8); q += 256) {
    const int row = q / (NP / 8), ch = q % (NP / 8);
    *(uint4*)(a.dZ + (size_t)(m0 + row) * a.lddz + ch * 8) = *(const uint4*)&sD[row * kPitchD + ch * 8];
  }
  // transposed copy: class n, 16-byte pieces of 8 consecutive rows
  for (int q = t; q < NP * (kCeRows / 8); q += 256) {
    const int n = q / (kCeRows / 8), rb8 = (q % (kCeRows / 8)) * 8;
    *(uint4*)(a.dZT + (size_t)n * a.lddzt + m0 + rb8) = *(const uint4*)&sT[n * kPitchT + rb8];
  }
  // the bias gradient's share of these 128 rows: class n's narrowed values added in row order
  for (int n = t; n < NP; n += 256) {
    float c = 0.f;
#pragma unroll 4
    for (int p8 = 0; p8 < kCeRows / 8; ++p8) {
      const uint4 v = *(const uint4*)&sT[n * kPitchT + p8 * 8];
      c += __uint_as_float(v.x << 16); c += __uint_as_float(v.x & 0xFFFF0000u);
      c += __uint_as_float(v.y << 16); c += __uint_as_float(v.y & 0xFFFF0000u);
      c += __uint_as_float(v.z << 16); c += __uint_as_float(v.z & 0xFFFF0000u);
      c += __uint_as_float(v.w << 16); c += __uint_as_float(v.w & 0xFFFF0000u);
    }
    a.colsum[(size_t)blockIdx.x * a.ldcs + n] = c;
  }
}

// ------------------------------------------------------------------ update + snapshot
// The update as a kernel of its own (a TileUpdate for a whole matrix): local SGD, the averaged change of
// the uploads, matrices whose rows are not 16-byte aligned, a round's last layer, the bf16 copies of w^0.
struct UpdateArgs : TileUpdate {
  // batched form (local SGD): blockIdx.z = upload a; partial a, nsplit = 1, the model read from
  // slot cur_index[a] of w_cur's ring and written to slot a of w_next's ring / shadow ring
  int batched;
  size_t cur_stride, next_stride, shadow_stride;
  uint16_t cur_index[ABS_MAX_WORKERS];
};
__device__ __forceinline__ void update_select_upload(UpdateArgs& u) {
  if (!u.batched) return;
  const int a = blockIdx.z;
  u.partial += (size_t)a * u.split_stride;
  u.w_cur += (size_t)u.cur_index[a] * u.cur_stride;
  u.w_next += (size_t)a * u.next_stride;
  if (u.wn) u.wn += (size_t)a * u.shadow_stride;
  u.wt += (size_t)a * u.shadow_stride;
}
template <int TJ>
__global__ __launch_bounds__(256) void mlp_update_kernel(UpdateArgs u) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[64 * (TJ + 2)];
  update_select_upload(u);
  update_block64<256, TJ>(u, blockIdx.y * 64, blockIdx.x * TJ, tile);
}

// Element-wise version for narrow or odd output widths (e.g. the 10-class output layer):
// one thread per weight, four partial loads in flight.
__global__ __launch_bounds__(256) void mlp_update_small_kernel(UpdateArgs u) {
  update_select_upload(u);
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= u.d_in * u.d_out) return;
  const int i = e / u.d_out, j = e - i * u.d_out;
  const float* pp = u.partial + (size_t)i * u.ldp + j;
  float G = 0.f;
  int z = 0;
  for (; z + 4 <= u.nsplit; z += 4) {
    float v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = pp[(size_t)(z + q) * u.split_stride];
#pragma unroll
    for (int q = 0; q < 4; ++q) G += v[q];
  }
  for (; z < u.nsplit; ++z) G += pp[(size_t)z * u.split_stride];
  const float wnew = u.w_cur[e] - G;
  u.w_next[e] = wnew;
  const uint16_t h = f32_to_bf16(wnew);
  if (u.wn) u.wn[(size_t)i * u.ldwn + j] = h;
  u.wt[(size_t)j * u.ldwt + i] = h;
}

// The bias update as a launch of its own.  Global form: all `prow[l]` blocks, model w_cur -> w_next.
// Per-upload form (local SGD, blockIdx.y = upload a): the blocks of a's own rows, model slot
// cur_index[a] of w_cur -> slot a of w_next.
struct BiasArgs : BiasCore {
  int batched;
  size_t cur_stride, next_stride;
  uint16_t cur_index[ABS_MAX_WORKERS];
};
__global__ __launch_bounds__(256) void mlp_bias_kernel(BiasArgs a) {
  __shared__ float s_part[16 * 17];
  const int up = blockIdx.y;
  const float* cur = a.w_cur + (a.batched ? (size_t)a.cur_index[up] * a.cur_stride : 0);
  float* nxt = a.w_next + (a.batched ? (size_t)up * a.next_stride : 0);
  bias_block(a, blockIdx.x, [&](int l) { return a.batched ? up * a.prow[l] : 0; }, cur, nxt, s_part);
}

// Local SGD: the uploads' mean minibatch losses of one local step, one thread per upload over the
// loss sums of its `nb` row blocks; lossacc carries the sum over the job's steps and the last step
// publishes the job's average local loss (worker part of Algorithm 1).  (With U = 1 the first
// workgroup of the input-gradient kernel publishes: publish_upload_losses.)
__global__ __launch_bounds__(128) void mlp_loss_kernel(const float* rowloss, int B, int nb, int K, uint32_t stamp,
                                                       LossMailbox* mailbox, float* lossacc, int first, int last,
                                                       int U) {
  __shared__ float s_loss[ABS_MAX_WORKERS];
  const int up = threadIdx.x;
  if (up < K) {
    float s = 0.f;
    for (int q = 0; q < nb; ++q) s += rowloss[(size_t)up * nb + q];
    s /= (float)B;
    s += first ? 0.f : lossacc[up];
    lossacc[up] = s;
    s_loss[up] = s / (float)U;
  }
  __syncthreads();
  if (last) publish_losses(mailbox, s_loss, K, stamp);
}

// ------------------------------------------------------------------ local SGD helpers
// Eq. 3 over the uploads: D = (1/K) sum_a (w^{t - tau_a} - w_a^{U}) in arrival order, for every
// parameter; bias entries are applied right away, weight matrices go through the update kernels
// (which also refresh the bf16 copies).
struct DeltaArgs {
  const float* ring; size_t slot_stride;
  const float* priv;
  float* D;
  size_t P;
  int L;
  size_t b_off[ABS_MAX_LAYERS]; int b_len[ABS_MAX_LAYERS];
  const float* w_cur; float* w_next;
};
__global__ __launch_bounds__(256) void mlp_delta_kernel(DeltaArgs a, RoundDesc rd) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= a.P) return;
  float s = 0.f;
  for (int up = 0; up < rd.K; ++up)
    s += a.ring[(size_t)rd.w[up].slot * a.slot_stride + i] - a.priv[(size_t)up * a.slot_stride + i];
  const float d = s / (float)rd.K;
  a.D[i] = d;
  for (int l = 0; l < a.L; ++l)
    if (i >= a.b_off[l] && i < a.b_off[l] + (size_t)a.b_len[l]) a.w_next[i] = a.w_cur[i] - d;
}

__global__ void mlp_fill_zero_kernel(uint4* p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t step = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += step) p[i] = make_uint4(0, 0, 0, 0);
}

// ------------------------------------------------------------------ held-out evaluation
// Sequential evaluation rows row0 .. row0 + n in the index arrays of the forward pass; the
// padding rows read a valid row and carry label -1.
__global__ void mlp_eval_index_kernel(uint32_t* rowidx, int32_t* label, const int32_t* y, int64_t row0, int n,
                                      int rows) {
  const int m = blockIdx.x * blockDim.x + threadIdx.x;
  if (m >= rows) return;
  rowidx[m] = (uint32_t)(row0 + (m < n ? m : 0));
  label[m] = m < n ? y[row0 + m] : -1;
}

// One wavefront per row of the logits: -log softmax(z)_y and whether the first largest logit
// is the label.  NC = logits width / 64.
template <int NC>
__global__ __launch_bounds__(256) void mlp_eval_rows_kernel(const float* Z, size_t ldz, int C, const int32_t* label,
                                                            int n, float* rowloss, float* correct) {
  const int lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= n) return;
  const int lab = label[m];
  float z[NC], zmax = -INFINITY;
  int best = 0;
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const int c = lane + 64 * q;
    z[q] = c < C ? Z[(size_t)m * ldz + c] : -INFINITY;
    if (z[q] > zmax) { zmax = z[q]; best = c; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {            // largest value, lowest class among equals
    const float ov = __shfl_xor(zmax, o, 64);
    const int ob = __shfl_xor(best, o, 64);
    if (ov > zmax || (ov == zmax && ob < best)) { zmax = ov; best = ob; }
  }
  float ssum = 0.f, zy = 0.f;
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const int c = lane + 64 * q;
    if (c == lab) zy = z[q] - zmax;
    ssum += c < C ? expf(z[q] - zmax) : 0.f;
  }
  ssum = wave_sum(ssum);
  zy = wave_sum(zy);
  if (lane == 0) { rowloss[m] = logf(ssum) - zy; correct[m] = best == lab ? 1.f : 0.f; }
}

template <typename T>
T* at(const MlpArgs& a, size_t off) { return (T*)(a.ws + off); }

// Number of row-range splits of a weight-gradient contraction.  `slots` workgroups run at
// once; a split costs one k-step time per step of its range and every extra split adds a
// partial tile to write and read back.  Picks the cheapest under that model.
int pick_split(int tiles, int ksteps, int slots, double tile_bytes) {
  const double step_us = 2.0, bytes_per_us = 3.0e6;
  int best = 1;
  double best_cost = 1e300;
  for (int z = 1; z <= std::min(ksteps, kMaxSplit); ++z) {
    const int rounds = (tiles * z + slots - 1) / slots;
    const int steps = (ksteps + z - 1) / z;
    const double cost = rounds * steps * step_us * (tile_bytes / (256.0 * 256 * 4)) +
                        (double)z * tiles * tile_bytes * 2.0 / bytes_per_us;
    if (cost < best_cost) { best_cost = cost; best = z; }
  }
  return best;
}

// Row-range splits of layer l's weight-gradient contraction over `rows` stacked rows
// (per_upload > 0: local SGD, one split per upload).
int wgrad_split(const MlpPlan& p, int l, int rows, int per_upload) {
  if (per_upload > 0) return per_upload;
  const int ksteps = rows / BK;
  const int tn = p.dp[l + 1] % 256 == 0 ? 256 : p.dp[l + 1] % 128 == 0 ? 128 : 64;
  const bool big = p.dp[l] % TM3 == 0 && p.dp[l + 1] % TN3 == 0;
  const int tiles = big ? (p.dp[l] / TM3) * (p.dp[l + 1] / TN3) : (p.dp[l] / TM) * (p.dp[l + 1] / tn);
  return big ? pick_split(tiles, ksteps, 256, 256.0 * 256 * 4) : pick_split(tiles, ksteps, 512, 128.0 * tn * 4);
}

}  // namespace

// ------------------------------------------------------------------ planning
bool mlp_plan(const abs_config& c, MlpPlan& p, const char** why) {
  p = MlpPlan{};
  const int L = c.n_layers;
  if (c.dims[0] % 8) { *why = "MLP: d_0 must be a multiple of 8"; return false; }
  if (c.dims[L] < 2 || c.dims[L] > 256) { *why = "MLP: 2 <= d_L <= 256"; return false; }
  for (int l = 0; l <= L; ++l)
    if (c.dims[l] < 1 || c.dims[l] > 16384) { *why = "MLP: layer widths must be in [1, 16384]"; return false; }
  p.L = L;
  for (int l = 0; l <= L; ++l) {
    p.d[l] = c.dims[l];
    p.dp[l] = (int)round_up((size_t)c.dims[l], 128);
  }
  if (c.dims[L] <= 64) p.dp[L] = 64;
  for (int l = 0; l <= L; ++l) p.ld[l] = p.dp[l] + kPitchPad;
  p.U = c.U > 1 ? c.U : 1;
  p.B = c.B;
  p.Bp = (int)round_up((size_t)c.B, TM);
  p.N = c.N;
  p.Mp = c.N * p.Bp;
  p.ldm = (size_t)p.Mp + kPitchPad;
  p.R = c.tau_cap + 3;
  size_t o = 0;
  for (int l = 0; l < L; ++l) {
    p.w_off[l] = o; o += (size_t)p.d[l] * p.d[l + 1];
    p.b_off[l] = o; o += (size_t)p.d[l + 1];
  }
  p.P = o;
  p.slot_stride = round_up(p.P, 64);
  o = 0;
  for (int l = 0; l < L; ++l) {
    p.wt_off[l] = o; o += (size_t)p.dp[l + 1] * p.ld[l];
    p.wn_off[l] = o; if (l >= 1) o += (size_t)p.dp[l] * p.ld[l + 1];
  }
  p.shadow_stride = round_up(o, 128);
  size_t b = 0;
  auto take = [&](size_t bytes) { size_t at = b; b = round_up(b + bytes, 256); return at; };
  const size_t Mp = (size_t)p.Mp;
  p.off_ring = take((size_t)p.R * p.slot_stride * 4);
  p.off_shadow = take((size_t)p.R * p.shadow_stride * 2);
  p.off_rowidx = take(Mp * 4);
  p.off_label = take(Mp * 4);
  p.off_xgt = take((size_t)p.dp[0] * p.ldm * 2);
  for (int l = 1; l < L; ++l) {
    p.off_h[l] = take(Mp * p.ld[l] * 2);
    p.off_ht[l] = take(p.ldm * p.dp[l] * 2);
  }
  p.off_z = take(Mp * p.dp[L] * 4);
  for (int l = 1; l <= L; ++l) {
    p.off_dz[l] = take(Mp * p.ld[l] * 2);
    p.off_dzt[l] = take(p.ldm * p.dp[l] * 2);
  }
  p.off_rowloss = take(Mp * 4);
  for (int l = 1; l <= L; ++l) p.off_colsum[l] = take(Mp / (l == L ? kCeRows : 64) * p.dp[l] * 4);
  for (int l = 1; l < L; ++l) p.off_maskbits[l] = take(round_up(Mp, 256) * round_up((size_t)p.dp[l], 256) / 8);
  for (int l = 0; l < L; ++l)
    p.off_partial[l] = take((size_t)p.dp[l] * (p.dp[l + 1] + kPartialPad) * 4 *
                            (p.U > 1 ? std::max<size_t>(kMaxSplit, (size_t)c.N) : (size_t)kMaxSplit));
  if (p.U > 1) {
    p.off_priv = take((size_t)c.N * p.slot_stride * 4);
    p.off_priv_shadow = take((size_t)c.N * p.shadow_stride * 2);
    p.off_lossacc = take((size_t)c.N * 4);
    p.off_delta = take(p.slot_stride * 4);
  }
  p.off_eval = take(eval_scratch_bytes((size_t)p.Mp));
  p.total = b;
  return true;
}

// ------------------------------------------------------------------ launches
namespace {

// Plan recording: with t_plan set, the launch functions below append what they would launch
// (kernel, tile shape, split count) and launch nothing; mlp_round_plan() uses it so that the
// description of a round's launches comes from the very code that issues them.
thread_local std::string* t_plan = nullptr;
#define ABS_LAUNCH(...) do { if (!t_plan) { __VA_ARGS__; } } while (0)
// A round's kernels carry their own start / stop events when the round is timed: kbegin() asks the
// hook for the pair, the next ABS_LAUNCH_K attaches it to its dispatch (null events: a plain launch).
thread_local hipEvent_t t_ev0 = nullptr, t_ev1 = nullptr;
void kbegin(LaunchHook* hook, int kind, double flops, double bytes) { hook->begin_kernel(kind, flops, bytes, &t_ev0, &t_ev1); }
void kend(LaunchHook* hook, int kind) { hook->end_kernel(kind); t_ev0 = t_ev1 = nullptr; }
#define ABS_LAUNCH_K(kernel, grid, block, stream, ...)                                                    \
  do {                                                                                                    \
    if (!t_plan) hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, t_ev0, t_ev1, 0, __VA_ARGS__);     \
  } while (0)
void plan_note(const char* what, int a, int b, int c) {
  if (t_plan) *t_plan += std::string(what) + ":" + std::to_string(a) + "x" + std::to_string(b) + "/" + std::to_string(c) + " ";
}

struct NullHook : LaunchHook {
  void begin(int, double, double) override {}
  void end(int) override {}
};

// The three uses of the update kernels:
//   UPD_GLOBAL  w^{t+1} = w^t - sum of the split partials                    (U = 1, Eq. 3)
//   UPD_LOCAL   private model of upload a <- its model - its own partial     (Eq. 2, step u)
//   UPD_DELTA   w^{t+1} = w^t - D, D = the averaged change of the uploads    (U > 1, Eq. 3)
// each also writes the bf16 copies of what it produced.
enum { UPD_GLOBAL = 0, UPD_LOCAL = 1, UPD_DELTA = 2 };
// Weight gradient of layer l over `rows` stacked rows on the 256 x 256 tile kernel: k-steps per run if
// the contraction should be cut into equal runs across the tiles (GemmArgs::sk_q), else 0.  Runs pay
// when equal row ranges per tile leave a good part of the CUs idle in the launch's last wave and a
// run is still long enough to amortise a tile's epilogue; a tile then gets up to *max_parts partials.
int wgrad_runs(const MlpPlan& p, int l, int rows, int nsplit, int* max_parts) {
  constexpr int kCUs = 256, kMinRun = 24;
  if (p.dp[l] % TM3 || p.dp[l + 1] % TN3 || p.d[l + 1] % 4 || p.w_off[l] % 4) return 0;   // (the tiled update kernels read the per-tile counts)
  const int tiles = (p.dp[l] / TM3) * (p.dp[l + 1] / TN3), ksteps = rows / BK;
  const int wgs = tiles * nsplit;
  if (wgs < 128) return 0;                                   // (not a launch of the large-tile kernel)
  const int waves = (wgs + kCUs - 1) / kCUs;
  if ((double)wgs / (waves * kCUs) >= 0.9) return 0;         // equal ranges already fill the CUs
  const long units = (long)tiles * ksteps;
  const int q = (int)((units + kCUs - 1) / kCUs);            // one run per CU
  if (q < kMinRun) return 0;
  const int parts = (ksteps + q - 1) / q + 1;
  if (parts > kMaxSplit) return 0;
  *max_parts = parts;
  return q;
}

// Eq. 3 for layer l's weight matrix from the split partials of its weight gradient (U = 1).
TileUpdate global_update_args(const MlpArgs& a, int l, const RoundDesc& rd, int nsplit) {
  const MlpPlan& p = a.plan;
  float* ring = at<float>(a, p.off_ring);
  uint16_t* shadow = at<uint16_t>(a, p.off_shadow) + (size_t)rd.slot_next * p.shadow_stride;
  TileUpdate u{};
  u.partial = at<float>(a, p.off_partial[l]);
  u.split_stride = (size_t)p.dp[l] * (p.dp[l + 1] + kPartialPad);
  u.ldp = (size_t)p.dp[l + 1] + kPartialPad;
  u.nsplit = nsplit;
  u.w_cur = ring + (size_t)rd.slot_cur * p.slot_stride + p.w_off[l];
  u.w_next = ring + (size_t)rd.slot_next * p.slot_stride + p.w_off[l];
  u.d_in = p.d[l];
  u.d_out = p.d[l + 1];
  u.wn = l >= 1 ? shadow + p.wn_off[l] : nullptr; u.ldwn = (size_t)p.ld[l + 1];
  u.wt = shadow + p.wt_off[l]; u.ldwt = (size_t)p.ld[l];
  return u;
}
// Whether the rows of layer l's fp32 weight matrix can be moved 16 bytes at a time.
bool update_rows_aligned(const MlpPlan& p, int l) { return p.d[l + 1] % 4 == 0 && p.w_off[l] % 4 == 0; }

void launch_update(const MlpArgs& a, int l, const RoundDesc& rd, int mode, int step, int nsplit,
                   hipStream_t s, LaunchHook* hook, int run_q = 0, int run_ksteps = 0) {
  const MlpPlan& p = a.plan;
  float* ring = at<float>(a, p.off_ring);
  UpdateArgs u{};
  u.d_in = p.d[l];
  u.d_out = p.d[l + 1];
  u.ldwn = (size_t)p.ld[l + 1];
  u.ldwt = (size_t)p.ld[l];
  int batch = 1;
  if (mode == UPD_LOCAL) {
    float* priv = at<float>(a, p.off_priv);
    uint16_t* pshadow = at<uint16_t>(a, p.off_priv_shadow);
    u.batched = 1;
    batch = rd.K;
    u.partial = at<float>(a, p.off_partial[l]);
    u.split_stride = (size_t)p.dp[l] * (p.dp[l + 1] + kPartialPad);
    u.ldp = (size_t)p.dp[l + 1] + kPartialPad;
    u.nsplit = 1;
    u.w_cur = (step == 0 ? ring : priv) + p.w_off[l];
    u.cur_stride = p.slot_stride;
    for (int k = 0; k < rd.K; ++k) u.cur_index[k] = (uint16_t)(step == 0 ? rd.w[k].slot : (uint32_t)k);
    u.w_next = priv + p.w_off[l];
    u.next_stride = p.slot_stride;
    u.wn = l >= 1 ? pshadow + p.wn_off[l] : nullptr;
    u.wt = pshadow + p.wt_off[l];
    u.shadow_stride = p.shadow_stride;
  } else {
    uint16_t* shadow = at<uint16_t>(a, p.off_shadow) + (size_t)rd.slot_next * p.shadow_stride;
    if (mode == UPD_GLOBAL) {
      u.partial = at<float>(a, p.off_partial[l]);
      u.split_stride = (size_t)p.dp[l] * (p.dp[l + 1] + kPartialPad);
      u.ldp = (size_t)p.dp[l + 1] + kPartialPad;
      u.nsplit = nsplit;
    } else {
      u.partial = at<float>(a, p.off_delta) + p.w_off[l];
      u.split_stride = 0;
      u.ldp = (size_t)p.d[l + 1];
      u.nsplit = 1;
    }
    u.w_cur = ring + (size_t)rd.slot_cur * p.slot_stride + p.w_off[l];
    u.w_next = ring + (size_t)rd.slot_next * p.slot_stride + p.w_off[l];
    u.wn = l >= 1 ? shadow + p.wn_off[l] : nullptr;
    u.wt = shadow + p.wt_off[l];
  }
  if (run_q) { u.sk_q = run_q; u.sk_ksteps = run_ksteps; u.sk_nt = p.dp[l + 1] / TN3; }
  const double n = (double)p.d[l] * p.d[l + 1] * batch;
  kbegin(hook, KK_MLP_UPDATE, n * (u.nsplit + 1), n * (4.0 * (u.nsplit + 2) + (l >= 1 ? 4.0 : 2.0)));
  const dim3 block(256);
  const bool vec = update_rows_aligned(p, l);
  // wide tiles (fewer, longer stores) only where they still give every CU a workgroup
  const bool wide = p.d[l + 1] >= 256 && ((p.d[l + 1] + 255) / 256) * ((p.d[l] + 63) / 64) * batch >= 256;
  plan_note("update", 64, vec && wide ? 256 : vec ? 64 : 1, u.nsplit);
  if (vec && wide) ABS_LAUNCH_K((mlp_update_kernel<256>), dim3((p.d[l + 1] + 255) / 256, (p.d[l] + 63) / 64, batch), block, s, u);
  else if (vec) ABS_LAUNCH_K((mlp_update_kernel<64>), dim3((p.d[l + 1] + 63) / 64, (p.d[l] + 63) / 64, batch), block, s, u);
  else     ABS_LAUNCH_K(mlp_update_small_kernel, dim3((p.d[l] * p.d[l + 1] + 255) / 256, 1, batch), block, s, u);
  kend(hook, KK_MLP_UPDATE);
}

// Whether a product goes to the 256 x 256 tile kernel.
inline bool gemm_is_big(bool gather, bool per_upload, const GemmArgs& g, int Mdim, int Ndim, int nsplit) {
  return Mdim % TM3 == 0 && Ndim % TN3 == 0 && (!per_upload || g.rows_per_upload % TM3 == 0) &&
         (!gather || g.a_kvalid == g.ksteps_total * BK) && (Mdim / TM3) * (Ndim / TN3) * nsplit >= 128;
}

// Returns whether the product went to the 256 x 256 tile kernel (only that one knows maskbits).
template <int EPI, bool GATHER, bool PER_UPLOAD, int TAG = 0>
bool launch_gemm(GemmArgs g, const RoundDesc& rd, int Mdim, int Ndim, int nsplit, hipStream_t s) {
  g.nsplit = nsplit;
  const bool big = g.sk_q > 0 || gemm_is_big(GATHER, PER_UPLOAD, g, Mdim, Ndim, nsplit);
  if (TAG == 3 && !big) {      // the caller picks TAG 3 with this very test: only the large-tile kernel reads a transposed A
    std::fprintf(stderr, "libabs: transposed-A product outside the large-tile kernel\n");
    std::abort();
  }
  if (big && g.sk_q > 0) {
    // runs of sk_q k-steps across the tiles: one workgroup per run
    g.mt = Mdim / TM3;
    g.nt = Ndim / TN3;
    g.rows_per_xcd = 0;
    const int runs = (g.mt * g.nt * g.ksteps_total + g.sk_q - 1) / g.sk_q;
    plan_note(TAG == 2 ? "wgrad_x_runs" : "wgrad_runs", TM3, TN3, g.sk_q);
    ABS_LAUNCH_K((mlp_gemm256_kernel<EPI, GATHER, PER_UPLOAD, TAG>), dim3((runs + 7) / 8 * 8 + g.pig_blocks + g.bias_blocks), dim3(512), s, g, rd);
    return true;
  }
  if (big) {
    g.mt = Mdim / TM3;
    g.nt = Ndim / TN3;
    g.rows_per_xcd = (g.mt * nsplit + 7) / 8;
    // long products with outputs beyond the caches stream them out (short ones are bound by these very
    // stores and were slower for it: the output layer's input gradient 75 -> 79 us at 32768 rows; so was
    // the first layer's forward product, whose gathered rows come from memory anyway: 368 -> 374 us)
    g.stream_out = (EPI == EPI_RELU || EPI == EPI_DGRAD) && !GATHER && g.ksteps_total >= 16 &&
                   (size_t)Mdim * (size_t)Ndim * 2 >= ABS_STREAM_MIN_BYTES;
    plan_note(EPI == EPI_RELU ? (TAG == 3 ? "fwd_t" : "fwd") : EPI == EPI_LOGITS ? "logits" : EPI == EPI_DGRAD ? (TAG == 3 ? "dgrad_t" : "dgrad")
              : TAG == 2 ? "wgrad_x" : "wgrad", TM3, TN3, nsplit);
    ABS_LAUNCH_K((mlp_gemm256_kernel<EPI, GATHER, PER_UPLOAD, TAG>), dim3(8 * g.rows_per_xcd * g.nt + g.pig_blocks + g.bias_blocks), dim3(512), s, g, rd);
    return true;
  }
  // widest column tile that still fills the GPU: 256-wide tiles only with two workgroups per CU
  // (the kernel is built for two: one's loads cover the other's barriers), 128-wide with one
  int tn = 64;
  for (int cand : {256, 128}) {
    if (Ndim % cand) continue;
    const int need = cand == 256 ? 512 : 256;
    if ((Mdim / TM) * (Ndim / cand) * nsplit >= need || Ndim % (cand / 2)) { tn = cand; break; }
  }
  g.mt = Mdim / TM;
  g.nt = Ndim / tn;
  g.rows_per_xcd = (g.mt * nsplit + 7) / 8;
  const dim3 block(256);
  const dim3 grid1(8 * g.rows_per_xcd * g.nt + g.pig_blocks + g.bias_blocks, 1, 1);
  // DMA ring: whole k-steps only
  const bool ring_ok = EPI != EPI_LOGITS && (!GATHER || (g.a_kvalid % BK == 0 && g.a_kvalid >= g.ksteps_total * BK));
  // 64-wide forward tiles: two k-steps per ring stage (one barrier, one wait, one batch of requests for
  // 128 of the contraction): these tiles do 8 MFMAs per wavefront and k-step, and what a k-step costs is
  // mostly its fixed part (cfg 3's first-layer forward 43-46 -> 35-38 us; three k-steps in a ring of two
  // stages 32-35 us.  The 128-wide tiles lose with it: two k-steps per stage leave room for one workgroup
  // per CU instead of two, cfg 4's first-layer forward 65 -> 91 us).  Widths are padded to 128, so a
  // forward product always has an even number of k-steps.
  // Where the k-step count allows, three k-steps per stage in a ring of two (the same 144 KB).
  if (ring_ok && tn == 64 && ABS_RING64 && EPI == EPI_RELU && g.ksteps_per_split % 3 == 0 && g.ksteps_total % 3 == 0) {
    plan_note("fwd_ring3", TM, tn, nsplit);
    ABS_LAUNCH_K((mlp_gemm_kernel<64, EPI, GATHER, PER_UPLOAD, TAG, 2, 3>), grid1, block, s, g, rd);
    return false;
  }
  if (ring_ok && tn == 64 && ABS_RING64 && EPI == EPI_RELU && g.ksteps_per_split % 2 == 0 && g.ksteps_total % 2 == 0) {
    plan_note("fwd_ring2", TM, tn, nsplit);
    ABS_LAUNCH_K((mlp_gemm_kernel<64, EPI, GATHER, PER_UPLOAD, TAG, ABS_RING64, 2>), grid1, block, s, g, rd);
    return false;
  }
  if (ring_ok && tn == 128 && ABS_RING128) {
    plan_note(EPI == EPI_RELU ? "fwd_ring" : EPI == EPI_DGRAD ? "dgrad_ring" : "wgrad_ring", TM, tn, nsplit);
    ABS_LAUNCH_K((mlp_gemm_kernel<128, EPI, GATHER, PER_UPLOAD, TAG, ABS_RING128>), grid1, block, s, g, rd);
    return false;
  }
  plan_note(EPI == EPI_RELU ? "fwd" : EPI == EPI_LOGITS ? "logits" : EPI == EPI_DGRAD ? "dgrad" : "wgrad", TM, tn, nsplit);
  if (tn == 256)      ABS_LAUNCH_K((mlp_gemm_kernel<256, EPI, GATHER, PER_UPLOAD, TAG>), grid1, block, s, g, rd);
  else if (tn == 128) ABS_LAUNCH_K((mlp_gemm_kernel<128, EPI, GATHER, PER_UPLOAD, TAG>), grid1, block, s, g, rd);
  else                ABS_LAUNCH_K((mlp_gemm_kernel<64, EPI, GATHER, PER_UPLOAD, TAG>), grid1, block, s, g, rd);
  return false;
}

// Forward pass over `rows` stacked rows: H_l and H_l^T for the hidden layers; the model of the rows
// of upload a is slot rd.w[a].slot of the ring given by wbase / sbase (own: slot a of the private
// models).  draw0 >= 0 (training): the first layer draws the minibatch rows itself (draw index
// draw0 + sample) and leaves them in rowidx / label, and the pass stops before the output layer
// (launch_logits_ce takes over); draw0 < 0 (evaluation): rowidx holds the rows of Xsrc and the fp32
// logits are written.
// Returns the set of hidden layers l (bit l) whose ReLU mask bits were written (want_bits and the
// layer's product ran on the 256 x 256 tile kernel).
unsigned mlp_forward(const MlpArgs& a, const uint16_t* Xsrc, const RoundDesc& rd, int rows, double arows,
                     const float* wbase, const uint16_t* sbase, bool own, bool want_bits, long draw0,
                     hipStream_t s, LaunchHook* hook) {
  unsigned have_bits = 0;
  const MlpPlan& p = a.plan;
  const int L = p.L;
  uint32_t* rowidx = at<uint32_t>(a, p.off_rowidx);
  const bool train = draw0 >= 0;
  // H_l is read row-major by the next layer's product and transposed by its weight gradient and mask.
  // When both the product that writes H_l and the one that reads it run on the 256 x 256 tile kernel,
  // the reader takes the transposed copy (transposing LDS reads, TAG 3) and the row-major copy is never
  // written: half of the writer's output bytes (cfg 5's first-layer forward at 32768 rows: 134 MB, 368 -> 351 us;
  // the reader pays 7 us for the two LDS reads per fragment; a round at K = 128 -1.4 %, at K = 40 -2 %).
  // The last hidden layer keeps both: the output-layer kernels read it row-major.
  bool a_transposed = false;           // this layer reads H_l^T
  for (int l = 0; l < (train ? L - 1 : L); ++l) {
    GemmArgs g{};
    if (l == 0) {
      g.A = Xsrc; g.lda = (size_t)p.d[0]; g.a_rowidx = rowidx; g.a_kvalid = p.d[0];
      if (train) {
        g.gen_rows = 1; g.gen_B = p.B; g.gen_shard_rows = a.shard_rows; g.gen_batch_key = a.batch_key;
        g.gen_draw0 = (uint32_t)draw0; g.gen_y = a.y; g.gen_rowidx = rowidx; g.gen_label = at<int32_t>(a, p.off_label);
      }
    } else if (a_transposed) {
      g.A = at<uint16_t>(a, p.off_ht[l]); g.lda = p.ldm;
    } else {
      g.A = at<uint16_t>(a, p.off_h[l]); g.lda = (size_t)p.ld[l];
    }
    g.Bt = sbase + p.wt_off[l]; g.ldb = (size_t)p.ld[l];
    g.bt_slot_stride = p.shadow_stride;
    g.by_upload = own;
    g.rows_per_upload = p.Bp;
    g.ksteps_total = g.ksteps_per_split = p.dp[l] / BK;
    g.bias = wbase + p.b_off[l]; g.bias_slot_stride = p.slot_stride; g.n_valid = p.d[l + 1];
    const double fl = 2.0 * arows * p.d[l] * p.d[l + 1];
    if (l < L - 1) {
      g.out = at<uint16_t>(a, p.off_h[l + 1]); g.ldo = (size_t)p.ld[l + 1];
      g.outT = at<uint16_t>(a, p.off_ht[l + 1]); g.ldoT = p.ldm;
      const int kind = l == 0 ? KK_MLP_FWD_L1 : KK_MLP_FWD_HIDDEN;
      kbegin(hook, kind, fl, arows * (p.d[l] * 2.0 + p.d[l + 1] * 4.0));
      if (want_bits) g.maskbits = at<uint32_t>(a, p.off_maskbits[l + 1]);
      // does the next layer's product read H_{l+1} transposed?  (both on the large-tile kernel)
      bool next_transposed = false;
      if (l + 1 <= L - 2) {
        GemmArgs nx{};
        nx.rows_per_upload = p.Bp;
        next_transposed = gemm_is_big(l == 0, true, g, rows, p.dp[l + 1], 1) && gemm_is_big(false, true, nx, rows, p.dp[l + 2], 1);
      }
      if (next_transposed) g.out = nullptr;
      const bool big = l == 0        ? launch_gemm<EPI_RELU, true, true>(g, rd, rows, p.dp[l + 1], 1, s)
                       : a_transposed ? launch_gemm<EPI_RELU, false, true, 3>(g, rd, rows, p.dp[l + 1], 1, s)
                                      : launch_gemm<EPI_RELU, false, true>(g, rd, rows, p.dp[l + 1], 1, s);
      a_transposed = next_transposed;
      if (big && want_bits) have_bits |= 1u << (l + 1);
      kend(hook, kind);
    } else {
      g.outf = at<float>(a, p.off_z); g.ldof = (size_t)p.dp[L];
      kbegin(hook, KK_MLP_FWD_LOGITS, fl, arows * (p.d[l] * 2.0 + p.d[l + 1] * 4.0));
      launch_gemm<EPI_LOGITS, false, true>(g, rd, rows, p.dp[L], 1, s);
      kend(hook, KK_MLP_FWD_LOGITS);
    }
  }
  return have_bits;
}

// Output layer of a training pass: logits, loss sums per 32 rows, dZ_L in both orientations and its
// column sums, in one kernel (mlp_logits_ce_kernel).
void launch_logits_ce(const MlpArgs& a, const RoundDesc& rd, int rows, double arows, const float* wbase,
                      const uint16_t* sbase, bool own, hipStream_t s, LaunchHook* hook) {
  const MlpPlan& p = a.plan;
  const int L = p.L;
  LogitsCeArgs c{};
  c.H = at<uint16_t>(a, p.off_h[L - 1]); c.ldh = (size_t)p.ld[L - 1];
  c.ksteps = p.dp[L - 1] / BK;
  c.Wt = sbase + p.wt_off[L - 1]; c.ldw = (size_t)p.ld[L - 1];
  c.w_slot_stride = p.shadow_stride;
  c.bias = wbase + p.b_off[L - 1]; c.bias_slot_stride = p.slot_stride;
  c.C = p.d[L];
  c.rows_per_upload = p.Bp; c.by_upload = own;
  c.label = at<int32_t>(a, p.off_label);
  c.dZ = at<uint16_t>(a, p.off_dz[L]); c.lddz = (size_t)p.ld[L];
  c.dZT = at<uint16_t>(a, p.off_dzt[L]); c.lddzt = p.ldm;
  c.rowloss = at<float>(a, p.off_rowloss);
  c.colsum = at<float>(a, p.off_colsum[L]); c.ldcs = (size_t)p.dp[L];
  kbegin(hook, KK_MLP_LOGITS_CE, 2.0 * arows * p.d[L - 1] * p.d[L] + arows * p.d[L] * 8.0,
              arows * (p.d[L - 1] * 2.0 + p.d[L] * 4.0));
  plan_note("logits_ce", kCeRows, p.dp[L], 1);
  const dim3 grid(rows / kCeRows), block(256);
  switch (p.dp[L] / 64) {
    case 1: ABS_LAUNCH_K((mlp_logits_ce_kernel<2>), grid, block, s, c, rd); break;
    case 2: ABS_LAUNCH_K((mlp_logits_ce_kernel<4>), grid, block, s, c, rd); break;
    default: ABS_LAUNCH_K((mlp_logits_ce_kernel<8>), grid, block, s, c, rd); break;
  }
  kend(hook, KK_MLP_LOGITS_CE);
}

}  // namespace

hipError_t mlp_prepare(const MlpArgs& a, hipStream_t s) {
  const MlpPlan& p = a.plan;
  // padding of every bf16 weight copy must read as zero
  const size_t n16 = (size_t)p.R * p.shadow_stride * 2 / 16;
  mlp_fill_zero_kernel<<<dim3(1024), dim3(256), 0, s>>>(at<uint4>(a, p.off_shadow), n16);
  if (p.U > 1)
    mlp_fill_zero_kernel<<<dim3(1024), dim3(256), 0, s>>>(at<uint4>(a, p.off_priv_shadow),
                                                          (size_t)p.N * p.shadow_stride * 2 / 16);
  NullHook nh;
  RoundDesc rd0{};                       // slot_cur = slot_next = 0, no partials: w^0 onto itself
  for (int l = 0; l < p.L; ++l) launch_update(a, l, rd0, UPD_GLOBAL, 0, 0, s, &nh);   // bf16 copies of w^0
  return hipGetLastError();
}

// One pass of minibatch gradients for the K uploads of the round: U = 1 runs it once and folds
// the K-of-N reduction into the weight-gradient contraction (Eq. 3); U > 1 runs it U times on
// the uploads' private models (Eq. 2), each upload's weight gradient being its own range of
// the stacked rows, and then averages the uploads' changes into w^{t+1}.
hipError_t launch_mlp_round(const MlpArgs& a, const RoundDesc& rd, hipStream_t s, LaunchHook* hook) {
  const MlpPlan& p = a.plan;
  const int L = p.L, K = rd.K, U = p.U;
  const bool local = U > 1;
  const int rows = K * p.Bp;                 // stacked rows incl. padding (multiple of 128)
  const double arows = (double)K * p.B;      // rows that carry samples
  float* ring = at<float>(a, p.off_ring);
  const uint16_t* shadow = at<uint16_t>(a, p.off_shadow);
  float* priv = local ? at<float>(a, p.off_priv) : nullptr;
  const uint16_t* pshadow = local ? at<uint16_t>(a, p.off_priv_shadow) : nullptr;
  uint32_t* rowidx = at<uint32_t>(a, p.off_rowidx);

  for (int step = 0; step < U; ++step) {
    // where the uploads' models live during this step: the ring (by slot) or the private copies
    const bool own = local && step > 0;
    const float* wbase = own ? priv : ring;
    const uint16_t* sbase = own ? pshadow : shadow;

    // The first layer's weight gradient reads the minibatch rows straight from the dataset when
    // it runs on the 256 x 256 tile kernel and the rows are whole tiles wide; otherwise it needs
    // the transposed bf16 copy of the gathered rows.
    const bool wg0_direct = p.d[0] % TM3 == 0 && gemm_is_big(false, false, GemmArgs{}, p.dp[0], p.dp[1],
                                                               wgrad_split(p, 0, rows, local ? K : 0));

    // ---- forward at the uploads' model versions; the first layer draws the minibatch rows
    const unsigned have_bits = mlp_forward(a, a.X, rd, rows, arows, wbase, sbase, own, true,
                                           (long)step * (long)p.B, s, hook);

    // ---- output layer: loss and output gradient, already scaled by the uploads' coefficients
    launch_logits_ce(a, rd, rows, arows, wbase, sbase, own, s, hook);
    const int loss_blocks = p.Bp / kCeRows;          // row blocks of the loss sums per upload
    if (local) {
      kbegin(hook, KK_MLP_LOSS, arows, arows * 4.0);
      ABS_LAUNCH_K(mlp_loss_kernel, dim3(1), dim3(128), s, at<float>(a, p.off_rowloss), p.B, loss_blocks, K, rd.stamp,
                   a.mailbox, at<float>(a, p.off_lossacc), (int)(step == 0), (int)(step == U - 1), U);
      kend(hook, KK_MLP_LOSS);
    }

    // ---- input gradients back through W_{L-1} .. W_1 (none is needed for the first layer)
    // (dZ_l likewise: read row-major only by the next product down; when writer and reader both run on
    // the large-tile kernel the reader takes dZ_l^T and the row-major copy is not written)
    bool dz_transposed = false;          // this product reads dZ_{l+1}^T
    for (int l = L - 1; l >= 1; --l) {
      GemmArgs g{};
      if (dz_transposed) { g.A = at<uint16_t>(a, p.off_dzt[l + 1]); g.lda = p.ldm; }
      else               { g.A = at<uint16_t>(a, p.off_dz[l + 1]); g.lda = (size_t)p.ld[l + 1]; }
      g.Bt = sbase + p.wn_off[l]; g.ldb = (size_t)p.ld[l + 1];
      g.bt_slot_stride = p.shadow_stride;
      g.by_upload = own;
      g.rows_per_upload = p.Bp;
      g.ksteps_total = g.ksteps_per_split = p.dp[l + 1] / BK;
      g.maskT = at<uint16_t>(a, p.off_ht[l]); g.ldmaskT = p.ldm;
      if ((have_bits >> l) & 1u) g.maskbits = at<uint32_t>(a, p.off_maskbits[l]);   // the 128-row kernel ignores it
      g.out = l >= 2 ? at<uint16_t>(a, p.off_dz[l]) : nullptr; g.ldo = (size_t)p.ld[l];
      g.outT = at<uint16_t>(a, p.off_dzt[l]); g.ldoT = p.ldm;
      g.colsum = at<float>(a, p.off_colsum[l]); g.ldcs = (size_t)p.dp[l];
      if (!local && l == L - 1) {
        // the losses reach the host as the backward pass starts: it selects and enqueues the next
        // round while the device is still in this one
        g.pub_mailbox = a.mailbox; g.pub_rowloss = at<float>(a, p.off_rowloss);
        g.pub_nb = loss_blocks; g.pub_B = p.B;
      }
      // the product through the output layer contracts over the classes only: bandwidth-bound
      const int kind = l == L - 1 ? KK_MLP_DGRAD_OUT : KK_MLP_DGRAD;
      kbegin(hook, kind, 2.0 * arows * p.d[l] * p.d[l + 1], arows * (p.d[l + 1] * 2.0 + p.d[l] * 6.0));
      bool next_transposed = false;      // the product for layer l - 1 reads dZ_l^T
      if (l >= 2)
        next_transposed = gemm_is_big(false, true, g, rows, p.dp[l], 1) && gemm_is_big(false, true, g, rows, p.dp[l - 1], 1);
      if (next_transposed) g.out = nullptr;
      if (l == L - 1)         launch_gemm<EPI_DGRAD, false, true, 1>(g, rd, rows, p.dp[l], 1, s);
      else if (dz_transposed) launch_gemm<EPI_DGRAD, false, true, 3>(g, rd, rows, p.dp[l], 1, s);
      else                    launch_gemm<EPI_DGRAD, false, true, 0>(g, rd, rows, p.dp[l], 1, s);
      dz_transposed = next_transposed;
      kend(hook, kind);
    }

    // ---- weight gradients.  U = 1: one contraction over all stacked rows = the K-of-N
    //      reduction, split over row ranges for occupancy, then update + snapshot per layer.
    //      U > 1: split a = the rows of upload a, applied to that upload's private model.
    if (!wg0_direct) {
      kbegin(hook, KK_MLP_GATHER_T, 0, arows * p.d[0] * 4.0);
      plan_note("gather_t", 64, 64, 1);
      ABS_LAUNCH_K(mlp_gather_t_kernel, dim3(rows / 64, p.dp[0] / 64), dim3(256), s, a.X, p.d[0], (const uint32_t*)rowidx,
                   at<uint16_t>(a, p.off_xgt), p.ldm);
      kend(hook, KK_MLP_GATHER_T);
    }
    // U = 1: first layer first.  The update of a layer (Eq. 3: bound by memory) does not get a launch of
    // its own but rides along in the NEXT layer's weight-gradient launch (bound by the matrix cores) as
    // that launch's last workgroups: they take the CUs its last wave of tiles leaves idle and its tail,
    // and there is no gap between two launches.  Only the last layer's update, small, is launched by
    // itself.  (cfg 5, same box, microseconds per round at K = 32 / K = 128: 680 / 1838 with an update
    // launch per layer, 650 / 1811 this way.  Hiding the second layer's update under the first layer's
    // product instead - order 1, 0, 2, no runs: a quarter of the CUs is idle there at K = 32 - gave
    // 631 / 1807, but the product that bounds the round then carries another layer's traffic and its
    // own figure, 0.31 of the matrix peak instead of 0.37 with runs, says little about it.)
    // The bias update (column sums of every dZ_l, complete since the backward pass) rides along in the
    // same way: as the very last workgroups of the last layer's weight-gradient launch.
    BiasCore bias{};
    bias.L = L;
    int bias_cols = 0;
    for (int l = 0; l < L; ++l) {
      bias.col_begin[l] = bias_cols; bias_cols += p.d[l + 1];
      bias.colsum[l] = at<float>(a, p.off_colsum[l + 1]); bias.ldcs[l] = (size_t)p.dp[l + 1];
      bias.b_off[l] = p.b_off[l];
      bias.prow[l] = (local ? p.Bp : rows) / (l == L - 1 ? kCeRows : 64);
    }
    bias.col_begin[L] = bias_cols;
    bias.w_cur = ring + (size_t)rd.slot_cur * p.slot_stride;
    bias.w_next = ring + (size_t)rd.slot_next * p.slot_stride;
    int pend = -1, pend_split = 0, pend_q = 0;   // layer whose partials are complete and whose update is still due (its splits or run length)
    for (int li = 0; li < L; ++li) {
      const int l = local ? L - 1 - li : li;
      GemmArgs g{};
      if (!local && li == L - 1) {
        g.bias_blocks = (bias_cols + 15) / 16;
        g.bias_upd = bias;
        plan_note("with_biases", 16, 1, 1);
      }
      g.A = l == 0 ? at<uint16_t>(a, p.off_xgt) : at<uint16_t>(a, p.off_ht[l]); g.lda = p.ldm;
      g.Bt = at<uint16_t>(a, p.off_dzt[l + 1]); g.ldb = p.ldm;
      const int ksteps = rows / BK;
      const int nsplit = wgrad_split(p, l, rows, local ? K : 0);
      g.ksteps_total = ksteps;
      g.ksteps_per_split = local ? p.Bp / BK : (ksteps + nsplit - 1) / nsplit;
      g.outf = at<float>(a, p.off_partial[l]); g.ldof = (size_t)p.dp[l + 1] + kPartialPad;
      g.split_stride = (size_t)p.dp[l] * (p.dp[l + 1] + kPartialPad);
      int run_parts = 0;
      const int run_q = local ? 0 : wgrad_runs(p, l, rows, nsplit, &run_parts);
      if (run_q) { g.sk_q = run_q; }
      double upd_bytes = 0.0;
      if (pend >= 0) {
        g.nsplit = nsplit;
        const bool big = gemm_is_big(false, false, g, p.dp[l], p.dp[l + 1], nsplit);
        g.pig_upd = global_update_args(a, pend, rd, pend_split);
        if (pend_q) { g.pig_upd.sk_q = pend_q; g.pig_upd.sk_ksteps = ksteps; g.pig_upd.sk_nt = p.dp[pend + 1] / TN3; }
        g.pig_tj = big && p.d[pend + 1] >= 256 ? 256 : 64;
        g.pig_blocks = (((p.d[pend + 1] + g.pig_tj - 1) / g.pig_tj) * ((p.d[pend] + 63) / 64) + 7) / 8 * 8;
        upd_bytes = (double)p.d[pend] * p.d[pend + 1] * (4.0 * (pend_split + 2) + (pend >= 1 ? 4.0 : 2.0));
        plan_note("with_update_of_previous", 64, g.pig_tj, pend_split);
        pend = -1;
      }
      const int kind = l == 0 ? KK_MLP_WGRAD_L1 : l == L - 1 ? KK_MLP_WGRAD_OUT : KK_MLP_WGRAD;
      kbegin(hook, kind, 2.0 * arows * p.d[l] * p.d[l + 1],
             arows * (p.d[l] + p.d[l + 1]) * 2.0 + (double)nsplit * p.d[l] * p.d[l + 1] * 4.0 + upd_bytes);
      if (l == 0 && wg0_direct) {
        g.A = a.X; g.lda = (size_t)p.d[0]; g.a_rowidx = rowidx;
        launch_gemm<EPI_WGRAD, false, false, 2>(g, rd, p.dp[l], p.dp[l + 1], nsplit, s);
      } else if (l == 0) {
        launch_gemm<EPI_WGRAD, false, false, 1>(g, rd, p.dp[l], p.dp[l + 1], nsplit, s);
      } else {
        launch_gemm<EPI_WGRAD, false, false, 0>(g, rd, p.dp[l], p.dp[l + 1], nsplit, s);
      }
      kend(hook, kind);
      const int parts = run_q ? run_parts : nsplit;          // partials per tile (at most, with runs)
      if (!local && update_rows_aligned(p, l) && li + 1 < L) { pend = l; pend_split = parts; pend_q = run_q; }
      else launch_update(a, l, rd, local ? UPD_LOCAL : UPD_GLOBAL, step, parts, s, hook, run_q, ksteps);
    }

    // ---- biases (local steps: a launch of its own, per upload; else they rode on the last
    // weight-gradient launch)
    if (local) {
      BiasArgs b{};
      (BiasCore&)b = bias;
      {
        b.batched = 1;
        b.w_cur = wbase; b.cur_stride = p.slot_stride;
        b.w_next = priv; b.next_stride = p.slot_stride;
        for (int k = 0; k < K; ++k) b.cur_index[k] = (uint16_t)(own ? (uint32_t)k : rd.w[k].slot);
      }
      kbegin(hook, KK_MLP_BIAS_LOSS, (double)bias_cols * rows / 64, (double)bias_cols * rows / 64 * 4.0);
      ABS_LAUNCH_K(mlp_bias_kernel, dim3((bias_cols + 15) / 16, K), dim3(256), s, b);
      kend(hook, KK_MLP_BIAS_LOSS);
    }
  }

  if (local) {
    // ---- Eq. 3 over the uploads' changes, then update + snapshot per layer
    DeltaArgs d{};
    d.ring = ring; d.slot_stride = p.slot_stride;
    d.priv = priv;
    d.D = at<float>(a, p.off_delta);
    d.P = p.P;
    d.L = L;
    for (int l = 0; l < L; ++l) { d.b_off[l] = p.b_off[l]; d.b_len[l] = p.d[l + 1]; }
    d.w_cur = ring + (size_t)rd.slot_cur * p.slot_stride;
    d.w_next = ring + (size_t)rd.slot_next * p.slot_stride;
    kbegin(hook, KK_DELTA_UPDATE, 2.0 * K * p.P, (2.0 * K + 1.0) * p.P * 4.0);
    ABS_LAUNCH_K(mlp_delta_kernel, dim3((unsigned)((p.P + 255) / 256)), dim3(256), s, d, rd);
    kend(hook, KK_DELTA_UPDATE);
    for (int l = L - 1; l >= 0; --l) launch_update(a, l, rd, UPD_DELTA, 0, 1, s, hook);
  }
  return t_plan ? hipSuccess : hipGetLastError();
}

std::string mlp_round_plan(const abs_config& cfg, int K) {
  MlpArgs a{};
  const char* why = nullptr;
  if (K < 1 || K > cfg.N || !mlp_plan(cfg, a.plan, &why)) return std::string();
  RoundDesc rd{};
  rd.K = K;
  NullHook nh;
  std::string out;
  t_plan = &out;
  (void)launch_mlp_round(a, rd, nullptr, &nh);   // records, launches nothing, touches no memory
  t_plan = nullptr;
  if (!out.empty() && out.back() == ' ') out.pop_back();
  return out;
}

hipError_t launch_mlp_eval(const MlpArgs& a, uint32_t slot, const EvalArgs& e, hipStream_t s, LaunchHook* hook) {
  const MlpPlan& p = a.plan;
  if (e.cap < p.Mp) return hipErrorInvalidValue;
  uint32_t* rowidx = at<uint32_t>(a, p.off_rowidx);
  int32_t* label = at<int32_t>(a, p.off_label);
  hipError_t err = launch_eval_clear(e, s);
  for (int64_t row0 = 0; row0 < e.n_rows && err == hipSuccess; row0 += p.Mp) {
    const int n = (int)(e.n_rows - row0 < p.Mp ? e.n_rows - row0 : p.Mp);
    RoundDesc rd{};                               // every block of Bp rows uses the same version
    rd.K = (n + p.Bp - 1) / p.Bp;
    for (int k = 0; k < rd.K; ++k) rd.w[k].slot = slot;
    const int rows = rd.K * p.Bp;
    hook->begin(KK_EVAL, 0, 12.0 * n);
    mlp_eval_index_kernel<<<dim3((rows + 255) / 256), dim3(256), 0, s>>>(rowidx, label, (const int32_t*)e.y, row0, n, rows);
    hook->end(KK_EVAL);
    mlp_forward(a, (const uint16_t*)e.X, rd, rows, (double)n, at<float>(a, p.off_ring), at<uint16_t>(a, p.off_shadow),
                false, false, -1, s, hook);
    hook->begin(KK_EVAL, 8.0 * n * p.d[p.L], 4.0 * n * p.d[p.L]);
    const dim3 grid((n + 3) / 4), block(256);
    const float* Z = at<float>(a, p.off_z);
    const size_t ld = (size_t)p.dp[p.L];
    switch (p.dp[p.L] / 64) {
      case 1: mlp_eval_rows_kernel<1><<<grid, block, 0, s>>>(Z, ld, p.d[p.L], label, n, e.rowloss, e.correct); break;
      case 2: mlp_eval_rows_kernel<2><<<grid, block, 0, s>>>(Z, ld, p.d[p.L], label, n, e.rowloss, e.correct); break;
      default: mlp_eval_rows_kernel<4><<<grid, block, 0, s>>>(Z, ld, p.d[p.L], label, n, e.rowloss, e.correct); break;
    }
    hook->end(KK_EVAL);
    err = hipGetLastError();
    if (err == hipSuccess) err = launch_eval_reduce(e, n, s, hook);
  }
  return err;
}

}  // namespace abs_impl
