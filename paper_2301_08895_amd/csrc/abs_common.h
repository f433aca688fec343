// Shared by the host scheduler and the HIP translation units of libabs.
#pragma once
#include <cstdint>
#include <cstddef>
#include "../../include/abs.h"

#if defined(__HIPCC__)
#define ABS_HD __host__ __device__ __forceinline__
#else
#define ABS_HD inline
#endif

namespace abs_impl {

// ---- counter-based random numbers -------------------------------------------------
// 64 random bits per counter (seed, stream, worker, job, index), three rounds of the
// SplitMix64 output function (Steele, Lea, Flood 2014).  The paper only requires that
// minibatches are independent across workers, local steps and rounds (Section II-A)
// and that execution times are random (Section V-A).
constexpr uint64_t kGoldenGamma = 0x9E3779B97F4A7C15ull;
enum : uint32_t { kStreamTime = 0, kStreamBatch = 1 };

ABS_HD uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
ABS_HD uint64_t stream_key(uint64_t seed, uint32_t stream) {
  return mix64(seed + kGoldenGamma * (uint64_t)(stream + 1u));
}
ABS_HD uint64_t job_key(uint64_t skey, uint32_t n, uint32_t j) {
  return mix64(skey ^ (((uint64_t)n << 32) | (uint64_t)j));
}
ABS_HD uint64_t draw(uint64_t jkey, uint32_t i) {
  return mix64(jkey + kGoldenGamma * (uint64_t)(i + 1u));
}

// ---- what the host tells the kernels about one round --------------------------------
// Entry a describes the a-th upload in arrival order: which worker, which of its jobs
// (selects the minibatch), which ring slot holds the model it computed at, and its
// coefficient c = eta_k / (K^t B) in Eq. 3 (eta_k = eta or eta / max(1, tau_k)).
struct WorkerDesc {
  uint32_t id;
  uint32_t job;
  uint32_t slot;
  float    c;
};
// The losses travel through a small mailbox in device-visible host memory: loss[a] for
// upload a, then `stamp`, written last, so the host can pick them up by polling.
struct LossMailbox {
  float loss[ABS_MAX_WORKERS];
  volatile uint32_t stamp;
};

#if defined(__HIPCC__)
// Publish K losses that sit in LDS: one wavefront writes them all, fences once at system
// scope and only then writes the stamp, so a host that sees the stamp sees the losses.
// (One fence per loss would cost a trip over the host link each.)  Call with the whole
// workgroup after a __syncthreads() that follows the LDS writes.
__device__ __forceinline__ void publish_losses(LossMailbox* box, const float* s_loss, int K, uint32_t stamp) {
  if (threadIdx.x < 64) {
    for (int a = threadIdx.x; a < K; a += 64) box->loss[a] = s_loss[a];
    __threadfence_system();
    if (threadIdx.x == 0) box->stamp = stamp;
  }
}
#endif

struct RoundDesc {
  int32_t  K;          // uploads aggregated this round
  uint32_t slot_cur;   // ring slot of w^t
  uint32_t slot_next;  // ring slot that receives w^{t+1}
  uint32_t stamp;      // written to the loss mailbox after this round's losses (round + 1)
  WorkerDesc w[ABS_MAX_WORKERS];
};

}  // namespace abs_impl
