// Calibration of the matrix cores: nothing but the MFMA instructions of a GEMM tile (either form), on
// register operands, with no memory traffic at all.  What it reports is the rate the chip sustains
// on this instruction mix at the clock it settles at, i.e. the ceiling the GEMM kernels are measured
// against in practice (the published peak assumes the full boost clock).
#include <hip/hip_runtime.h>

#include <string>

#include "../../include/abs.h"

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// flops per wavefront and iteration: one 64-wide k-step of a 128 x 64 wavefront tile, as 4 x 2 blocks x 4 sub-steps of
// 32x32x16 or as 8 x 4 blocks x 2 sub-steps of 16x16x32
constexpr double kWaveFlopsPerIter = 2.0 * 128 * 64 * 64;

__device__ __forceinline__ uint32_t hash32(uint32_t x) {
  x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
  return x;
}

// data_mode 0: every operand element is 1.0 (the multipliers see constant inputs);
// data_mode 1: operand elements are bf16 values of random mantissa and sign with exponents in
// [2^-2, 2^1), different in every lane and register - what a GEMM on real data feeds them.
// FORM 32: v_mfma_f32_32x32x16_bf16 (the 128-row kernels);  FORM 16: v_mfma_f32_16x16x32_bf16 (the large-tile kernel)
template <int FORM>
__global__ __launch_bounds__(512, 1) void mfma_only_kernel(int iters, int data_mode, float* out) {
  const uint32_t gid = blockIdx.x * 512u + threadIdx.x;
  union { uint32_t u[4]; bf16x8_t v; } fa[4], fb[2];
#pragma unroll
  for (int i = 0; i < 6; ++i) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      uint32_t w = 0x3F803F80u;          // two bf16 ones
      if (data_mode) {
        const uint32_t h = hash32(gid * 24u + i * 4u + q + 1u);
        // per half: sign (1) | exponent 125..127 (8) | mantissa (7)
        const uint32_t lo = ((h & 1u) << 15) | ((125u + ((h >> 1) % 3u)) << 7) | ((h >> 4) & 0x7Fu);
        const uint32_t hi = (((h >> 11) & 1u) << 15) | ((125u + ((h >> 12) % 3u)) << 7) | ((h >> 15) & 0x7Fu);
        w = lo | (hi << 16);
      }
      (i < 4 ? fa[i].u[q] : fb[i - 4].u[q]) = w;
    }
  }
  float sum = 0.f;
  if (FORM == 32) {
    f32x16_t acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
          for (int ni = 0; ni < 2; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi].v, fb[ni].v, acc[mi][ni], 0, 0, 0);
    }
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[mi][ni][r];
  } else {
    f32x4_t acc[8][4];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[a][b][r] = 0.f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int a = 0; a < 8; ++a)
#pragma unroll
          for (int b = 0; b < 4; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[(a + s) & 3].v, fb[(b + s) & 1].v, acc[a][b], 0, 0, 0);
    }
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 4; ++r) sum += acc[a][b][r];
  }
  if (sum == 12345.678f) out[gid] = sum;       // keeps the accumulators alive; practically never taken
}

}  // namespace

extern "C" int abs_calibrate_mfma(int32_t data_mode, int32_t iters, int32_t workgroups, float* d_scratch,
                                  void* hip_stream, double* h_ms, double* h_tflops) {
  if (!h_ms || !h_tflops || !d_scratch || iters < 1 || workgroups < 1 || workgroups > 65536 ||
      data_mode < 0 || data_mode > 3)
    return ABS_E_ARG;
  const int form16 = data_mode >> 1;
  data_mode &= 1;
  void (*const kernel)(int, int, float*) = form16 ? mfma_only_kernel<16> : mfma_only_kernel<32>;
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return ABS_E_HIP;
  kernel<<<dim3(workgroups), dim3(512), 0, s>>>(iters, data_mode, d_scratch);      // warm-up
  hipError_t e = hipEventRecord(e0, s);
  kernel<<<dim3(workgroups), dim3(512), 0, s>>>(iters, data_mode, d_scratch);
  if (e == hipSuccess) e = hipGetLastError();
  if (e == hipSuccess) e = hipEventRecord(e1, s);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  if (e != hipSuccess) return ABS_E_HIP;
  const double flops = (double)workgroups * 8.0 * (double)iters * kWaveFlopsPerIter;
  *h_ms = ms;
  *h_tflops = flops / (ms * 1e-3) / 1e12;
  return ABS_OK;
}
