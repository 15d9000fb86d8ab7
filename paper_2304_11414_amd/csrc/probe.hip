// Measurement helper, not part of the layer: a register-resident bf16 MFMA loop with the grouped
// GEMM's launch shape (one block of four wavefronts per CU, 4 x 4 accumulator blocks of 32x32x16 per
// wavefront) and no memory traffic at all.  What it sustains is the practical ceiling of the matrix
// cores on this device for the operand values given: with random operands the clock settles lower
// (power limit) than with constant ones.

#include "common.h"

namespace ppmoe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__global__ __launch_bounds__(256) void mfma_probe_kernel(float* __restrict__ sink, int64_t iters,
                                                         int random_operands) {
  f32x16 acc[4][4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
  bf16x8 a[4], b[4];
  uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      h = h * 1664525u + 1013904223u;
      const float ua = random_operands ? static_cast<float>(h >> 8) * (2.0f / 16777216.0f) - 1.0f : 1.0f;
      h = h * 1664525u + 1013904223u;
      const float ub = random_operands ? static_cast<float>(h >> 8) * (2.0f / 16777216.0f) - 1.0f : 1.0f;
      a[i][e] = static_cast<__bf16>(ua * 0.03125f);
      b[i][e] = static_cast<__bf16>(ub);
    }
  for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 4; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ni], b[mi], acc[mi][ni], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) s += acc[mi][ni][v];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

hipError_t launch_mfma_probe(int64_t iters, int random_operands, float* sink, int* blocks_out,
                             hipStream_t s) {
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  if (cus > kMaxPersistentBlocks) cus = kMaxPersistentBlocks;
  if (cus < 1) return hipErrorInvalidConfiguration;
  *blocks_out = cus;
  mfma_probe_kernel<<<cus, 256, 0, s>>>(sink, iters, random_operands);
  return hipGetLastError();
}

}  // namespace ppmoe
