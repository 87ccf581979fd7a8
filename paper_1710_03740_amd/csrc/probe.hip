// Diagnostic: the sustained rate of v_mfma_f32_16x16x32_f16 out of registers, with no memory traffic at all.
// The GPU's clock under matrix work depends on the operand bits (all-zero operands run at the maximum clock,
// operands with random mantissas pull it down to the power limit), so this is the ceiling against which the GEMM
// kernels' FLOP rates on a given kind of data are to be read.  gfx950 only.
#include "mpt_internal.h"

typedef _Float16 ph8 __attribute__((ext_vector_type(8)));
typedef float pf4 __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// zeros, or random sign and mantissa with magnitude 2^-5 .. 2^-1 (the range of normalised activations and weights)
__device__ __forceinline__ _Float16 probe_value(int random, uint32_t seed) {
  const uint32_t h = probe_hash(seed);
  const uint16_t bits = random ? (uint16_t)(((h & 1u) << 15) | ((10u + (h >> 1) % 5u) << 10) | ((h >> 8) & 0x3FFu)) : (uint16_t)0;
  return __builtin_bit_cast(_Float16, bits);
}

// One wavefront per SIMD (the GEMM kernel's shape): 64 independent accumulator blocks, 8 x 8 operand fragments.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_probe_mfma(int iters, int random, float* sink) {
  ph8 x[8], y[8];
  const uint32_t id = blockIdx.x * 256u + threadIdx.x;
  for (int j = 0; j < 8; ++j)
    for (int i = 0; i < 8; ++i) {
      x[j][i] = probe_value(random, id * 64u + j * 8u + i);
      y[j][i] = probe_value(random, 0x9e3779b9u + id * 64u + j * 8u + i);
    }
  pf4 acc[64];
  for (int a = 0; a < 64; ++a)
    for (int v = 0; v < 4; ++v) acc[a][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int a = 0; a < 64; ++a) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc[a]) : "v"(x[a & 7]), "v"(y[a >> 3]));
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");       // the MFMAs are opaque to the compiler's hazard handling
  float s = 0.f;
  for (int a = 0; a < 64; ++a)
    for (int v = 0; v < 4; ++v) s += acc[a][v];
  if (s == 1.2345f) sink[0] = s;                            // keeps the loop alive; practically never true
}

}  // namespace

extern "C" int mpt_probe_mfma(void* stream, int iters, int random_operands, float* sink_dev) {
  if (sink_dev == nullptr) return MPT_ERR_NULL;
  if (iters < 1 || iters > (1 << 20)) return MPT_ERR_ARG;
  if (!mpt_aligned(sink_dev, 4)) return MPT_ERR_ALIGN;
  hipLaunchKernelGGL(k_probe_mfma, dim3(256), dim3(256), 0, static_cast<hipStream_t>(stream), iters, random_operands ? 1 : 0, sink_dev);
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}
