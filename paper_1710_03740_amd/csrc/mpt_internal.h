// Internal helpers shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "mpt.h"

#define MPT_LAUNCH_CHECK()                                   \
  do {                                                       \
    hipError_t e__ = hipGetLastError();                      \
    if (e__ != hipSuccess) return MPT_ERR_HIP;               \
  } while (0)

static inline bool mpt_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
static inline bool mpt_finite(float x) { return x == x && x - x == 0.0f; }

// Correctly rounded FP32 division and square root (the compiler's default for the plain operators; HIP's
// __fdiv_rn / __fsqrt_rn intrinsics map to the approximate hardware forms and are not used).
__device__ __forceinline__ float div_rn(float a, float b) { return a / b; }
__device__ __forceinline__ float sqrt_rn(float a) { return __builtin_sqrtf(a); }

// An FP32 value that is rounded to FP16 right after a multiplication gets fused by the compiler into
// v_fma_mixlo_f16, which on gfx950 rounds the exact product once to FP16 instead of first to FP32 (measured: 1 in
// ~25000 results differs by one FP16 step).  Where the contract is "FP32 operation, then FP16 rounding", the value
// passes through this before the conversion.
__device__ __forceinline__ float mpt_rounded_f32(float v) {
  asm("" : "+v"(v));
  return v;
}

// Tunables.  The library as shipped has none: MPT_TUNABLE(name, default) is the default, a compile-time constant, and
// the alternative kernels are not built.  A tuning build (-DMPT_TUNING; measurements only, never the product) reads
// each value once from the environment variable of that name.
#ifdef MPT_TUNING
int mpt_env_int(const char* name, int dflt);
#define MPT_TUNABLE(name, dflt) mpt_env_int(name, dflt)
#else
#define MPT_TUNABLE(name, dflt) (dflt)
#endif
