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

// Tunables read once from the environment (benchmark sweeps only; defaults are the tuned values).
int mpt_env_int(const char* name, int dflt);
