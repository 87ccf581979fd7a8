// Host-only parts of the C ABI: status strings, version, and the loss-scale
// policy on a host-resident struct (paper Sec. 5; constants are the caller's).
#include "mpt.h"
#include <math.h>

extern "C" const char* mpt_status_string(int status) {
  switch (status) {
    case MPT_OK: return "ok";
    case MPT_ERR_NULL: return "required pointer is NULL";
    case MPT_ERR_SHAPE: return "bad size or leading dimension";
    case MPT_ERR_ALIGN: return "pointer not aligned to its element type";
    case MPT_ERR_WORKSPACE: return "workspace too small (or: split partials exceed the library's static scratch array)";
    case MPT_ERR_ARG: return "scalar argument out of range";
    case MPT_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

extern "C" int mpt_version(void) { return 106; }

extern "C" int mpt_scaler_init(mpt_scaler* s, float scale, int32_t growth_interval) {
  if (s == nullptr) return MPT_ERR_NULL;
  if (!(scale > 0.f) || !isfinite(scale) || growth_interval < 1) return MPT_ERR_ARG;
  s->scale = scale;
  s->inv_scale = 1.0f / scale;
  s->good_steps = 0;
  s->growth_interval = growth_interval;
  s->growth = 2.0f;
  s->backoff = 0.5f;
  s->min_scale = 1.0f;
  s->max_scale = 16777216.0f;
  return MPT_OK;
}

extern "C" int mpt_loss_scale_update(mpt_scaler* s, int overflow) {
  if (s == nullptr) return MPT_ERR_NULL;
  if (overflow) {
    s->scale = fmaxf(s->scale * s->backoff, s->min_scale);
    s->good_steps = 0;
  } else {
    s->good_steps += 1;
    if (s->good_steps == s->growth_interval) {
      s->scale = fminf(s->scale * s->growth, s->max_scale);
      s->good_steps = 0;
    }
  }
  s->inv_scale = 1.0f / s->scale;
  return MPT_OK;
}

// Largest power of two 2^k with 2^k * max <= 65504 (paper Sec. 3.2), from the FP16 bit pattern of max.
// Exact integer arithmetic: max = m * 2^q with integer m < 2^11, and 65504 = 2047 * 2^5.
extern "C" int mpt_suggest_loss_scale_log2(uint32_t absmax_bits, int if_zero) {
  const uint32_t mag = absmax_bits & 0x7FFFu;
  if (mag == 0u || mag >= 0x7C00u) return if_zero;
  const uint32_t ef = mag >> 10, mant = mag & 0x3FFu;
  const int64_t m = ef ? (int64_t)(1024 + mant) : (int64_t)mant;       // value = m * 2^q
  const int q = ef ? (int)ef - 25 : -24;
  // 2^k * m * 2^q <= 2047 * 2^5  <=>  m * 2^sh <= 2047 with sh = k + q - 5  (m < 2^11)
  for (int k = 40; k >= -24; --k) {
    const int sh = k + q - 5;
    bool ok;
    if (sh >= 0) ok = sh <= 11 && (m << sh) <= 2047;
    else ok = -sh >= 11 || m <= ((int64_t)2047 << -sh);
    if (ok) return k;
  }
  return -24;
}
