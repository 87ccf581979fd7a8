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
    case MPT_ERR_WORKSPACE: return "workspace too small";
    case MPT_ERR_ARG: return "scalar argument out of range";
    case MPT_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

extern "C" int mpt_version(void) { return 102; }

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
