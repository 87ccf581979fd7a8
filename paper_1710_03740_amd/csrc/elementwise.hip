// HBM-bound passes of the mixed-precision step for gfx950:
//   unscale + Inf/NaN check            (paper Sec. 3.2)
//   FP32 master update + FP16 copy     (paper Sec. 3.1, skip rule Sec. 3.2)
//   device-side loss-scale policy      (paper Sec. 5)
//   ReLU, scaled softmax cross-entropy (paper Sec. 3.3 glue)
// Every thread moves 16-byte vectors; a wavefront therefore touches 1 KiB
// contiguous per stream per instruction.  Arithmetic is written with the
// non-contracting intrinsics so each FP32 operation rounds on its own.
#include "mpt_internal.h"
#include <stdlib.h>

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

#ifdef MPT_TUNING
int mpt_env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  return v && *v ? atoi(v) : dflt;
}
#endif

namespace {

constexpr int kThreads = 256;

template <bool NT, class T>
__device__ __forceinline__ T ld(const T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT, class T>
__device__ __forceinline__ void st(T* p, T v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

__device__ __forceinline__ bool half_special(uint32_t bits16) { return (bits16 & 0x7C00u) == 0x7C00u; }
__device__ __forceinline__ bool float_special(uint32_t bits32) { return (bits32 & 0x7F800000u) == 0x7F800000u; }

// One optimizer step on a single element; the order and the separate rounding
// of the four operations is the contract (no fused multiply-add).
template <bool MOM>
__device__ __forceinline__ float step1(float w, float& m, float graw, float inv, float lr, float mu) {
  const float g = __fmul_rn(graw, inv);
  float d;
  if constexpr (MOM) {
    m = __fadd_rn(__fmul_rn(mu, m), g);
    d = __fmul_rn(lr, m);
  } else {
    d = __fmul_rn(lr, g);
  }
  return __fsub_rn(w, d);
}

// 2 consecutive elements per thread per trip, and consecutive threads own consecutive pairs, so every load and
// store instruction of a wavefront covers one contiguous span (512 B of an FP32 stream, 256 B of an FP16 stream).
// Six streams move per element: gradient, master and momentum in; master, momentum and FP16 copy out.  Measured
// on MI355X, this narrow shape sustains more of HBM for the six-stream 1:1 read/write mix than 16-byte-per-lane
// accesses do (6.6 vs 6.2 TB/s at 116M elements).
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f2 __attribute__((ext_vector_type(2)));

template <bool MOM, bool G32, bool NT, int BS>
__global__ __launch_bounds__(BS) void k_master_update(
    size_t n, float* __restrict__ w32, float* __restrict__ m32, const void* __restrict__ grad,
    uint16_t* __restrict__ w16, float inv_scale, const mpt_scaler* __restrict__ scaler, float lr, float mu,
    const uint32_t* __restrict__ flag) {
  // The flag and the scale are fetched while the vector loads below are already in flight; nothing is stored
  // before the flag has been seen.  (A skipped step therefore still reads its operands; it writes nothing.)
  const size_t npair = n >> 1;
  const size_t stride = (size_t)gridDim.x * BS;
  for (size_t q = (size_t)blockIdx.x * BS + threadIdx.x; q < npair; q += stride) {
    float g[2];
    if constexpr (G32) {
      const f2 a = ld<NT>(reinterpret_cast<const f2*>(grad) + q);
      g[0] = a[0]; g[1] = a[1];
    } else {
      const h2 a = ld<NT>(reinterpret_cast<const h2*>(grad) + q);
      g[0] = (float)a[0]; g[1] = (float)a[1];
    }
    f2* wp = reinterpret_cast<f2*>(w32) + q;
    f2 w = ld<NT>(wp);
    f2 m = {0, 0};
    f2* mp = nullptr;
    if constexpr (MOM) {
      mp = reinterpret_cast<f2*>(m32) + q;
      m = ld<NT>(mp);
    }
    if (flag != nullptr && *flag != 0u) return;            // overflow: the whole step is a no-op
    const float inv = scaler != nullptr ? scaler->inv_scale : inv_scale;
    h2 h;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      float mi = m[i];
      w[i] = step1<MOM>(w[i], mi, g[i], inv, lr, mu);
      m[i] = mi;
      h[i] = (_Float16)w[i];
    }
    st<NT>(wp, w);
    if constexpr (MOM) st<NT>(mp, m);
    st<NT>(reinterpret_cast<h2*>(w16) + q, h);
  }
  // odd tail: the last element, by one thread
  if ((n & 1) && blockIdx.x == 0 && threadIdx.x == 0) {
    if (flag != nullptr && *flag != 0u) return;
    const float inv = scaler != nullptr ? scaler->inv_scale : inv_scale;
    const size_t i = n - 1;
    float graw;
    if constexpr (G32) graw = reinterpret_cast<const float*>(grad)[i];
    else graw = (float)reinterpret_cast<const _Float16*>(grad)[i];
    float m = 0.f;
    if constexpr (MOM) m = m32[i];
    const float w = step1<MOM>(w32[i], m, graw, inv, lr, mu);
    w32[i] = w;
    if constexpr (MOM) m32[i] = m;
    reinterpret_cast<_Float16*>(w16)[i] = (_Float16)w;
  }
}

// One pass over the gradient: overflow vote and update together, results into a second set of buffers (the caller
// adopts them only if the flag stayed clear).  Same access shape as k_master_update; PAIRS = false is the
// element-wise form for buffers that are only element-aligned.
template <bool MOM, bool G32, bool PAIRS>
__global__ __launch_bounds__(kThreads) void k_master_update_fused(
    size_t n, const float* __restrict__ w_in, const float* __restrict__ m_in, const void* __restrict__ grad,
    float* __restrict__ w_out, float* __restrict__ m_out, uint16_t* __restrict__ h_out, float inv_scale,
    const mpt_scaler* __restrict__ scaler, float lr, float mu, uint32_t* __restrict__ flag) {
  const float inv = scaler != nullptr ? scaler->inv_scale : inv_scale;
  const size_t stride = (size_t)gridDim.x * kThreads;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  bool bad = false;
  auto one = [&](size_t i) {
    float graw;
    if constexpr (G32) {
      graw = reinterpret_cast<const float*>(grad)[i];
      bad |= float_special(__float_as_uint(graw));
    } else {
      const uint16_t b = reinterpret_cast<const uint16_t*>(grad)[i];
      bad |= (b & 0x7C00u) == 0x7C00u;
      graw = (float)__builtin_bit_cast(_Float16, b);
    }
    float m = 0.f;
    if constexpr (MOM) m = m_in[i];
    const float w = step1<MOM>(w_in[i], m, graw, inv, lr, mu);
    w_out[i] = w;
    if constexpr (MOM) m_out[i] = m;
    reinterpret_cast<_Float16*>(h_out)[i] = (_Float16)w;
  };
  if constexpr (PAIRS) {
    const size_t npair = n >> 1;
    for (size_t q = tid; q < npair; q += stride) {
      float g[2];
      if constexpr (G32) {
        const f2 a = ld<true>(reinterpret_cast<const f2*>(grad) + q);
        g[0] = a[0]; g[1] = a[1];
        bad |= float_special(__float_as_uint(a[0])) | float_special(__float_as_uint(a[1]));
      } else {
        const h2 a = ld<true>(reinterpret_cast<const h2*>(grad) + q);
        const uint32_t b = __builtin_bit_cast(uint32_t, a);
        bad |= ((b & 0x7C00u) == 0x7C00u) | ((b & 0x7C000000u) == 0x7C000000u);
        g[0] = (float)a[0]; g[1] = (float)a[1];
      }
      f2 w = ld<true>(reinterpret_cast<const f2*>(w_in) + q);
      f2 m = {0, 0};
      if constexpr (MOM) m = ld<true>(reinterpret_cast<const f2*>(m_in) + q);
      h2 h;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        float mi = m[i];
        w[i] = step1<MOM>(w[i], mi, g[i], inv, lr, mu);
        m[i] = mi;
        h[i] = (_Float16)w[i];
      }
      st<true>(reinterpret_cast<f2*>(w_out) + q, w);
      if constexpr (MOM) st<true>(reinterpret_cast<f2*>(m_out) + q, m);
      st<true>(reinterpret_cast<h2*>(h_out) + q, h);
    }
    if ((n & 1) && tid == 0) one(n - 1);
  } else {
    for (size_t i = tid; i < n; i += stride) one(i);
  }
  const unsigned long long vote = __builtin_amdgcn_ballot_w64(bad);
  if (vote != 0ull && (threadIdx.x & 63) == 0) atomicOr(flag, 1u);
}

// Same step for buffers that are only element-aligned: one element per thread per trip.
template <bool MOM, bool G32>
__global__ __launch_bounds__(kThreads) void k_master_update_scalar(
    size_t n, float* __restrict__ w32, float* __restrict__ m32, const void* __restrict__ grad,
    uint16_t* __restrict__ w16, float inv_scale, const mpt_scaler* __restrict__ scaler, float lr, float mu,
    const uint32_t* __restrict__ flag) {
  if (flag != nullptr && *flag != 0u) return;
  const float inv = scaler != nullptr ? scaler->inv_scale : inv_scale;
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
    float graw;
    if constexpr (G32) graw = reinterpret_cast<const float*>(grad)[i];
    else graw = (float)reinterpret_cast<const _Float16*>(grad)[i];
    float m = 0.f;
    if constexpr (MOM) m = m32[i];
    const float w = step1<MOM>(w32[i], m, graw, inv, lr, mu);
    w32[i] = w;
    if constexpr (MOM) m32[i] = m;
    reinterpret_cast<_Float16*>(w16)[i] = (_Float16)w;
  }
}

// Many parameter tensors in one launch (a network's layers each own a weight, a master copy and a momentum buffer;
// a launch per tensor costs more than the update of a small one).  The tensors' pointers and sizes travel in the
// kernel's arguments; a workgroup finds its tensor by walking the table of first workgroups (wavefront-uniform) and
// then does what k_master_update / k_master_update_scalar do for that tensor: pairs where the tensor's buffers are
// aligned for them, single elements else, one trip per thread.  Same operations, same results.
constexpr int kMultiMax = 48;
struct MultiItems {
  float* w32[kMultiMax];
  float* m32[kMultiMax];
  const void* grad[kMultiMax];
  uint16_t* w16[kMultiMax];
  unsigned long long n[kMultiMax];
  unsigned first_block[kMultiMax + 1];     // workgroups [first_block[k], first_block[k + 1]) belong to tensor k
  unsigned pairs_mask_lo, pairs_mask_hi;   // bit k: tensor k moves in pairs
  int count;
};

template <bool MOM, bool G32>
__global__ __launch_bounds__(kThreads) void k_master_update_multi(MultiItems it, float inv_scale, const mpt_scaler* __restrict__ scaler,
                                                                 float lr, float mu, const uint32_t* __restrict__ flag) {
  int k = 0;
  while (k + 1 < it.count && blockIdx.x >= it.first_block[k + 1]) ++k;
  const size_t n = (size_t)it.n[k];
  float* w32 = it.w32[k];
  float* m32 = it.m32[k];
  const void* grad = it.grad[k];
  uint16_t* w16 = it.w16[k];
  const bool pairs = ((k < 32 ? it.pairs_mask_lo >> k : it.pairs_mask_hi >> (k - 32)) & 1u) != 0u;
  const size_t local = (size_t)(blockIdx.x - it.first_block[k]) * kThreads + threadIdx.x;
  if (pairs) {
    const size_t q = local;
    const bool tail = (n & 1) && local == 0;                 // the odd last element goes with the tensor's first thread
    if (q >= (n >> 1) && !tail) return;
    float g[2] = {0.f, 0.f};
    f2 w = {0, 0}, m = {0, 0};
    f2* wp = reinterpret_cast<f2*>(w32) + q;
    f2* mp = MOM ? reinterpret_cast<f2*>(m32) + q : nullptr;
    const bool has_pair = q < (n >> 1);
    if (has_pair) {
      if constexpr (G32) {
        const f2 a = reinterpret_cast<const f2*>(grad)[q];
        g[0] = a[0]; g[1] = a[1];
      } else {
        const h2 a = reinterpret_cast<const h2*>(grad)[q];
        g[0] = (float)a[0]; g[1] = (float)a[1];
      }
      w = *wp;
      if constexpr (MOM) m = *mp;
    }
    if (flag != nullptr && *flag != 0u) return;             // overflow: the whole step is a no-op
    const float inv = scaler != nullptr ? scaler->inv_scale : inv_scale;
    if (has_pair) {
      h2 h;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        float mi = m[i];
        w[i] = step1<MOM>(w[i], mi, g[i], inv, lr, mu);
        m[i] = mi;
        h[i] = (_Float16)w[i];
      }
      *wp = w;
      if constexpr (MOM) *mp = m;
      reinterpret_cast<h2*>(w16)[q] = h;
    }
    if (tail) {
      const size_t i = n - 1;
      float graw;
      if constexpr (G32) graw = reinterpret_cast<const float*>(grad)[i];
      else graw = (float)reinterpret_cast<const _Float16*>(grad)[i];
      float mm = 0.f;
      if constexpr (MOM) mm = m32[i];
      const float wn = step1<MOM>(w32[i], mm, graw, inv, lr, mu);
      w32[i] = wn;
      if constexpr (MOM) m32[i] = mm;
      reinterpret_cast<_Float16*>(w16)[i] = (_Float16)wn;
    }
  } else {
    const size_t i = local;
    if (i >= n) return;
    if (flag != nullptr && *flag != 0u) return;
    const float inv = scaler != nullptr ? scaler->inv_scale : inv_scale;
    float graw;
    if constexpr (G32) graw = reinterpret_cast<const float*>(grad)[i];
    else graw = (float)reinterpret_cast<const _Float16*>(grad)[i];
    float mm = 0.f;
    if constexpr (MOM) mm = m32[i];
    const float wn = step1<MOM>(w32[i], mm, graw, inv, lr, mu);
    w32[i] = wn;
    if constexpr (MOM) m32[i] = mm;
    reinterpret_cast<_Float16*>(w16)[i] = (_Float16)wn;
  }
}

// Inf/NaN scan (+ optional FP32 unscaled copy).  The exponent-field test runs on
// the stored bits; each wavefront votes and at most one lane per wavefront
// touches the flag.
template <bool G32, bool WRITE, bool VEC>
__global__ __launch_bounds__(kThreads) void k_unscale_check(
    const void* __restrict__ grad, size_t n, float inv, float* __restrict__ out, uint32_t* __restrict__ flag) {
  bool bad = false;
  const size_t stride = (size_t)gridDim.x * kThreads;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  size_t done = 0;
  if constexpr (VEC) {
    const size_t nvec = n >> 3;
    done = nvec << 3;
    for (size_t v = tid; v < nvec; v += stride) {
      if constexpr (G32) {
        const u4* gp = reinterpret_cast<const u4*>(grad) + 2 * v;
        const u4 a = ld<true>(gp), b = ld<true>(gp + 1);
#pragma unroll
        for (int i = 0; i < 4; ++i) bad |= float_special(a[i]) | float_special(b[i]);
        if constexpr (WRITE) {
          f4 oa, ob;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            oa[i] = __fmul_rn(__uint_as_float(a[i]), inv);
            ob[i] = __fmul_rn(__uint_as_float(b[i]), inv);
          }
          f4* op = reinterpret_cast<f4*>(out) + 2 * v;
          st<true>(op, oa);
          st<true>(op + 1, ob);
        }
      } else {
        const u4 a = ld<true>(reinterpret_cast<const u4*>(grad) + v);
#pragma unroll
        for (int i = 0; i < 4; ++i) bad |= half_special(a[i]) | half_special(a[i] >> 16);
        if constexpr (WRITE) {
          const h8 hv = __builtin_bit_cast(h8, a);
          f4 oa, ob;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            oa[i] = __fmul_rn((float)hv[i], inv);
            ob[i] = __fmul_rn((float)hv[4 + i], inv);
          }
          f4* op = reinterpret_cast<f4*>(out) + 2 * v;
          st<true>(op, oa);
          st<true>(op + 1, ob);
        }
      }
    }
  }
  // scalar path: the whole buffer when unaligned, else the < 8 element tail
  for (size_t i = done + tid; i < n; i += stride) {
    float x;
    if constexpr (G32) {
      const uint32_t u = reinterpret_cast<const uint32_t*>(grad)[i];
      bad |= float_special(u);
      x = __uint_as_float(u);
    } else {
      const uint16_t u = reinterpret_cast<const uint16_t*>(grad)[i];
      bad |= half_special(u);
      x = (float)__builtin_bit_cast(_Float16, u);
    }
    if constexpr (WRITE) out[i] = __fmul_rn(x, inv);
  }
  const unsigned long long vote = __builtin_amdgcn_ballot_w64(bad);
  if (vote != 0ull && (threadIdx.x & 63) == 0) atomicOr(flag, 1u);
}

__global__ void k_scaler_update(mpt_scaler* __restrict__ s, uint32_t* __restrict__ flag) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  float scale = s->scale;
  int good = s->good_steps;
  if (*flag != 0u) {
    scale = fmaxf(__fmul_rn(scale, s->backoff), s->min_scale);
    good = 0;
  } else {
    good += 1;
    if (good == s->growth_interval) {
      scale = fminf(__fmul_rn(scale, s->growth), s->max_scale);
      good = 0;
    }
  }
  s->scale = scale;
  s->inv_scale = div_rn(1.0f, scale);
  s->good_steps = good;
  *flag = 0u;
}

__global__ __launch_bounds__(kThreads) void k_relu_fwd(size_t n, const uint16_t* __restrict__ y, uint16_t* __restrict__ h, bool vec) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  size_t done = 0;
  if (vec) {
    const size_t nvec = n >> 3;
    done = nvec << 3;
    for (size_t v = tid; v < nvec; v += stride) {
      h8 a = reinterpret_cast<const h8*>(y)[v];
#pragma unroll
      for (int i = 0; i < 8; ++i) a[i] = a[i] > (_Float16)0 ? a[i] : (_Float16)0;
      reinterpret_cast<h8*>(h)[v] = a;
    }
  }
  for (size_t i = done + tid; i < n; i += stride) {
    const _Float16 a = reinterpret_cast<const _Float16*>(y)[i];
    reinterpret_cast<_Float16*>(h)[i] = a > (_Float16)0 ? a : (_Float16)0;
  }
}

// out = rne16(float(a) + float(b)): the sum of two FP16 values is exact in FP32, so this is one rounding of the exact sum
__global__ __launch_bounds__(kThreads) void k_add_fp16(size_t n, const uint16_t* __restrict__ a, const uint16_t* __restrict__ b,
                                                        uint16_t* __restrict__ out, bool vec) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  size_t done = 0;
  if (vec) {
    const size_t nvec = n >> 3;
    done = nvec << 3;
    for (size_t v = tid; v < nvec; v += stride) {
      const h8 x = reinterpret_cast<const h8*>(a)[v];
      const h8 y = reinterpret_cast<const h8*>(b)[v];
      h8 r;
#pragma unroll
      for (int i = 0; i < 8; ++i) r[i] = (_Float16)__fadd_rn((float)x[i], (float)y[i]);
      reinterpret_cast<h8*>(out)[v] = r;
    }
  }
  for (size_t i = done + tid; i < n; i += stride)
    reinterpret_cast<_Float16*>(out)[i] = (_Float16)__fadd_rn((float)reinterpret_cast<const _Float16*>(a)[i], (float)reinterpret_cast<const _Float16*>(b)[i]);
}

__global__ __launch_bounds__(kThreads) void k_relu_bwd(size_t n, const uint16_t* __restrict__ dh, const uint16_t* __restrict__ y,
                                                        uint16_t* __restrict__ dy, bool vec) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  size_t done = 0;
  if (vec) {
    const size_t nvec = n >> 3;
    done = nvec << 3;
    for (size_t v = tid; v < nvec; v += stride) {
      const h8 a = reinterpret_cast<const h8*>(y)[v];
      h8 d = reinterpret_cast<const h8*>(dh)[v];
#pragma unroll
      for (int i = 0; i < 8; ++i) d[i] = a[i] > (_Float16)0 ? d[i] : (_Float16)0;
      reinterpret_cast<h8*>(dy)[v] = d;
    }
  }
  for (size_t i = done + tid; i < n; i += stride) {
    const _Float16 a = reinterpret_cast<const _Float16*>(y)[i];
    const _Float16 d = reinterpret_cast<const _Float16*>(dh)[i];
    reinterpret_cast<_Float16*>(dy)[i] = a > (_Float16)0 ? d : (_Float16)0;
  }
}

typedef _Float16 sm_h2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = __fadd_rn(v, __shfl_xor(v, o, 64));
  return v;
}

// Softmax cross-entropy with the loss scale folded into the gradient: FP16 logits in, FP32 max / sum / probabilities,
// FP16 scaled gradient out, FP32 loss of the row out.  A row is held in registers between its single read and its
// single write (4 bytes of traffic per element): WAVES wavefronts per row, NCH 16-byte chunks per lane, so a row of
// up to WAVES*64*8*NCH classes (65536 at most; the row stays packed in FP16 and the exponential is evaluated twice).
// Exponentials use the hardware 2^x (about 1 ulp of FP32, far inside one FP16 step).
template <int WAVES, int NCH, bool VEC>
__global__ __launch_bounds__((WAVES * 64 > kThreads ? WAVES * 64 : kThreads)) void k_softmax_xent_rows(
    int64_t B, int64_t C, const uint16_t* __restrict__ logits, int64_t ldl, const int32_t* __restrict__ labels,
    float factor, uint16_t* __restrict__ dlogits, int64_t ldd, float* __restrict__ row_loss, bool stream) {
  constexpr int NT = WAVES * 64 > kThreads ? WAVES * 64 : kThreads;   // threads per workgroup
  constexpr int T = 64 * WAVES;                                        // threads per row
  __shared__ float red[NT / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rslot = wave / WAVES, tr = threadIdx.x - rslot * T;
  const int64_t row = (int64_t)blockIdx.x * (NT / T) + rslot;
  const bool live = row < B;
  const _Float16* z = reinterpret_cast<const _Float16*>(logits) + (live ? row : 0) * ldl;
  h8 q[NCH];                                                           // the row stays packed; padding is -inf
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int64_t c0 = ((int64_t)i * T + tr) * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) q[i][e] = (_Float16)(-INFINITY);
    if constexpr (VEC) {
      if (live && c0 < C) q[i] = stream ? __builtin_nontemporal_load(reinterpret_cast<const h8*>(z + c0)) : *reinterpret_cast<const h8*>(z + c0);
    } else {
      // no branch around a load: every lane reads some element of the row (its own, or the row's last) and keeps it only
      // if the element exists - behind branches the eight loads would go out one after the other, each waited for
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const _Float16 v = z[min(c0 + e, C - 1)];
        if (live && c0 + e < C) q[i][e] = v;
      }
    }
    // row maximum on packed pairs (one instruction per two elements), widened once per chunk
    sm_h2 m2 = __builtin_elementwise_max(sm_h2{q[i][0], q[i][1]}, sm_h2{q[i][2], q[i][3]});
    m2 = __builtin_elementwise_max(m2, __builtin_elementwise_max(sm_h2{q[i][4], q[i][5]}, sm_h2{q[i][6], q[i][7]}));
    mx = fmaxf(mx, fmaxf((float)m2[0], (float)m2[1]));
  }
  auto across = [&](float x, bool is_max) {                // over the row's wavefronts, fixed order
    x = is_max ? wave_max(x) : wave_sum(x);
    if constexpr (WAVES > 1) {
      __syncthreads();
      if (lane == 0) red[wave] = x;
      __syncthreads();
      float t = red[rslot * WAVES];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) t = is_max ? fmaxf(t, red[rslot * WAVES + w]) : __fadd_rn(t, red[rslot * WAVES + w]);
      x = t;
    }
    return x;
  };
  mx = across(mx, true);
  constexpr float kLog2e = 1.44269504088896340736f;
  // exp(z - max) = 2^(z * log2(e) - max * log2(e)), one fused multiply-add (rounded once, so at least as accurate as
  // the two-operation form); exp(-inf) = 0 for the padding
  const float nmx = -__fmul_rn(mx, kLog2e);
  auto ex = [&](_Float16 h) { return __builtin_amdgcn_exp2f(__builtin_fmaf((float)h, kLog2e, nmx)); };
  // With few chunks per lane the exponentials are kept in registers for the output pass (the kernel is close to
  // ALU-bound, so the instruction count per element is kept down: packed maximum, fused exponent argument, one
  // multiplication per stored value, the label's element handled apart); with many they are recomputed.
  constexpr bool KEEP = NCH <= 4;
  float ev[KEEP ? NCH : 1][8];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x = ex(q[i][e]);
      if constexpr (KEEP) ev[i][e] = x;
      sum = __fadd_rn(sum, x);
    }
  sum = across(sum, false);
  if (!live) return;
  const int32_t lab = min(max(labels[row], 0), (int32_t)(C - 1));      // a label outside [0, C) is the caller's error; it must not become a wild read
  const float inv = div_rn(1.0f, sum);
  const float scale_all = __fmul_rn(inv, factor);                        // every element but the label's: p * factor in one multiplication
  _Float16* d = reinterpret_cast<_Float16*>(dlogits) + row * ldd;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int64_t c0 = ((int64_t)i * T + tr) * 8;
    h8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x;
      if constexpr (KEEP) x = ev[i][e];
      else x = ex(q[i][e]);
      o[e] = (_Float16)__fmul_rn(x, scale_all);
    }
    if (lab >= c0 && lab < c0 + 8) {                                     // one chunk of the row holds the label: (p - 1) * factor there
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (c0 + e == lab) {
          float x;
          if constexpr (KEEP) x = ev[i][e];
          else x = ex(q[i][e]);
          o[e] = (_Float16)__fmul_rn(__fsub_rn(__fmul_rn(x, inv), 1.0f), factor);
        }
    }
    if constexpr (VEC) {
      if (c0 < C) {
        if (stream) __builtin_nontemporal_store(o, reinterpret_cast<h8*>(d + c0));
        else *reinterpret_cast<h8*>(d + c0) = o;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (c0 + e < C) d[c0 + e] = o[e];
    }
  }
  if (row_loss != nullptr && tr == 0) {
    // -log p[label] = log(sum) - (z[label] - max)
    row_loss[row] = __fsub_rn(logf(sum), __fsub_rn((float)z[lab], mx));
  }
}

// Rows too long to hold in registers: one workgroup of 1024 threads per row, three passes over the row (the
// re-reads come from cache), 16-byte accesses when the row allows.
template <bool VEC>
__global__ __launch_bounds__(1024) void k_softmax_xent_long(
    int64_t B, int64_t C, const uint16_t* __restrict__ logits, int64_t ldl, const int32_t* __restrict__ labels,
    float factor, uint16_t* __restrict__ dlogits, int64_t ldd, float* __restrict__ row_loss) {
  constexpr int NT = 1024, W = VEC ? 8 : 1;
  __shared__ float red[NT / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = blockIdx.x;
  const _Float16* z = reinterpret_cast<const _Float16*>(logits) + row * ldl;
  auto across = [&](float x, bool is_max) {
    x = is_max ? wave_max(x) : wave_sum(x);
    __syncthreads();
    if (lane == 0) red[wave] = x;
    __syncthreads();
    float t = red[0];
    for (int w = 1; w < NT / 64; ++w) t = is_max ? fmaxf(t, red[w]) : __fadd_rn(t, red[w]);
    return t;
  };
  auto fetch = [&](int64_t c, float (&v)[W]) {
    if constexpr (VEC) {
      const h8 q = *reinterpret_cast<const h8*>(z + c);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (float)q[e];
    } else {
      v[0] = (float)z[c];
    }
  };
  float mx = -INFINITY;
  for (int64_t c = (int64_t)threadIdx.x * W; c < C; c += (int64_t)NT * W) {
    float v[W];
    fetch(c, v);
#pragma unroll
    for (int e = 0; e < W; ++e) mx = fmaxf(mx, v[e]);
  }
  mx = across(mx, true);
  constexpr float kLog2e = 1.44269504088896340736f;
  float sum = 0.f;
  for (int64_t c = (int64_t)threadIdx.x * W; c < C; c += (int64_t)NT * W) {
    float v[W];
    fetch(c, v);
#pragma unroll
    for (int e = 0; e < W; ++e) sum = __fadd_rn(sum, __builtin_amdgcn_exp2f(__fmul_rn(__fsub_rn(v[e], mx), kLog2e)));
  }
  sum = across(sum, false);
  const int32_t lab = min(max(labels[row], 0), (int32_t)(C - 1));      // a label outside [0, C) is the caller's error; it must not become a wild read
  const float inv = div_rn(1.0f, sum);
  _Float16* d = reinterpret_cast<_Float16*>(dlogits) + row * ldd;
  for (int64_t c = (int64_t)threadIdx.x * W; c < C; c += (int64_t)NT * W) {
    float v[W];
    fetch(c, v);
    _Float16 o[W];
#pragma unroll
    for (int e = 0; e < W; ++e) {
      const float p = __fmul_rn(__builtin_amdgcn_exp2f(__fmul_rn(__fsub_rn(v[e], mx), kLog2e)), inv);
      o[e] = (_Float16)__fmul_rn(__fsub_rn(p, c + e == lab ? 1.0f : 0.0f), factor);
    }
    if constexpr (VEC) {
      h8 q;
#pragma unroll
      for (int e = 0; e < 8; ++e) q[e] = o[e];
      *reinterpret_cast<h8*>(d + c) = q;
    } else {
      d[c] = o[0];
    }
  }
  if (row_loss != nullptr && threadIdx.x == 0) row_loss[row] = __fsub_rn(logf(sum), __fsub_rn((float)z[lab], mx));
}

// Mean of the row losses: one workgroup, each thread a strided share in row order, then a fixed-order sum (reproducible).
__global__ __launch_bounds__(kThreads) void k_loss_mean(int64_t B, const float* __restrict__ row_loss, float* __restrict__ loss) {
  __shared__ float part[kThreads];
  float acc = 0.f;
  for (int64_t r = threadIdx.x; r < B; r += kThreads) acc = __fadd_rn(acc, row_loss[r]);
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int w = kThreads / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) part[threadIdx.x] = __fadd_rn(part[threadIdx.x], part[threadIdx.x + w]);
    __syncthreads();
  }
  if (threadIdx.x == 0) loss[0] = div_rn(part[0], (float)B);
}

// Grid size for a streaming pass over `units` thread-trips.
unsigned grid_for(size_t units) {
  static const int per_cu = MPT_TUNABLE("MPT_EW_BLOCKS_PER_CU", 0);   // 0: one trip per thread
  size_t blocks = (units + kThreads - 1) / kThreads;
  if (blocks < 1) blocks = 1;
  if (per_cu > 0) {
    const size_t cap = (size_t)per_cu * 256;
    if (blocks > cap) blocks = cap;
  }
  const size_t hard = 0x7FFFFFFFu;
  return (unsigned)(blocks > hard ? hard : blocks);
}

}  // namespace

extern "C" int mpt_unscale_check(void* stream, const void* grad, int grad_is_fp32, size_t n, float inv_scale,
                                 float* g32_out, uint32_t* flag) {
  if (n == 0) return MPT_OK;
  if (grad == nullptr || flag == nullptr) return MPT_ERR_NULL;
  if (!mpt_finite(inv_scale) || !(inv_scale > 0.f)) return MPT_ERR_ARG;
  const size_t esz = grad_is_fp32 ? 4 : 2;
  if (!mpt_aligned(grad, esz) || !mpt_aligned(flag, 4) || (g32_out && !mpt_aligned(g32_out, 4))) return MPT_ERR_ALIGN;
  const bool vec = mpt_aligned(grad, 16) && (g32_out == nullptr || mpt_aligned(g32_out, 16));
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned grid = grid_for(vec ? (n + 7) / 8 : n);
#define MPT_UC(G, W, V) hipLaunchKernelGGL((k_unscale_check<G, W, V>), dim3(grid), dim3(kThreads), 0, s, grad, n, inv_scale, g32_out, flag)
  const int sel = (grad_is_fp32 ? 4 : 0) | (g32_out ? 2 : 0) | (vec ? 1 : 0);
  switch (sel) {
    case 0: MPT_UC(false, false, false); break;
    case 1: MPT_UC(false, false, true); break;
    case 2: MPT_UC(false, true, false); break;
    case 3: MPT_UC(false, true, true); break;
    case 4: MPT_UC(true, false, false); break;
    case 5: MPT_UC(true, false, true); break;
    case 6: MPT_UC(true, true, false); break;
    default: MPT_UC(true, true, true); break;
  }
#undef MPT_UC
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_master_update(void* stream, size_t n, float* w32, float* m32, const void* grad, int grad_is_fp32,
                                 uint16_t* w16, float inv_scale, const mpt_scaler* scaler, float lr, float momentum,
                                 const uint32_t* flag) {
  if (n == 0) return MPT_OK;
  if (w32 == nullptr || grad == nullptr || w16 == nullptr) return MPT_ERR_NULL;
  if (!mpt_finite(lr) || !mpt_finite(momentum)) return MPT_ERR_ARG;
  if (scaler == nullptr && (!mpt_finite(inv_scale) || !(inv_scale > 0.f))) return MPT_ERR_ARG;
  const size_t gsz = grad_is_fp32 ? 4 : 2;
  if (!mpt_aligned(w32, 4) || (m32 && !mpt_aligned(m32, 4)) || !mpt_aligned(grad, gsz) || !mpt_aligned(w16, 2) ||
      (flag && !mpt_aligned(flag, 4)) || (scaler && !mpt_aligned(scaler, 4)))
    return MPT_ERR_ALIGN;
  const bool vec = mpt_aligned(w32, 8) && (m32 == nullptr || mpt_aligned(m32, 8)) && mpt_aligned(grad, grad_is_fp32 ? 8 : 4) &&
                   mpt_aligned(w16, 4);
  static const bool nt = MPT_TUNABLE("MPT_EW_NONTEMPORAL", 1) != 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool mom = m32 != nullptr;
  const bool g32 = grad_is_fp32 != 0;
  if (vec) {
    const size_t quads = (n + 1) / 2;    // thread-trips: one pair each
#define MPT_MU256(M, G, T)                                                                                                \
  hipLaunchKernelGGL((k_master_update<M, G, T, 256>), dim3(grid_for(quads)), dim3(256), 0, s, n, w32, m32, grad, w16, inv_scale, scaler, lr, momentum, flag)
#ifdef MPT_TUNING
    static const int bs = MPT_TUNABLE("MPT_EW_BLOCK", 256);             // 64 or 256
#define MPT_MU(M, G, T)                                                                                                   \
  do {                                                                                                                    \
    if (bs == 64) {                                                                                                       \
      const size_t blocks = (quads + 63) / 64;                                                                            \
      hipLaunchKernelGGL((k_master_update<M, G, T, 64>), dim3((unsigned)(blocks > 0x7FFFFFFFu ? 0x7FFFFFFFu : blocks)), dim3(64), 0, s, n, w32, m32, \
                         grad, w16, inv_scale, scaler, lr, momentum, flag);                                                 \
    } else {                                                                                                              \
      MPT_MU256(M, G, T);                                                                                                 \
    }                                                                                                                     \
  } while (0)
    const int sel = (mom ? 4 : 0) | (g32 ? 2 : 0) | (nt ? 1 : 0);
    switch (sel) {
      case 0: MPT_MU(false, false, false); break;
      case 1: MPT_MU(false, false, true); break;
      case 2: MPT_MU(false, true, false); break;
      case 3: MPT_MU(false, true, true); break;
      case 4: MPT_MU(true, false, false); break;
      case 5: MPT_MU(true, false, true); break;
      case 6: MPT_MU(true, true, false); break;
      default: MPT_MU(true, true, true); break;
    }
#undef MPT_MU
#else
    (void)nt;                            // nontemporal accesses, 256-thread workgroups
    if (mom) { if (g32) MPT_MU256(true, true, true); else MPT_MU256(true, false, true); }
    else     { if (g32) MPT_MU256(false, true, true); else MPT_MU256(false, false, true); }
#endif
#undef MPT_MU256
  } else {
    const unsigned grid = grid_for(n);
#define MPT_MS(M, G) hipLaunchKernelGGL((k_master_update_scalar<M, G>), dim3(grid), dim3(kThreads), 0, s, n, w32, m32, grad, w16, inv_scale, scaler, lr, momentum, flag)
    if (mom) { if (g32) MPT_MS(true, true); else MPT_MS(true, false); }
    else     { if (g32) MPT_MS(false, true); else MPT_MS(false, false); }
#undef MPT_MS
  }
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_master_update_multi(void* stream, int count, const mpt_update_item* items, int grad_is_fp32, float inv_scale,
                                       const mpt_scaler* scaler, float lr, float momentum, const uint32_t* flag) {
  if (count == 0) return MPT_OK;
  if (count < 0) return MPT_ERR_ARG;
  if (items == nullptr) return MPT_ERR_NULL;
  if (!mpt_finite(lr) || !mpt_finite(momentum)) return MPT_ERR_ARG;
  if (scaler == nullptr && (!mpt_finite(inv_scale) || !(inv_scale > 0.f))) return MPT_ERR_ARG;
  if ((flag && !mpt_aligned(flag, 4)) || (scaler && !mpt_aligned(scaler, 4))) return MPT_ERR_ALIGN;
  const size_t gsz = grad_is_fp32 ? 4 : 2;
  int with_mom = 0, live = 0;
  for (int k = 0; k < count; ++k) {          // everything is validated before anything is launched
    const mpt_update_item& t = items[k];
    if (t.n == 0) continue;
    if (t.w32_dev == nullptr || t.grad_dev == nullptr || t.w16_dev == nullptr) return MPT_ERR_NULL;
    if (!mpt_aligned(t.w32_dev, 4) || (t.m32_dev && !mpt_aligned(t.m32_dev, 4)) || !mpt_aligned(t.grad_dev, gsz) || !mpt_aligned(t.w16_dev, 2))
      return MPT_ERR_ALIGN;
    if (t.n > ((size_t)1 << 40)) return MPT_ERR_SHAPE;
    ++live;
    with_mom += t.m32_dev != nullptr;
  }
  if (live == 0) return MPT_OK;
  if (with_mom != 0 && with_mom != live) return MPT_ERR_ARG;      // momentum buffers for all tensors or for none
  const bool mom = with_mom != 0, g32 = grad_is_fp32 != 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  MultiItems it;
  auto flush = [&](int filled) -> int {
    if (filled == 0) return MPT_OK;
    it.count = filled;
    const unsigned grid = it.first_block[filled];
#define MPT_MM(M, G) hipLaunchKernelGGL((k_master_update_multi<M, G>), dim3(grid), dim3(kThreads), 0, s, it, inv_scale, scaler, lr, momentum, flag)
    if (mom) { if (g32) MPT_MM(true, true); else MPT_MM(true, false); }
    else     { if (g32) MPT_MM(false, true); else MPT_MM(false, false); }
#undef MPT_MM
    MPT_LAUNCH_CHECK();
    return MPT_OK;
  };
  int filled = 0;
  it.first_block[0] = 0; it.pairs_mask_lo = it.pairs_mask_hi = 0;
  for (int k = 0; k < count; ++k) {
    const mpt_update_item& t = items[k];
    if (t.n == 0) continue;
    const bool pairs = mpt_aligned(t.w32_dev, 8) && (t.m32_dev == nullptr || mpt_aligned(t.m32_dev, 8)) &&
                       mpt_aligned(t.grad_dev, g32 ? 8 : 4) && mpt_aligned(t.w16_dev, 4);
    const size_t units = pairs ? (t.n + 1) / 2 : t.n;
    const size_t blocks = (units + kThreads - 1) / kThreads;
    if (filled == kMultiMax || (size_t)it.first_block[filled] + blocks > 0x7FFFFFFFu) {
      const int st = flush(filled);
      if (st != MPT_OK) return st;
      filled = 0; it.first_block[0] = 0; it.pairs_mask_lo = it.pairs_mask_hi = 0;
    }
    if (blocks > 0x7FFFFFFFu) return MPT_ERR_SHAPE;
    it.w32[filled] = t.w32_dev; it.m32[filled] = t.m32_dev; it.grad[filled] = t.grad_dev; it.w16[filled] = t.w16_dev;
    it.n[filled] = (unsigned long long)t.n;
    it.first_block[filled + 1] = it.first_block[filled] + (unsigned)blocks;
    if (pairs) { if (filled < 32) it.pairs_mask_lo |= 1u << filled; else it.pairs_mask_hi |= 1u << (filled - 32); }
    ++filled;
  }
  return flush(filled);
}

extern "C" int mpt_master_update_fused(void* stream, size_t n, const float* w_in, const float* m_in, const void* grad, int grad_is_fp32,
                                       float* w_out, float* m_out, uint16_t* h_out, float inv_scale, const mpt_scaler* scaler,
                                       float lr, float momentum, uint32_t* flag) {
  if (n == 0) return MPT_OK;
  if (w_in == nullptr || grad == nullptr || w_out == nullptr || h_out == nullptr || flag == nullptr) return MPT_ERR_NULL;
  if ((m_in == nullptr) != (m_out == nullptr)) return MPT_ERR_ARG;
  if (!mpt_finite(lr) || !mpt_finite(momentum)) return MPT_ERR_ARG;
  if (scaler == nullptr && (!mpt_finite(inv_scale) || !(inv_scale > 0.f))) return MPT_ERR_ARG;
  auto overlap = [n](const float* a, const float* b) { return a != nullptr && b != nullptr && a < b + n && b < a + n; };
  if (overlap(w_in, w_out) || overlap(m_in, m_out) || overlap(w_in, m_out) || overlap(m_in, w_out)) return MPT_ERR_ARG;
  const size_t gsz = grad_is_fp32 ? 4 : 2;
  if (!mpt_aligned(w_in, 4) || !mpt_aligned(w_out, 4) || (m_in && (!mpt_aligned(m_in, 4) || !mpt_aligned(m_out, 4))) ||
      !mpt_aligned(grad, gsz) || !mpt_aligned(h_out, 2) || !mpt_aligned(flag, 4) || (scaler && !mpt_aligned(scaler, 4)))
    return MPT_ERR_ALIGN;
  const bool pairs = mpt_aligned(w_in, 8) && mpt_aligned(w_out, 8) && (m_in == nullptr || (mpt_aligned(m_in, 8) && mpt_aligned(m_out, 8))) &&
                     mpt_aligned(grad, grad_is_fp32 ? 8 : 4) && mpt_aligned(h_out, 4);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned grid = grid_for(pairs ? (n + 1) / 2 : n);
#define MPT_MF(M, G, P) hipLaunchKernelGGL((k_master_update_fused<M, G, P>), dim3(grid), dim3(kThreads), 0, s, n, w_in, m_in, grad, w_out, m_out, h_out, inv_scale, scaler, lr, momentum, flag)
  const int sel = (m_in ? 4 : 0) | (grad_is_fp32 ? 2 : 0) | (pairs ? 1 : 0);
  switch (sel) {
    case 0: MPT_MF(false, false, false); break;
    case 1: MPT_MF(false, false, true); break;
    case 2: MPT_MF(false, true, false); break;
    case 3: MPT_MF(false, true, true); break;
    case 4: MPT_MF(true, false, false); break;
    case 5: MPT_MF(true, false, true); break;
    case 6: MPT_MF(true, true, false); break;
    default: MPT_MF(true, true, true); break;
  }
#undef MPT_MF
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_loss_scale_update_dev(void* stream, mpt_scaler* s_dev, uint32_t* flag) {
  if (s_dev == nullptr || flag == nullptr) return MPT_ERR_NULL;
  if (!mpt_aligned(s_dev, 4) || !mpt_aligned(flag, 4)) return MPT_ERR_ALIGN;
  hipLaunchKernelGGL(k_scaler_update, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), s_dev, flag);
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_add_fp16(void* stream, size_t n, const uint16_t* a, const uint16_t* b, uint16_t* out) {
  if (n == 0) return MPT_OK;
  if (a == nullptr || b == nullptr || out == nullptr) return MPT_ERR_NULL;
  if (!mpt_aligned(a, 2) || !mpt_aligned(b, 2) || !mpt_aligned(out, 2)) return MPT_ERR_ALIGN;
  const bool vec = mpt_aligned(a, 16) && mpt_aligned(b, 16) && mpt_aligned(out, 16);
  hipLaunchKernelGGL(k_add_fp16, dim3(grid_for(vec ? (n + 7) / 8 : n)), dim3(kThreads), 0, static_cast<hipStream_t>(stream), n, a, b, out, vec);
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_relu_fwd(void* stream, size_t n, const uint16_t* y, uint16_t* h) {
  if (n == 0) return MPT_OK;
  if (y == nullptr || h == nullptr) return MPT_ERR_NULL;
  if (!mpt_aligned(y, 2) || !mpt_aligned(h, 2)) return MPT_ERR_ALIGN;
  const bool vec = mpt_aligned(y, 16) && mpt_aligned(h, 16);
  hipLaunchKernelGGL(k_relu_fwd, dim3(grid_for(vec ? (n + 7) / 8 : n)), dim3(kThreads), 0, static_cast<hipStream_t>(stream), n, y, h, vec);
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_relu_bwd(void* stream, size_t n, const uint16_t* dh, const uint16_t* y, uint16_t* dy) {
  if (n == 0) return MPT_OK;
  if (dh == nullptr || y == nullptr || dy == nullptr) return MPT_ERR_NULL;
  if (!mpt_aligned(dh, 2) || !mpt_aligned(y, 2) || !mpt_aligned(dy, 2)) return MPT_ERR_ALIGN;
  const bool vec = mpt_aligned(dh, 16) && mpt_aligned(y, 16) && mpt_aligned(dy, 16);
  hipLaunchKernelGGL(k_relu_bwd, dim3(grid_for(vec ? (n + 7) / 8 : n)), dim3(kThreads), 0, static_cast<hipStream_t>(stream), n, dh, y, dy, vec);
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_softmax_xent_scaled(void* stream, int64_t B, int64_t C, const uint16_t* logits, int64_t ldl,
                                       const int32_t* labels, float scale, float* loss, float* row_loss, uint16_t* dlogits, int64_t ldd) {
  if (logits == nullptr || labels == nullptr || dlogits == nullptr || (loss != nullptr && row_loss == nullptr)) return MPT_ERR_NULL;
  if (B < 1 || C < 1 || C > (1 << 24) || B > 0x7FFFFFFF || ldl < C || ldd < C) return MPT_ERR_SHAPE;
  if (!mpt_finite(scale) || !(scale > 0.f)) return MPT_ERR_ARG;
  if (!mpt_aligned(logits, 2) || !mpt_aligned(dlogits, 2) || !mpt_aligned(labels, 4) || (loss && !mpt_aligned(loss, 4)) ||
      (row_loss && !mpt_aligned(row_loss, 4)))
    return MPT_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const float factor = scale / (float)B;
  const bool vec = mpt_aligned(logits, 16) && mpt_aligned(dlogits, 16) && (ldl % 8) == 0 && (ldd % 8) == 0 && (C % 8) == 0;
  const bool nontemporal = B * C * 2 > (192LL << 20);   // beyond the memory-side cache
#define MPT_SM_LAUNCH(WAVES, NCH)                                                                                                   \
  do {                                                                                                                              \
    constexpr unsigned nt = WAVES * 64 > kThreads ? WAVES * 64 : kThreads;                                                          \
    const unsigned rows = nt / (64 * WAVES);                                                                                        \
    const unsigned grid = (unsigned)((B + rows - 1) / rows);                                                                        \
    if (vec) hipLaunchKernelGGL((k_softmax_xent_rows<WAVES, NCH, true>), dim3(grid), dim3(nt), 0, s, B, C, logits, ldl, labels,     \
                                factor, dlogits, ldd, row_loss, nontemporal);                                                       \
    else hipLaunchKernelGGL((k_softmax_xent_rows<WAVES, NCH, false>), dim3(grid), dim3(nt), 0, s, B, C, logits, ldl, labels,        \
                            factor, dlogits, ldd, row_loss, nontemporal);                                                           \
  } while (0)
  if (C <= 512) MPT_SM_LAUNCH(1, 1);
  else if (C <= 2048) MPT_SM_LAUNCH(1, 4);
  else if (C <= 8192) MPT_SM_LAUNCH(4, 4);
  else if (C <= 32768) MPT_SM_LAUNCH(16, 4);      // measured: 16 wavefronts x 4 chunks 5.0 TB/s, 4 x 16 4.4 TB/s
  else if (C <= 65536) MPT_SM_LAUNCH(16, 8);
  else if (vec) hipLaunchKernelGGL(k_softmax_xent_long<true>, dim3((unsigned)B), dim3(1024), 0, s, B, C, logits, ldl, labels, factor, dlogits, ldd, row_loss);
  else hipLaunchKernelGGL(k_softmax_xent_long<false>, dim3((unsigned)B), dim3(1024), 0, s, B, C, logits, ldl, labels, factor, dlogits, ldd, row_loss);
#undef MPT_SM_LAUNCH
  MPT_LAUNCH_CHECK();
  if (loss != nullptr) {
    hipLaunchKernelGGL(k_loss_mean, dim3(1), dim3(kThreads), 0, s, B, row_loss, loss);
    MPT_LAUNCH_CHECK();
  }
  return MPT_OK;
}
