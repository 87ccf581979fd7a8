// Master-weight optimizers beyond heavy-ball SGD, and gradient statistics, for gfx950.
//   * k_optimizer_update: momentum / Nesterov / Adagrad / Adam on the unscaled FP32 gradient, optional weight decay,
//     FP32 state, FP16 copy of the new master in the same pass, skipped as a whole on overflow (paper Sec. 3.1, 3.2;
//     the optimizers are the ones Sec. 4 trains with).  Same access shape as the momentum kernel: 2 consecutive
//     elements per thread, nontemporal, one trip per thread.  Every FP32 operation rounds on its own.
//   * k_grad_stats: exponent histogram, zero / special counts and largest finite magnitude of an FP16 gradient
//     buffer (Sec. 3.2: how a constant loss scale is chosen).  Integer counting, so results are order-independent.
#include "mpt_internal.h"

typedef _Float16 oh2 __attribute__((ext_vector_type(2)));
typedef float of2 __attribute__((ext_vector_type(2)));
typedef uint32_t ou4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kBS = 256;

struct OptP { float lr, mu, b2, eps, wd, omb1, omb2, bc1, bc2; };

// One element.  a: momentum / Adagrad sum / Adam first moment; b: Adam second moment.
template <int KIND>
__device__ __forceinline__ float opt_step(float w, float& a, float& b, float graw, float inv, const float* clip, float clipf, const OptP& p) {
  float g = __fmul_rn(graw, inv);
  if (clip != nullptr) g = __fmul_rn(g, clipf);          // clip-by-global-norm factor, after unscaling and before weight decay
  if (p.wd != 0.f) g = __fadd_rn(g, __fmul_rn(p.wd, w));
  if constexpr (KIND == MPT_OPT_MOMENTUM) {
    a = __fadd_rn(__fmul_rn(p.mu, a), g);
    return __fsub_rn(w, __fmul_rn(p.lr, a));
  } else if constexpr (KIND == MPT_OPT_NESTEROV) {
    a = __fadd_rn(__fmul_rn(p.mu, a), g);
    return __fsub_rn(w, __fmul_rn(p.lr, __fadd_rn(g, __fmul_rn(p.mu, a))));
  } else if constexpr (KIND == MPT_OPT_ADAGRAD) {
    a = __fadd_rn(a, __fmul_rn(g, g));
    return __fsub_rn(w, div_rn(__fmul_rn(p.lr, g), __fadd_rn(sqrt_rn(a), p.eps)));
  } else {
    a = __fadd_rn(__fmul_rn(p.mu, a), __fmul_rn(p.omb1, g));
    b = __fadd_rn(__fmul_rn(p.b2, b), __fmul_rn(p.omb2, __fmul_rn(g, g)));
    const float mh = div_rn(a, p.bc1), vh = div_rn(b, p.bc2);
    return __fsub_rn(w, div_rn(__fmul_rn(p.lr, mh), __fadd_rn(sqrt_rn(vh), p.eps)));
  }
}

template <class T> __device__ __forceinline__ T ntl(const T* q) { return __builtin_nontemporal_load(q); }
template <class T> __device__ __forceinline__ void nts(T* q, T v) { __builtin_nontemporal_store(v, q); }

// W = 2: pairs (8-byte FP32 / 4-byte FP16 accesses, arrays aligned accordingly); W = 1: element-wise.
template <int KIND, bool G32, int W>
__global__ __launch_bounds__(kBS) void k_optimizer_update(size_t n, float* __restrict__ w32, float* __restrict__ s1, float* __restrict__ s2,
                                                          const void* __restrict__ grad, uint16_t* __restrict__ w16, float inv_scale,
                                                          const mpt_scaler* __restrict__ scaler, OptP p, const uint32_t* __restrict__ flag,
                                                          const float* __restrict__ clip) {
  constexpr bool TWO = KIND == MPT_OPT_ADAM;
  const size_t units = W == 2 ? (n >> 1) : n;
  const size_t stride = (size_t)gridDim.x * kBS;
  for (size_t q = (size_t)blockIdx.x * kBS + threadIdx.x; q < units; q += stride) {
    float g[W], w[W], a[W], b[W];
    if constexpr (W == 2) {
      if constexpr (G32) { const of2 t = ntl(reinterpret_cast<const of2*>(grad) + q); g[0] = t[0]; g[1] = t[1]; }
      else { const oh2 t = ntl(reinterpret_cast<const oh2*>(grad) + q); g[0] = (float)t[0]; g[1] = (float)t[1]; }
      const of2 tw = ntl(reinterpret_cast<const of2*>(w32) + q); w[0] = tw[0]; w[1] = tw[1];
      const of2 ta = ntl(reinterpret_cast<const of2*>(s1) + q); a[0] = ta[0]; a[1] = ta[1];
      if constexpr (TWO) { const of2 tb = ntl(reinterpret_cast<const of2*>(s2) + q); b[0] = tb[0]; b[1] = tb[1]; }
      else { b[0] = b[1] = 0.f; }
    } else {
      g[0] = G32 ? reinterpret_cast<const float*>(grad)[q] : (float)reinterpret_cast<const _Float16*>(grad)[q];
      w[0] = w32[q]; a[0] = s1[q]; b[0] = TWO ? s2[q] : 0.f;
    }
    // flag and scale are read after the vector loads are in flight; nothing is stored before the flag is seen
    if (flag != nullptr && *flag != 0u) return;
    const float inv = scaler != nullptr ? scaler->inv_scale : inv_scale;
    const float clipf = clip != nullptr ? *clip : 1.f;
#pragma unroll
    for (int i = 0; i < W; ++i) w[i] = opt_step<KIND>(w[i], a[i], b[i], g[i], inv, clip, clipf, p);
    if constexpr (W == 2) {
      nts(reinterpret_cast<of2*>(w32) + q, of2{w[0], w[1]});
      nts(reinterpret_cast<of2*>(s1) + q, of2{a[0], a[1]});
      if constexpr (TWO) nts(reinterpret_cast<of2*>(s2) + q, of2{b[0], b[1]});
      nts(reinterpret_cast<oh2*>(w16) + q, oh2{(_Float16)w[0], (_Float16)w[1]});
    } else {
      w32[q] = w[0]; s1[q] = a[0];
      if constexpr (TWO) s2[q] = b[0];
      reinterpret_cast<_Float16*>(w16)[q] = (_Float16)w[0];
    }
  }
  if (W == 2 && (n & 1) && blockIdx.x == 0 && threadIdx.x == 0) {      // odd tail
    if (flag != nullptr && *flag != 0u) return;
    const float inv = scaler != nullptr ? scaler->inv_scale : inv_scale;
    const size_t i = n - 1;
    const float graw = G32 ? reinterpret_cast<const float*>(grad)[i] : (float)reinterpret_cast<const _Float16*>(grad)[i];
    float a = s1[i], b = TWO ? s2[i] : 0.f;
    const float w = opt_step<KIND>(w32[i], a, b, graw, inv, clip, clip != nullptr ? *clip : 1.f, p);
    w32[i] = w; s1[i] = a;
    if constexpr (TWO) s2[i] = b;
    reinterpret_cast<_Float16*>(w16)[i] = (_Float16)w;
  }
}

template <int KIND>
int launch_opt(hipStream_t st, size_t n, float* w32, float* s1, float* s2, const void* grad, int g32, uint16_t* w16, float inv,
               const mpt_scaler* scaler, const OptP& p, const uint32_t* flag, const float* clip) {
  const bool vec = mpt_aligned(w32, 8) && mpt_aligned(s1, 8) && (s2 == nullptr || mpt_aligned(s2, 8)) && mpt_aligned(w16, 4) &&
                   mpt_aligned(grad, g32 ? 8 : 4);
  const size_t units = vec ? (n >> 1) : n;
  size_t blocks = (units + kBS - 1) / kBS;
  if (blocks < 1) blocks = 1;
  if (blocks > 0x7FFFFFFFu) blocks = 0x7FFFFFFFu;
  const dim3 grid((unsigned)blocks);
  if (vec) {
    if (g32) hipLaunchKernelGGL((k_optimizer_update<KIND, true, 2>), grid, dim3(kBS), 0, st, n, w32, s1, s2, grad, w16, inv, scaler, p, flag, clip);
    else hipLaunchKernelGGL((k_optimizer_update<KIND, false, 2>), grid, dim3(kBS), 0, st, n, w32, s1, s2, grad, w16, inv, scaler, p, flag, clip);
  } else {
    if (g32) hipLaunchKernelGGL((k_optimizer_update<KIND, true, 1>), grid, dim3(kBS), 0, st, n, w32, s1, s2, grad, w16, inv, scaler, p, flag, clip);
    else hipLaunchKernelGGL((k_optimizer_update<KIND, false, 1>), grid, dim3(kBS), 0, st, n, w32, s1, s2, grad, w16, inv, scaler, p, flag, clip);
  }
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

// ---------------------------------------------------------------- gradient statistics
constexpr int kBins = 42;

typedef _Float16 sh2 __attribute__((ext_vector_type(2)));
typedef short ss2 __attribute__((ext_vector_type(2)));
typedef unsigned short su2 __attribute__((ext_vector_type(2)));

// bin of one FP16 value: 0 zero; 1 + (e + 24) for floor(log2 |g|) = e in -24 .. 15; 41 Inf / NaN.  The conversion
// to FP32 normalises FP16 subnormals, so the FP32 exponent field is e + 127 for every finite non-zero value,
// 0 for zeros and 255 for Inf / NaN; clamping (field - 102) to [0, 41] gives the bin.
__device__ __forceinline__ int stat_bin(_Float16 h) {
  const int field = (int)((__float_as_uint((float)h) >> 23) & 0xFFu);
  return min(max(field - 102, 0), 41);
}

// Every thread counts into its own column of an LDS table [42][256] (conflict-free: the bank is the thread), 16-byte
// vectors, eight in flight per thread, grid-stride; a workgroup then adds its 42 totals to the global histogram.  The largest finite magnitude
// is kept per lane as packed 16-bit values biased by 0x0400, so that Inf / NaN (>= 0x7C00) turn negative and drop
// out of a signed maximum; it travels as its bit pattern (order-preserving for magnitudes).
template <bool VEC>
__global__ __launch_bounds__(kBS) void k_grad_stats(const uint16_t* __restrict__ g, size_t n, unsigned long long* __restrict__ hist,
                                                    uint32_t* __restrict__ absmax_bits) {
  __shared__ uint32_t table[kBins][kBS];
  __shared__ uint32_t lmax;
  for (int b = 0; b < kBins; ++b) table[b][threadIdx.x] = 0u;
  if (threadIdx.x == 0) lmax = 0u;
  __syncthreads();
  ss2 mx = {0x0400, 0x0400};
  const size_t stride = (size_t)gridDim.x * kBS, tid = (size_t)blockIdx.x * kBS + threadIdx.x;
  auto two = [&](uint32_t q) {
    const sh2 h = __builtin_bit_cast(sh2, q);
    atomicAdd(&table[stat_bin(h[0])][threadIdx.x], 1u);
    atomicAdd(&table[stat_bin(h[1])][threadIdx.x], 1u);
    const su2 mag = __builtin_bit_cast(su2, q & 0x7FFF7FFFu) + su2{0x0400, 0x0400};
    const ss2 t = __builtin_bit_cast(ss2, mag);
    mx[0] = max(mx[0], t[0]);
    mx[1] = max(mx[1], t[1]);
  };
  size_t done = 0;
  if constexpr (VEC) {
    const size_t nvec = n >> 3;
    done = nvec << 3;
    // eight vectors in flight per thread: with 12 wavefronts per CU (the table takes 42 KiB of LDS per workgroup) one
    // 16-byte load per thread at a time leaves the memory system idle most of the time
    size_t v = tid;
    constexpr int kInFlight = 8;
    for (; v + (kInFlight - 1) * stride < nvec; v += kInFlight * stride) {
      ou4 q[kInFlight];
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) q[u] = __builtin_nontemporal_load(reinterpret_cast<const ou4*>(g) + v + u * stride);
#pragma unroll
      for (int u = 0; u < kInFlight; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) two(q[u][i]);
    }
    for (; v < nvec; v += stride) {
      const ou4 q = __builtin_nontemporal_load(reinterpret_cast<const ou4*>(g) + v);
#pragma unroll
      for (int i = 0; i < 4; ++i) two(q[i]);
    }
  }
  for (size_t i = done + tid; i < n; i += stride) {
    const uint32_t h = g[i];
    atomicAdd(&table[stat_bin(__builtin_bit_cast(_Float16, (uint16_t)h))][threadIdx.x], 1u);
    const short t = (short)((h & 0x7FFFu) + 0x0400u);
    mx[0] = max(mx[0], t);
  }
  const uint32_t mymax = (uint32_t)(max(mx[0], mx[1]) - 0x0400);
  if (mymax != 0u) atomicMax(&lmax, mymax);
  __syncthreads();
  if (threadIdx.x < kBins) {
    uint32_t tot = 0u;
    for (int c = 0; c < kBS; ++c) tot += table[threadIdx.x][(c + threadIdx.x) & (kBS - 1)];     // skewed: distinct banks
    if (tot != 0u) atomicAdd(&hist[threadIdx.x], (unsigned long long)tot);
  }
  if (threadIdx.x == 0 && lmax != 0u) atomicMax(absmax_bits, lmax);
}

// ---------------------------------------------------------------- global gradient norm (for clipping)
// Sum of squares of the unscaled gradient (Sec. 3.2: clipping acts on unscaled values) and the overflow vote, from one
// read of the buffer.  Every element is unscaled with the update's own FP32 multiplication; its square is exact in
// FP64 and is added there (one fused multiply-add per element).  The order of additions is fixed by the launch shape
// alone (which depends only on n and the alignment): each thread walks a fixed set of vectors, lanes are combined
// in a fixed butterfly, wavefronts in index order, and the per-workgroup partials are added in index order by a
// second, single-workgroup kernel - so a buffer gives the same bits every time.
constexpr int kNormBlocks = 2048;        // workgroups of the first pass = partials in the workspace

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

template <bool G32, bool VEC>
__global__ __launch_bounds__(kBS) void k_grad_sumsq(const void* __restrict__ grad, size_t n, float inv_scale, const mpt_scaler* __restrict__ scaler,
                                                    double* __restrict__ partial, uint32_t* __restrict__ flag) {
  __shared__ double wsum[kBS / 64];
  const float inv = scaler != nullptr ? scaler->inv_scale : inv_scale;
  const size_t stride = (size_t)gridDim.x * kBS, tid = (size_t)blockIdx.x * kBS + threadIdx.x;
  double acc = 0.0;
  bool bad = false;
  auto one32 = [&](float raw) {
    bad |= (__float_as_uint(raw) & 0x7F800000u) == 0x7F800000u;
    const double g = (double)__fmul_rn(raw, inv);
    acc = __builtin_fma(g, g, acc);
  };
  auto two16 = [&](uint32_t q) {
    bad |= ((q & 0x7C00u) == 0x7C00u) | ((q & 0x7C000000u) == 0x7C000000u);
    const sh2 h = __builtin_bit_cast(sh2, q);
    const double g0 = (double)__fmul_rn((float)h[0], inv), g1 = (double)__fmul_rn((float)h[1], inv);
    acc = __builtin_fma(g0, g0, acc);
    acc = __builtin_fma(g1, g1, acc);
  };
  size_t done = 0;
  if constexpr (VEC) {                              // 16-byte vectors, eight in flight per thread
    constexpr int EPV = G32 ? 4 : 8;
    const size_t nvec = n / EPV;
    done = nvec * EPV;
    constexpr int kInFlight = 8;
    size_t v = tid;
    for (; v + (kInFlight - 1) * stride < nvec; v += kInFlight * stride) {
      ou4 q[kInFlight];
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) q[u] = __builtin_nontemporal_load(reinterpret_cast<const ou4*>(grad) + v + u * stride);
#pragma unroll
      for (int u = 0; u < kInFlight; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if constexpr (G32) one32(__uint_as_float(q[u][i]));
          else two16(q[u][i]);
        }
    }
    for (; v < nvec; v += stride) {
      const ou4 q = __builtin_nontemporal_load(reinterpret_cast<const ou4*>(grad) + v);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (G32) one32(__uint_as_float(q[i]));
        else two16(q[i]);
      }
    }
  }
  for (size_t i = done + tid; i < n; i += stride) {
    if constexpr (G32) {
      one32(reinterpret_cast<const float*>(grad)[i]);
    } else {
      const uint32_t h = reinterpret_cast<const uint16_t*>(grad)[i];
      bad |= (h & 0x7C00u) == 0x7C00u;
      const double g = (double)__fmul_rn((float)__builtin_bit_cast(_Float16, (uint16_t)h), inv);
      acc = __builtin_fma(g, g, acc);
    }
  }
  acc = wave_sum_f64(acc);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
  if (flag != nullptr) {
    const unsigned long long vote = __builtin_amdgcn_ballot_w64(bad);
    if (vote != 0ull && (threadIdx.x & 63) == 0) atomicOr(flag, 1u);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = wsum[0];
#pragma unroll
    for (int w = 1; w < kBS / 64; ++w) t += wsum[w];
    partial[blockIdx.x] = t;
  }
}

// One workgroup: adds the partials in index order (thread t takes partials t, t + 256, ...; then lanes, then
// wavefronts, all in fixed order) and stores or accumulates the total.
__global__ __launch_bounds__(kBS) void k_grad_sumsq_finish(const double* __restrict__ partial, int count, int accumulate, double* __restrict__ sumsq) {
  __shared__ double wsum[kBS / 64];
  double acc = 0.0;
  for (int i = threadIdx.x; i < count; i += kBS) acc += partial[i];
  acc = wave_sum_f64(acc);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = wsum[0];
    for (int w = 1; w < kBS / 64; ++w) t += wsum[w];
    *sumsq = accumulate ? *sumsq + t : t;
  }
}

// factor = 1 if the norm does not exceed max_norm (or is NaN), else the FP64 quotient max_norm / norm rounded once
__global__ void k_clip_factor(const double* __restrict__ sumsq, float max_norm, float* __restrict__ factor, float* __restrict__ norm_out) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const double norm = __builtin_sqrt(*sumsq);
  *factor = norm > (double)max_norm ? (float)((double)max_norm / norm) : 1.f;
  if (norm_out != nullptr) *norm_out = (float)norm;
}

__global__ void k_grad_stats_clear(unsigned long long* hist, uint32_t* absmax_bits) {
  if (threadIdx.x < kBins) hist[threadIdx.x] = 0ull;
  if (threadIdx.x == 0) *absmax_bits = 0u;
}

}  // namespace

extern "C" int mpt_optimizer_update(void* stream, size_t n, int kind, const mpt_opt_params* hp, float* w32, float* state1, float* state2,
                                    const void* grad, int grad_is_fp32, uint16_t* w16, float inv_scale, const mpt_scaler* scaler_dev,
                                    const uint32_t* flag) {
  if (n == 0) return MPT_OK;
  if (hp == nullptr || w32 == nullptr || state1 == nullptr || grad == nullptr || w16 == nullptr) return MPT_ERR_NULL;
  if (kind < MPT_OPT_MOMENTUM || kind > MPT_OPT_ADAM) return MPT_ERR_ARG;
  if (kind == MPT_OPT_ADAM && state2 == nullptr) return MPT_ERR_NULL;
  if (!mpt_finite(hp->lr) || !mpt_finite(hp->momentum) || !mpt_finite(hp->weight_decay) || hp->weight_decay < 0.f) return MPT_ERR_ARG;
  if (scaler_dev == nullptr && (!mpt_finite(inv_scale) || !(inv_scale > 0.f))) return MPT_ERR_ARG;
  if ((kind == MPT_OPT_ADAGRAD || kind == MPT_OPT_ADAM) && (!mpt_finite(hp->eps) || hp->eps < 0.f)) return MPT_ERR_ARG;
  if (kind == MPT_OPT_ADAM && (!mpt_finite(hp->beta2) || !(hp->bias_corr1 > 0.f) || !(hp->bias_corr2 > 0.f) || !mpt_finite(hp->bias_corr1) ||
                               !mpt_finite(hp->bias_corr2) || !mpt_finite(hp->one_minus_beta1) || !mpt_finite(hp->one_minus_beta2)))
    return MPT_ERR_ARG;
  if (!mpt_aligned(w32, 4) || !mpt_aligned(state1, 4) || (state2 && !mpt_aligned(state2, 4)) || !mpt_aligned(w16, 2) ||
      !mpt_aligned(grad, grad_is_fp32 ? 4 : 2) || (flag && !mpt_aligned(flag, 4)) || (scaler_dev && !mpt_aligned(scaler_dev, 4)) ||
      (hp->clip_factor_dev && !mpt_aligned(hp->clip_factor_dev, 4)))
    return MPT_ERR_ALIGN;
  const OptP p{hp->lr, hp->momentum, hp->beta2, hp->eps, hp->weight_decay, hp->one_minus_beta1, hp->one_minus_beta2, hp->bias_corr1, hp->bias_corr2};
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* s2 = kind == MPT_OPT_ADAM ? state2 : nullptr;
  const float* clip = hp->clip_factor_dev;
  switch (kind) {
    case MPT_OPT_MOMENTUM: return launch_opt<MPT_OPT_MOMENTUM>(st, n, w32, state1, s2, grad, grad_is_fp32, w16, inv_scale, scaler_dev, p, flag, clip);
    case MPT_OPT_NESTEROV: return launch_opt<MPT_OPT_NESTEROV>(st, n, w32, state1, s2, grad, grad_is_fp32, w16, inv_scale, scaler_dev, p, flag, clip);
    case MPT_OPT_ADAGRAD: return launch_opt<MPT_OPT_ADAGRAD>(st, n, w32, state1, s2, grad, grad_is_fp32, w16, inv_scale, scaler_dev, p, flag, clip);
    default: return launch_opt<MPT_OPT_ADAM>(st, n, w32, state1, s2, grad, grad_is_fp32, w16, inv_scale, scaler_dev, p, flag, clip);
  }
}

extern "C" int mpt_grad_stats(void* stream, const uint16_t* grad, size_t n, int accumulate, uint64_t* hist, uint32_t* absmax_bits) {
  if (hist == nullptr || absmax_bits == nullptr || (n != 0 && grad == nullptr)) return MPT_ERR_NULL;
  if (!mpt_aligned(hist, 8) || !mpt_aligned(absmax_bits, 4) || (grad && !mpt_aligned(grad, 2))) return MPT_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned long long* h = reinterpret_cast<unsigned long long*>(hist);
  if (!accumulate) {
    hipLaunchKernelGGL(k_grad_stats_clear, dim3(1), dim3(64), 0, st, h, absmax_bits);
    MPT_LAUNCH_CHECK();
  }
  if (n == 0) return MPT_OK;
  const bool vec = mpt_aligned(grad, 16);
  const size_t units = vec ? (n >> 3) + 7 : n;
  size_t blocks = (units + kBS - 1) / kBS;
  if (blocks < 1) blocks = 1;
  if (blocks > 768) blocks = 768;                  // grid-stride beyond: few workgroups, so few global atomics per bin
  if (vec) hipLaunchKernelGGL(k_grad_stats<true>, dim3((unsigned)blocks), dim3(kBS), 0, st, grad, n, h, absmax_bits);
  else hipLaunchKernelGGL(k_grad_stats<false>, dim3((unsigned)blocks), dim3(kBS), 0, st, grad, n, h, absmax_bits);
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" size_t mpt_grad_norm_workspace_bytes(void) { return (size_t)kNormBlocks * sizeof(double); }

extern "C" int mpt_grad_sumsq(void* stream, const void* grad, int grad_is_fp32, size_t n, float inv_scale, const mpt_scaler* scaler_dev,
                              int accumulate, double* sumsq, uint32_t* flag, void* ws, size_t ws_bytes) {
  if (sumsq == nullptr || ws == nullptr || (n != 0 && grad == nullptr)) return MPT_ERR_NULL;
  if (scaler_dev == nullptr && (!mpt_finite(inv_scale) || !(inv_scale > 0.f))) return MPT_ERR_ARG;
  if (!mpt_aligned(sumsq, 8) || !mpt_aligned(ws, 8) || (grad && !mpt_aligned(grad, grad_is_fp32 ? 4 : 2)) || (flag && !mpt_aligned(flag, 4)) ||
      (scaler_dev && !mpt_aligned(scaler_dev, 4)))
    return MPT_ERR_ALIGN;
  if (ws_bytes < mpt_grad_norm_workspace_bytes()) return MPT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  double* partial = reinterpret_cast<double*>(ws);
  int blocks = 0;
  if (n != 0) {
    const bool vec = mpt_aligned(grad, 16);
    const size_t units = vec ? n / (grad_is_fp32 ? 4 : 8) + 7 : n;
    size_t b = (units + (size_t)kBS * 8 - 1) / ((size_t)kBS * 8);    // about eight vectors per thread before the grid stops growing
    if (b < 1) b = 1;
    if (b > (size_t)kNormBlocks) b = kNormBlocks;
    blocks = (int)b;
    if (grad_is_fp32) {
      if (vec) hipLaunchKernelGGL((k_grad_sumsq<true, true>), dim3(blocks), dim3(kBS), 0, st, grad, n, inv_scale, scaler_dev, partial, flag);
      else hipLaunchKernelGGL((k_grad_sumsq<true, false>), dim3(blocks), dim3(kBS), 0, st, grad, n, inv_scale, scaler_dev, partial, flag);
    } else {
      if (vec) hipLaunchKernelGGL((k_grad_sumsq<false, true>), dim3(blocks), dim3(kBS), 0, st, grad, n, inv_scale, scaler_dev, partial, flag);
      else hipLaunchKernelGGL((k_grad_sumsq<false, false>), dim3(blocks), dim3(kBS), 0, st, grad, n, inv_scale, scaler_dev, partial, flag);
    }
    MPT_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(k_grad_sumsq_finish, dim3(1), dim3(kBS), 0, st, partial, blocks, accumulate ? 1 : 0, sumsq);
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_clip_factor(void* stream, const double* sumsq, float max_norm, float* factor, float* norm_out) {
  if (sumsq == nullptr || factor == nullptr) return MPT_ERR_NULL;
  if (!mpt_finite(max_norm) || !(max_norm > 0.f)) return MPT_ERR_ARG;
  if (!mpt_aligned(sumsq, 8) || !mpt_aligned(factor, 4) || (norm_out && !mpt_aligned(norm_out, 4))) return MPT_ERR_ALIGN;
  hipLaunchKernelGGL(k_clip_factor, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), sumsq, max_norm, factor, norm_out);
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}
