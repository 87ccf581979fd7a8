// Pointwise part of an LSTM cell with FP16 tensors and FP32 math (paper Sec. 3.3, "point-wise operations"; the
// recurrent layers of Sec. 4), forward and backward, for gfx950.  The matrix products around it are the GEMM entry
// points.  Gate order (i, f, g, o) along the 4H axis.  A thread owns 8 consecutive hidden units of one batch row:
// every tensor is touched with 16-byte accesses, once.  HBM-bound at large B*H: 30 bytes per hidden unit forward
// (two pre-activation tensors of 4 gates, previous state in; activations, state, output out), 22 bytes backward.
#include "mpt_internal.h"

typedef _Float16 lh8 __attribute__((ext_vector_type(8)));
typedef _Float16 lh4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kT = 256;

__device__ __forceinline__ float sigmoidf_(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
// tanh to a relative error of about 1e-6 (the results are stored as FP16, whose step is 5e-4): (1 - t) / (1 + t) with
// t = exp(-2|x|); below 2^-4, where 1 - t cancels, the odd series x - x^3/3 + 2x^5/15 (next term 3e-9 relative).
// A third of the instructions of the library routine, which matters here: the kernels are within reach of HBM speed.
__device__ __forceinline__ float tanhf_(float x) {
  const float ax = fabsf(x);
  const float t = __expf(-2.0f * ax);
  const float big = (1.0f - t) * __builtin_amdgcn_rcpf(1.0f + t);
  const float x2 = ax * ax;
  const float small = ax * (1.0f + x2 * (-0.33333334f + x2 * 0.13333334f));
  return copysignf(ax < 0.0625f ? small : big, x);
}

// NT: nontemporal accesses, for tensors that outgrow the 256 MB memory-side cache (streaming them is faster there,
// slower for small tensors that the next kernel reads again).
template <int V, bool NT = false>
__device__ __forceinline__ void ld16(const uint16_t* p, float (&v)[V]) {
  if constexpr (V == 8) {
    const lh8 q = NT ? __builtin_nontemporal_load(reinterpret_cast<const lh8*>(p)) : *reinterpret_cast<const lh8*>(p);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)q[e];
  } else if constexpr (V == 4) {
    const lh4 q = NT ? __builtin_nontemporal_load(reinterpret_cast<const lh4*>(p)) : *reinterpret_cast<const lh4*>(p);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = (float)q[e];
  } else {
    v[0] = (float)*reinterpret_cast<const _Float16*>(p);
  }
}
template <int V, bool NT = false>
__device__ __forceinline__ void st16(uint16_t* p, const float (&v)[V]) {
  if constexpr (V == 8) {
    lh8 q;
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] = (_Float16)mpt_rounded_f32(v[e]);
    if constexpr (NT) __builtin_nontemporal_store(q, reinterpret_cast<lh8*>(p));
    else *reinterpret_cast<lh8*>(p) = q;
  } else if constexpr (V == 4) {
    lh4 q;
#pragma unroll
    for (int e = 0; e < 4; ++e) q[e] = (_Float16)mpt_rounded_f32(v[e]);
    if constexpr (NT) __builtin_nontemporal_store(q, reinterpret_cast<lh4*>(p));
    else *reinterpret_cast<lh4*>(p) = q;
  } else {
    *reinterpret_cast<_Float16*>(p) = (_Float16)mpt_rounded_f32(v[0]);
  }
}

template <int V, bool NT>
__global__ __launch_bounds__(kT) void k_lstm_cell_fwd(int64_t B, int64_t H, const uint16_t* __restrict__ gx, int64_t ldgx,
                                                      const uint16_t* __restrict__ gr, int64_t ldgr, const float* __restrict__ bias,
                                                      const uint16_t* cprev, int64_t ldcp, uint16_t* __restrict__ act, int64_t ldact,
                                                      uint16_t* c, int64_t ldc, uint16_t* __restrict__ h, int64_t ldh) {
  const int64_t per_row = H / V;
  const int64_t u = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (u >= B * per_row) return;
  const int64_t b = u / per_row, j = (u - b * per_row) * V;
  float a[4][V], cp[V];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    ld16<V, NT>(gx + b * ldgx + g * H + j, a[g]);
    if (gr != nullptr) {
      float r[V];
      ld16<V, NT>(gr + b * ldgr + g * H + j, r);
#pragma unroll
      for (int e = 0; e < V; ++e) a[g][e] = __fadd_rn(a[g][e], r[e]);
    }
    if (bias != nullptr) {
#pragma unroll
      for (int e = 0; e < V; ++e) a[g][e] = __fadd_rn(a[g][e], bias[g * H + j + e]);
    }
  }
  ld16<V, NT>(cprev + b * ldcp + j, cp);
  float cn[V], hn[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    const float i = sigmoidf_(a[0][e]), f = sigmoidf_(a[1][e]), g = tanhf_(a[2][e]), o = sigmoidf_(a[3][e]);
    a[0][e] = i; a[1][e] = f; a[2][e] = g; a[3][e] = o;
    cn[e] = __fadd_rn(__fmul_rn(f, cp[e]), __fmul_rn(i, g));
    hn[e] = __fmul_rn(o, tanhf_(cn[e]));
  }
#pragma unroll
  for (int g = 0; g < 4; ++g) st16<V, NT>(act + b * ldact + g * H + j, a[g]);
  st16<V, NT>(c + b * ldc + j, cn);
  st16<V, NT>(h + b * ldh + j, hn);
}

template <int V, bool NT>
__global__ __launch_bounds__(kT) void k_lstm_cell_bwd(int64_t B, int64_t H, const uint16_t* __restrict__ dh, int64_t lddh,
                                                      const uint16_t* dcn, int64_t lddcn, const uint16_t* __restrict__ act, int64_t ldact,
                                                      const uint16_t* __restrict__ c, int64_t ldc, const uint16_t* __restrict__ cprev, int64_t ldcp,
                                                      uint16_t* __restrict__ da, int64_t ldda, uint16_t* dcp, int64_t lddcp) {
  const int64_t per_row = H / V;
  const int64_t u = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (u >= B * per_row) return;
  const int64_t b = u / per_row, j = (u - b * per_row) * V;
  float a[4][V], dhv[V], dc[V], cv[V], cp[V];
#pragma unroll
  for (int g = 0; g < 4; ++g) ld16<V, NT>(act + b * ldact + g * H + j, a[g]);
  ld16<V, NT>(dh + b * lddh + j, dhv);
  ld16<V, NT>(c + b * ldc + j, cv);
  ld16<V, NT>(cprev + b * ldcp + j, cp);
  if (dcn != nullptr) {
    ld16<V, NT>(dcn + b * lddcn + j, dc);
  } else {
#pragma unroll
    for (int e = 0; e < V; ++e) dc[e] = 0.f;
  }
  float out[4][V], dprev[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    const float i = a[0][e], f = a[1][e], g = a[2][e], o = a[3][e];
    const float tc = tanhf_(cv[e]);
    const float d = __fadd_rn(__fmul_rn(__fmul_rn(dhv[e], o), __fsub_rn(1.0f, __fmul_rn(tc, tc))), dc[e]);
    out[0][e] = __fmul_rn(__fmul_rn(d, g), __fmul_rn(i, __fsub_rn(1.0f, i)));
    out[1][e] = __fmul_rn(__fmul_rn(d, cp[e]), __fmul_rn(f, __fsub_rn(1.0f, f)));
    out[2][e] = __fmul_rn(__fmul_rn(d, i), __fsub_rn(1.0f, __fmul_rn(g, g)));
    out[3][e] = __fmul_rn(__fmul_rn(dhv[e], tc), __fmul_rn(o, __fsub_rn(1.0f, o)));
    dprev[e] = __fmul_rn(d, f);
  }
#pragma unroll
  for (int g = 0; g < 4; ++g) st16<V, NT>(da + b * ldda + g * H + j, out[g]);
  st16<V, NT>(dcp + b * lddcp + j, dprev);
}

bool vec_ok(const void* p, int64_t ld) { return p == nullptr || (mpt_aligned(p, 16) && (ld % 8) == 0); }
bool dims_ok(int64_t B, int64_t H) { return B >= 1 && H >= 1 && B <= (1LL << 31) && H <= (1LL << 24); }

}  // namespace

extern "C" int mpt_lstm_cell_fwd(void* stream, int64_t B, int64_t H, const uint16_t* gx, int64_t ldgx, const uint16_t* gr, int64_t ldgr,
                                 const float* bias, const uint16_t* c_prev, int64_t ldcp, uint16_t* act, int64_t ldact,
                                 uint16_t* c, int64_t ldc, uint16_t* h, int64_t ldh) {
  if (gx == nullptr || c_prev == nullptr || act == nullptr || c == nullptr || h == nullptr) return MPT_ERR_NULL;
  if (!dims_ok(B, H) || ldgx < 4 * H || (gr && ldgr < 4 * H) || ldcp < H || ldact < 4 * H || ldc < H || ldh < H) return MPT_ERR_SHAPE;
  if (!mpt_aligned(gx, 2) || !mpt_aligned(gr, 2) || !mpt_aligned(c_prev, 2) || !mpt_aligned(act, 2) || !mpt_aligned(c, 2) || !mpt_aligned(h, 2) ||
      !mpt_aligned(bias, 4))
    return MPT_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool vec = (H % 8) == 0 && vec_ok(gx, ldgx) && vec_ok(gr, ldgr) && vec_ok(c_prev, ldcp) && vec_ok(act, ldact) && vec_ok(c, ldc) && vec_ok(h, ldh);
  const int64_t units = vec ? B * (H / 4) : B * H;          // 4 cells (8 bytes) per lane: measured 5.5 vs 5.3 TB/s against 8 cells
  const unsigned grid = (unsigned)((units + kT - 1) / kT);
  const bool stream_it = vec && B * H * 30 > (192LL << 20);   // bytes moved beyond the memory-side cache
  if (stream_it) hipLaunchKernelGGL((k_lstm_cell_fwd<4, true>), dim3(grid), dim3(kT), 0, st, B, H, gx, ldgx, gr, ldgr, bias, c_prev, ldcp, act, ldact, c, ldc, h, ldh);
  else if (vec) hipLaunchKernelGGL((k_lstm_cell_fwd<4, false>), dim3(grid), dim3(kT), 0, st, B, H, gx, ldgx, gr, ldgr, bias, c_prev, ldcp, act, ldact, c, ldc, h, ldh);
  else hipLaunchKernelGGL((k_lstm_cell_fwd<1, false>), dim3(grid), dim3(kT), 0, st, B, H, gx, ldgx, gr, ldgr, bias, c_prev, ldcp, act, ldact, c, ldc, h, ldh);
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_lstm_cell_bwd(void* stream, int64_t B, int64_t H, const uint16_t* dh, int64_t lddh, const uint16_t* dc_next, int64_t lddcn,
                                 const uint16_t* act, int64_t ldact, const uint16_t* c, int64_t ldc, const uint16_t* c_prev, int64_t ldcp,
                                 uint16_t* da, int64_t ldda, uint16_t* dc_prev, int64_t lddcp) {
  if (dh == nullptr || act == nullptr || c == nullptr || c_prev == nullptr || da == nullptr || dc_prev == nullptr) return MPT_ERR_NULL;
  if (!dims_ok(B, H) || lddh < H || (dc_next && lddcn < H) || ldact < 4 * H || ldc < H || ldcp < H || ldda < 4 * H || lddcp < H) return MPT_ERR_SHAPE;
  if (!mpt_aligned(dh, 2) || !mpt_aligned(dc_next, 2) || !mpt_aligned(act, 2) || !mpt_aligned(c, 2) || !mpt_aligned(c_prev, 2) || !mpt_aligned(da, 2) ||
      !mpt_aligned(dc_prev, 2))
    return MPT_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool vec = (H % 8) == 0 && vec_ok(dh, lddh) && vec_ok(dc_next, lddcn) && vec_ok(act, ldact) && vec_ok(c, ldc) && vec_ok(c_prev, ldcp) &&
                   vec_ok(da, ldda) && vec_ok(dc_prev, lddcp);
  const int64_t units = vec ? B * (H / 4) : B * H;          // 4 cells (8 bytes) per lane: measured 5.5 vs 5.3 TB/s against 8 cells
  const unsigned grid = (unsigned)((units + kT - 1) / kT);
  const bool stream_it = vec && B * H * 22 > (192LL << 20);
  if (stream_it) hipLaunchKernelGGL((k_lstm_cell_bwd<4, true>), dim3(grid), dim3(kT), 0, st, B, H, dh, lddh, dc_next, lddcn, act, ldact, c, ldc, c_prev, ldcp, da, ldda, dc_prev, lddcp);
  else if (vec) hipLaunchKernelGGL((k_lstm_cell_bwd<4, false>), dim3(grid), dim3(kT), 0, st, B, H, dh, lddh, dc_next, lddcn, act, ldact, c, ldc, c_prev, ldcp, da, ldda, dc_prev, lddcp);
  else hipLaunchKernelGGL((k_lstm_cell_bwd<1, false>), dim3(grid), dim3(kT), 0, st, B, H, dh, lddh, dc_next, lddcn, act, ldact, c, ldc, c_prev, ldcp, da, ldda, dc_prev, lddcp);
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}
