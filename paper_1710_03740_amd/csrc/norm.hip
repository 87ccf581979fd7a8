// Batch normalisation over FP16 tensors x[P, C] (channels contiguous) for gfx950: reductions read FP16 and
// accumulate wide, pointwise parts compute in FP32 and store FP16 (paper Sec. 3.3, the "reductions" category).
// All four passes are HBM-bound and share one shape: a thread owns 4 consecutive channels (one 8-byte load per
// row; 8 channels where a row would not fit one workgroup) and walks rows; the threads of a workgroup that share a channel group sit on different rows, so a wavefront
// instruction covers whole contiguous rows.  Per-channel constants are formed once per thread, not per element.
//
// Reductions: FP32 chains of at most 16 rows, folded into FP64 per thread, across the workgroup through LDS and
// across workgroups through an FP64 partial buffer summed in a fixed order (run-to-run reproducible).  The
// statistics are accumulated about a per-channel pivot (the channel's first element), so that
// var = E[(x-k)^2] - E[x-k]^2 does not cancel when the mean is large against the spread.
#include "mpt_internal.h"

typedef _Float16 h8v __attribute__((ext_vector_type(8)));
typedef _Float16 h4v __attribute__((ext_vector_type(4)));

namespace {

constexpr int kBlock = 256;
constexpr int kChain = 16;        // rows summed in FP32 before folding into FP64
constexpr int kMaxBlocks = 1024;

struct BnShape {
  int64_t P;
  int C;
  int cg;          // channel groups: ceil(C / V)
  int tpr;         // threads of a workgroup along a row (each owns one channel group)
  int slots;       // rows a workgroup visits at once
  int cgy;         // workgroups along the channels (grid.y)
  int nblk;        // row blocks (grid.x)
  int64_t rows_per_block;
};

// A workgroup is tpr channel groups wide (at most a wavefront in the reductions, so that several rows are visited at
// once whatever C is; up to the whole workgroup in the pointwise passes, whose stores like whole rows) and `slots` rows tall; wider tensors take more workgroups along the channels.  The reductions keep the grid
// near 1024 workgroups so that the FP64 partial buffer stays a few percent of the tensor.
template <int V>
BnShape bn_shape(int64_t P, int64_t C, int rows_per_thread, int max_blocks, int max_tpr) {
  BnShape s;
  s.P = P; s.C = (int)C;
  s.cg = (int)((C + V - 1) / V);
  s.tpr = s.cg < max_tpr ? s.cg : max_tpr;
  s.slots = kBlock / s.tpr;
  s.cgy = (s.cg + s.tpr - 1) / s.tpr;
  int64_t nb = (P + (int64_t)s.slots * rows_per_thread - 1) / ((int64_t)s.slots * rows_per_thread);
  int64_t cap = max_blocks / s.cgy;
  if (cap < 1) cap = 1;
  if (nb > cap) nb = cap;
  if (nb < 1) nb = 1;
  s.rows_per_block = (P + nb - 1) / nb;
  s.nblk = (int)((P + s.rows_per_block - 1) / s.rows_per_block);
  return s;
}
template <int V> BnShape bn_shape(int64_t P, int64_t C) { return bn_shape<V>(P, C, kChain, kMaxBlocks, 64); }

// V channels of one row as floats; channels at or beyond C read as 0.
template <int V, bool NT>
__device__ __forceinline__ void load_row(const uint16_t* __restrict__ base, int64_t ld, int64_t p, int c0, int C, float (&v)[V]) {
  if constexpr (V == 8) {
    const h8v* q = reinterpret_cast<const h8v*>(base + p * ld + c0);
    const h8v h = NT ? __builtin_nontemporal_load(q) : *q;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)h[e];
  } else if constexpr (V == 4) {
    const h4v* q = reinterpret_cast<const h4v*>(base + p * ld + c0);
    const h4v h = NT ? __builtin_nontemporal_load(q) : *q;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = (float)h[e];
  } else {
    v[0] = c0 < C ? (float)reinterpret_cast<const _Float16*>(base)[p * ld + c0] : 0.f;
  }
}
template <int V, bool NT>
__device__ __forceinline__ void store_row(uint16_t* __restrict__ base, int64_t ld, int64_t p, int c0, int C, const float (&v)[V]) {
  if constexpr (V == 8) {
    h8v h;
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = (_Float16)mpt_rounded_f32(v[e]);
    h8v* q = reinterpret_cast<h8v*>(base + p * ld + c0);
    if (NT) __builtin_nontemporal_store(h, q);
    else *q = h;
  } else if constexpr (V == 4) {
    h4v h;
#pragma unroll
    for (int e = 0; e < 4; ++e) h[e] = (_Float16)mpt_rounded_f32(v[e]);
    h4v* q = reinterpret_cast<h4v*>(base + p * ld + c0);
    if (NT) __builtin_nontemporal_store(h, q);
    else *q = h;
  } else {
    if (c0 < C) reinterpret_cast<_Float16*>(base)[p * ld + c0] = (_Float16)mpt_rounded_f32(v[0]);
  }
}

// thread -> (row slot, channel group); returns false for idle threads
__device__ __forceinline__ bool bn_thread(const BnShape& s, int& slot, int& cgi) {
  slot = threadIdx.x / s.tpr;
  cgi = blockIdx.y * s.tpr + (threadIdx.x - slot * s.tpr);
  return slot < s.slots && cgi < s.cg;
}

// MODE 0: S1 = sum (x - k), S2 = sum (x - k)^2 with k = x[0, c].
// MODE 1: S1 = sum dy, S2 = sum dy * ((x - mean) * invstd), each factor rounded to FP32 on its own.
// part[blk][2][C] in FP64.
template <int V, int MODE, bool NT>
__global__ __launch_bounds__(kBlock) void k_bn_partial(BnShape s, const uint16_t* __restrict__ x, int64_t ldx,
                                                       const uint16_t* __restrict__ dy, int64_t lddy,
                                                       const float* __restrict__ mean, const float* __restrict__ var, float eps,
                                                       double* __restrict__ part) {
  __shared__ double red[2][kBlock * V];
  int slot, cgi;
  const bool active = bn_thread(s, slot, cgi);
  const int c0 = cgi * V;
  double a1[V], a2[V];
#pragma unroll
  for (int e = 0; e < V; ++e) a1[e] = a2[e] = 0.0;
  if (active) {
    float k[V], istd[V];
    if constexpr (MODE == 0) {
      load_row<V, false>(x, ldx, 0, c0, s.C, k);
    } else {
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const int c = c0 + e;
        k[e] = c < s.C ? mean[c] : 0.f;
        istd[e] = c < s.C ? div_rn(1.0f, sqrt_rn(__fadd_rn(var[c], eps))) : 0.f;
      }
    }
    const int64_t r0 = (int64_t)blockIdx.x * s.rows_per_block;
    const int64_t r1 = min(r0 + s.rows_per_block, s.P);
    auto add_row = [&](const float (&xv)[V], const float (&gv)[V], float (&c1)[V], float (&c2)[V]) {
      if constexpr (MODE == 0) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
          const float d = __fsub_rn(xv[e], k[e]);
          c1[e] = __fadd_rn(c1[e], d);
          c2[e] = __fadd_rn(c2[e], __fmul_rn(d, d));
        }
      } else {
#pragma unroll
        for (int e = 0; e < V; ++e) {
          const float xh = __fmul_rn(__fsub_rn(xv[e], k[e]), istd[e]);
          c1[e] = __fadd_rn(c1[e], gv[e]);
          c2[e] = __fadd_rn(c2[e], __fmul_rn(gv[e], xh));
        }
      }
    };
    for (int64_t pb = r0 + slot; pb < r1; pb += (int64_t)s.slots * kChain) {
      float c1[V], c2[V];
#pragma unroll
      for (int e = 0; e < V; ++e) c1[e] = c2[e] = 0.f;
      if (pb + (int64_t)(kChain - 1) * s.slots < r1) {
        // whole chain: rows are fetched four at a time ahead of the arithmetic, added in row order
#pragma unroll
        for (int i0 = 0; i0 < kChain; i0 += 4) {
          float xv[4][V], gv[4][V];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int64_t p = pb + (int64_t)(i0 + i) * s.slots;
            load_row<V, NT>(x, ldx, p, c0, s.C, xv[i]);
            if constexpr (MODE == 1) load_row<V, NT>(dy, lddy, p, c0, s.C, gv[i]);
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) add_row(xv[i], gv[i], c1, c2);
        }
      } else {
        for (int i = 0; i < kChain; ++i) {
          const int64_t p = pb + (int64_t)i * s.slots;
          if (p >= r1) break;
          float xv[V], gv[V];
          load_row<V, NT>(x, ldx, p, c0, s.C, xv);
          if constexpr (MODE == 1) load_row<V, NT>(dy, lddy, p, c0, s.C, gv);
          add_row(xv, gv, c1, c2);
        }
      }
#pragma unroll
      for (int e = 0; e < V; ++e) { a1[e] += (double)c1[e]; a2[e] += (double)c2[e]; }
    }
  }
  // across the workgroup's row slots, in slot order
#pragma unroll
  for (int e = 0; e < V; ++e) { red[0][threadIdx.x * V + e] = a1[e]; red[1][threadIdx.x * V + e] = a2[e]; }
  __syncthreads();
  if (active && slot == 0) {
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const int c = c0 + e;
      if (c >= s.C) continue;
      double t1 = 0.0, t2 = 0.0;
      for (int q = 0; q < s.slots; ++q) {
        const int th = q * s.tpr + (threadIdx.x % s.tpr);
        t1 += red[0][th * V + e];
        t2 += red[1][th * V + e];
      }
      part[((int64_t)blockIdx.x * 2 + 0) * s.C + c] = t1;
      part[((int64_t)blockIdx.x * 2 + 1) * s.C + c] = t2;
    }
  }
}

// 16 channels per workgroup; 16 thread groups each sum a contiguous range of row blocks in block order, the 16
// results are added in group order; then the closing arithmetic in FP64 and one rounding to FP32.
template <int MODE>
__global__ __launch_bounds__(256) void k_bn_finalize(BnShape s, const double* __restrict__ part, const uint16_t* __restrict__ x,
                                                     float* __restrict__ out1, float* __restrict__ out2) {
  __shared__ double red[2][16][16];
  const int cl = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cl;
  const int per = (s.nblk + 15) / 16;
  const int b0 = grp * per, b1 = min(b0 + per, s.nblk);
  double t1 = 0.0, t2 = 0.0;
  if (c < s.C) {
#pragma unroll 8
    for (int b = b0; b < b1; ++b) {
      t1 += part[((int64_t)b * 2 + 0) * s.C + c];
      t2 += part[((int64_t)b * 2 + 1) * s.C + c];
    }
  }
  red[0][grp][cl] = t1;
  red[1][grp][cl] = t2;
  __syncthreads();
  if (grp != 0 || c >= s.C) return;
  t1 = t2 = 0.0;
  for (int g = 0; g < 16; ++g) { t1 += red[0][g][cl]; t2 += red[1][g][cl]; }
  if constexpr (MODE == 0) {
    const double k = (double)(float)reinterpret_cast<const _Float16*>(x)[c];
    const double d1 = t1 / (double)s.P;
    double v = t2 / (double)s.P - d1 * d1;
    if (!(v > 0.0)) v = (v != v) ? v : 0.0;       // rounding can leave a tiny negative; NaN stays NaN
    out1[c] = (float)(k + d1);
    out2[c] = (float)v;
  } else {
    out1[c] = (float)t2;                          // dgamma
    out2[c] = (float)t1;                          // dbeta
  }
}

// Per-channel constants of a pointwise pass are formed once per workgroup (square root and divisions are tens of
// instructions each) and handed to the row walkers through LDS.  Returns the first channel the workgroup covers
// and how many it covers.
template <int V>
__device__ __forceinline__ int bn_covered(const BnShape& s, int& count) {
  const int cbase = blockIdx.y * s.tpr * V;
  count = min(s.C - cbase, s.tpr * V);
  return cbase;
}

// y = rne16(x * scale + shift), scale = gamma * (1 / sqrt(var + eps)), shift = beta - mean * scale; optional ReLU.
template <int V, bool NT>
__global__ __launch_bounds__(kBlock) void k_bn_apply(BnShape s, const uint16_t* __restrict__ x, int64_t ldx,
                                                     const float* __restrict__ mean, const float* __restrict__ var,
                                                     const float* __restrict__ gamma, const float* __restrict__ beta, float eps, int relu,
                                                     uint16_t* __restrict__ y, int64_t ldy) {
  __shared__ float cst[2][kBlock * V];
  int count;
  const int cbase = bn_covered<V>(s, count);
  for (int j = threadIdx.x; j < count; j += kBlock) {
    const int c = cbase + j;
    const float sc = __fmul_rn(gamma[c], div_rn(1.0f, sqrt_rn(__fadd_rn(var[c], eps))));
    cst[0][j] = sc;
    cst[1][j] = __fsub_rn(beta[c], __fmul_rn(mean[c], sc));
  }
  __syncthreads();
  int slot, cgi;
  if (!bn_thread(s, slot, cgi)) return;
  const int c0 = cgi * V;
  float scale[V], shift[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    const int j = c0 - cbase + e;
    scale[e] = j < count ? cst[0][j] : 0.f;
    shift[e] = j < count ? cst[1][j] : 0.f;
  }
  const int64_t r0 = (int64_t)blockIdx.x * s.rows_per_block;
  const int64_t r1 = min(r0 + s.rows_per_block, s.P);
  auto one = [&](float (&v)[V]) {
#pragma unroll
    for (int e = 0; e < V; ++e) {
      v[e] = __fadd_rn(__fmul_rn(v[e], scale[e]), shift[e]);
      if (relu) v[e] = v[e] > 0.f ? v[e] : 0.f;
    }
  };
  int64_t p = r0 + slot;
  for (; p + 3 * (int64_t)s.slots < r1; p += 4 * (int64_t)s.slots) {      // four rows in flight
    float v[4][V];
#pragma unroll
    for (int i = 0; i < 4; ++i) load_row<V, NT>(x, ldx, p + (int64_t)i * s.slots, c0, s.C, v[i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) { one(v[i]); store_row<V, NT>(y, ldy, p + (int64_t)i * s.slots, c0, s.C, v[i]); }
  }
  for (; p < r1; p += s.slots) {
    float v[V];
    load_row<V, NT>(x, ldx, p, c0, s.C, v);
    one(v);
    store_row<V, NT>(y, ldy, p, c0, s.C, v);
  }
}

// dx = rne16( a * ((dy - b) - xhat * g) ), a = gamma * invstd, b = dbeta / P, g = dgamma / P, xhat = (x - mean) * invstd.
template <int V, bool NT>
__global__ __launch_bounds__(kBlock) void k_bn_bwd_apply(BnShape s, const uint16_t* __restrict__ x, int64_t ldx,
                                                         const uint16_t* __restrict__ dy, int64_t lddy,
                                                         const float* __restrict__ mean, const float* __restrict__ var,
                                                         const float* __restrict__ gamma, float eps,
                                                         const float* __restrict__ dgamma, const float* __restrict__ dbeta,
                                                         uint16_t* __restrict__ dx, int64_t lddx) {
  __shared__ float cst[5][kBlock * V];
  int count;
  const int cbase = bn_covered<V>(s, count);
  const float Pf = (float)s.P;
  for (int j = threadIdx.x; j < count; j += kBlock) {
    const int c = cbase + j;
    const float is = div_rn(1.0f, sqrt_rn(__fadd_rn(var[c], eps)));
    cst[0][j] = mean[c];
    cst[1][j] = is;
    cst[2][j] = __fmul_rn(gamma[c], is);
    cst[3][j] = div_rn(dbeta[c], Pf);
    cst[4][j] = div_rn(dgamma[c], Pf);
  }
  __syncthreads();
  int slot, cgi;
  if (!bn_thread(s, slot, cgi)) return;
  const int c0 = cgi * V;
  float mu[V], istd[V], a[V], b[V], g[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    const int j = c0 - cbase + e;
    const bool in = j < count;
    mu[e] = in ? cst[0][j] : 0.f;
    istd[e] = in ? cst[1][j] : 0.f;
    a[e] = in ? cst[2][j] : 0.f;
    b[e] = in ? cst[3][j] : 0.f;
    g[e] = in ? cst[4][j] : 0.f;
  }
  const int64_t r0 = (int64_t)blockIdx.x * s.rows_per_block;
  const int64_t r1 = min(r0 + s.rows_per_block, s.P);
  auto one = [&](float (&xv)[V], const float (&gv)[V]) {
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const float xh = __fmul_rn(__fsub_rn(xv[e], mu[e]), istd[e]);
      const float t = __fsub_rn(__fsub_rn(gv[e], b[e]), __fmul_rn(xh, g[e]));
      xv[e] = __fmul_rn(a[e], t);
    }
  };
  int64_t p = r0 + slot;
  for (; p + (int64_t)s.slots < r1; p += 2 * (int64_t)s.slots) {          // two rows of both tensors in flight
    float xv[2][V], gv[2][V];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      load_row<V, NT>(x, ldx, p + (int64_t)i * s.slots, c0, s.C, xv[i]);
      load_row<V, NT>(dy, lddy, p + (int64_t)i * s.slots, c0, s.C, gv[i]);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) { one(xv[i], gv[i]); store_row<V, NT>(dx, lddx, p + (int64_t)i * s.slots, c0, s.C, xv[i]); }
  }
  for (; p < r1; p += s.slots) {
    float xv[V], gv[V];
    load_row<V, NT>(x, ldx, p, c0, s.C, xv);
    load_row<V, NT>(dy, lddy, p, c0, s.C, gv);
    one(xv, gv);
    store_row<V, NT>(dx, lddx, p, c0, s.C, xv);
  }
}

bool bn_dims_ok(int64_t P, int64_t C) { return P >= 1 && C >= 1 && P < (1LL << 40) && C <= (1 << 21); }
// Tensors beyond the memory-side cache are streamed with nontemporal accesses (about 8 % faster there); smaller ones
// are left cacheable, since their producer or consumer is likely to find them on chip (nontemporal costs 15 % there).
bool bn_stream(int64_t P, int64_t C) { return P * C * 2 > (192LL << 20); }
bool bn_vec(const void* p, int64_t ld, int64_t C) { return mpt_aligned(p, 16) && (ld % 8) == 0 && (C % 8) == 0; }
// the pointwise passes need no partial buffer and may use more, shorter row blocks (about 16 rows per thread)
template <int V> BnShape bn_shape_pointwise(int64_t P, int64_t C) { return bn_shape<V>(P, C, 16, 1 << 20, kBlock); }

}  // namespace

extern "C" size_t mpt_bn_workspace_bytes(int64_t P, int64_t C) {
  if (!bn_dims_ok(P, C)) return 0;
  // sized for the scalar layout, which never has fewer row blocks than the vector one
  const BnShape s1 = bn_shape<1>(P, C), s4 = bn_shape<4>(P, C);
  const int nb = s1.nblk > s4.nblk ? s1.nblk : s4.nblk;
  return (size_t)nb * 2 * (size_t)C * sizeof(double);
}

extern "C" int mpt_bn_stats(void* stream, int64_t P, int64_t C, const uint16_t* x, int64_t ldx, float* mean, float* var,
                            void* ws, size_t ws_bytes) {
  if (x == nullptr || mean == nullptr || var == nullptr || ws == nullptr) return MPT_ERR_NULL;
  if (!bn_dims_ok(P, C) || ldx < C) return MPT_ERR_SHAPE;
  if (!mpt_aligned(x, 2) || !mpt_aligned(mean, 4) || !mpt_aligned(var, 4) || !mpt_aligned(ws, 16)) return MPT_ERR_ALIGN;
  if (ws_bytes < mpt_bn_workspace_bytes(P, C)) return MPT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  double* part = reinterpret_cast<double*>(ws);
  // 8 bytes per lane sustain more of HBM than 16 (measured 5.7 vs 5.6 TB/s here, 4.0 vs 3.2 at 64 channels)
  if (bn_vec(x, ldx, C)) {
    const BnShape s = bn_shape<4>(P, C);
    if (bn_stream(P, C)) hipLaunchKernelGGL((k_bn_partial<4, 0, true>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, nullptr, 0, nullptr, nullptr, 0.f, part);
    else hipLaunchKernelGGL((k_bn_partial<4, 0, false>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, nullptr, 0, nullptr, nullptr, 0.f, part);
    MPT_LAUNCH_CHECK();
    hipLaunchKernelGGL((k_bn_finalize<0>), dim3((s.C + 15) / 16), dim3(256), 0, st, s, part, x, mean, var);
  } else {
    const BnShape s = bn_shape<1>(P, C);
    if (bn_stream(P, C)) hipLaunchKernelGGL((k_bn_partial<1, 0, true>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, nullptr, 0, nullptr, nullptr, 0.f, part);
    else hipLaunchKernelGGL((k_bn_partial<1, 0, false>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, nullptr, 0, nullptr, nullptr, 0.f, part);
    MPT_LAUNCH_CHECK();
    hipLaunchKernelGGL((k_bn_finalize<0>), dim3((s.C + 15) / 16), dim3(256), 0, st, s, part, x, mean, var);
  }
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_bn_apply(void* stream, int64_t P, int64_t C, const uint16_t* x, int64_t ldx, const float* mean, const float* var,
                            const float* gamma, const float* beta, float eps, int relu, uint16_t* y, int64_t ldy) {
  if (x == nullptr || mean == nullptr || var == nullptr || gamma == nullptr || beta == nullptr || y == nullptr) return MPT_ERR_NULL;
  if (!bn_dims_ok(P, C) || ldx < C || ldy < C) return MPT_ERR_SHAPE;
  if (!mpt_finite(eps) || eps < 0.f) return MPT_ERR_ARG;
  if (!mpt_aligned(x, 2) || !mpt_aligned(y, 2) || !mpt_aligned(mean, 4) || !mpt_aligned(var, 4) || !mpt_aligned(gamma, 4) || !mpt_aligned(beta, 4))
    return MPT_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // 8 bytes per lane while a row still fits one workgroup (C <= 1024), else 16 (measured 6.0 vs 5.6 TB/s at 256 channels)
  if (C <= 4 * kBlock && bn_vec(x, ldx, C) && bn_vec(y, ldy, C)) {
    const BnShape s = bn_shape_pointwise<4>(P, C);
    if (bn_stream(P, C)) hipLaunchKernelGGL((k_bn_apply<4, true>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, mean, var, gamma, beta, eps, relu, y, ldy);
    else hipLaunchKernelGGL((k_bn_apply<4, false>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, mean, var, gamma, beta, eps, relu, y, ldy);
  } else if (bn_vec(x, ldx, C) && bn_vec(y, ldy, C)) {
    const BnShape s = bn_shape_pointwise<8>(P, C);
    if (bn_stream(P, C)) hipLaunchKernelGGL((k_bn_apply<8, true>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, mean, var, gamma, beta, eps, relu, y, ldy);
    else hipLaunchKernelGGL((k_bn_apply<8, false>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, mean, var, gamma, beta, eps, relu, y, ldy);
  } else {
    const BnShape s = bn_shape_pointwise<1>(P, C);
    if (bn_stream(P, C)) hipLaunchKernelGGL((k_bn_apply<1, true>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, mean, var, gamma, beta, eps, relu, y, ldy);
    else hipLaunchKernelGGL((k_bn_apply<1, false>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, mean, var, gamma, beta, eps, relu, y, ldy);
  }
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_bn_bwd_reduce(void* stream, int64_t P, int64_t C, const uint16_t* x, int64_t ldx, const uint16_t* dy, int64_t lddy,
                                 const float* mean, const float* var, float eps, float* dgamma, float* dbeta, void* ws, size_t ws_bytes) {
  if (x == nullptr || dy == nullptr || mean == nullptr || var == nullptr || dgamma == nullptr || dbeta == nullptr || ws == nullptr)
    return MPT_ERR_NULL;
  if (!bn_dims_ok(P, C) || ldx < C || lddy < C) return MPT_ERR_SHAPE;
  if (!mpt_finite(eps) || eps < 0.f) return MPT_ERR_ARG;
  if (!mpt_aligned(x, 2) || !mpt_aligned(dy, 2) || !mpt_aligned(mean, 4) || !mpt_aligned(var, 4) || !mpt_aligned(dgamma, 4) ||
      !mpt_aligned(dbeta, 4) || !mpt_aligned(ws, 16))
    return MPT_ERR_ALIGN;
  if (ws_bytes < mpt_bn_workspace_bytes(P, C)) return MPT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  double* part = reinterpret_cast<double*>(ws);
  if (bn_vec(x, ldx, C) && bn_vec(dy, lddy, C)) {
    const BnShape s = bn_shape<4>(P, C);
    if (bn_stream(P, C)) hipLaunchKernelGGL((k_bn_partial<4, 1, true>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, dy, lddy, mean, var, eps, part);
    else hipLaunchKernelGGL((k_bn_partial<4, 1, false>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, dy, lddy, mean, var, eps, part);
    MPT_LAUNCH_CHECK();
    hipLaunchKernelGGL((k_bn_finalize<1>), dim3((s.C + 15) / 16), dim3(256), 0, st, s, part, x, dgamma, dbeta);
  } else {
    const BnShape s = bn_shape<1>(P, C);
    if (bn_stream(P, C)) hipLaunchKernelGGL((k_bn_partial<1, 1, true>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, dy, lddy, mean, var, eps, part);
    else hipLaunchKernelGGL((k_bn_partial<1, 1, false>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, dy, lddy, mean, var, eps, part);
    MPT_LAUNCH_CHECK();
    hipLaunchKernelGGL((k_bn_finalize<1>), dim3((s.C + 15) / 16), dim3(256), 0, st, s, part, x, dgamma, dbeta);
  }
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

extern "C" int mpt_bn_bwd_apply(void* stream, int64_t P, int64_t C, const uint16_t* x, int64_t ldx, const uint16_t* dy, int64_t lddy,
                                const float* mean, const float* var, const float* gamma, float eps, const float* dgamma,
                                const float* dbeta, uint16_t* dx, int64_t lddx) {
  if (x == nullptr || dy == nullptr || mean == nullptr || var == nullptr || gamma == nullptr || dgamma == nullptr || dbeta == nullptr ||
      dx == nullptr)
    return MPT_ERR_NULL;
  if (!bn_dims_ok(P, C) || ldx < C || lddy < C || lddx < C) return MPT_ERR_SHAPE;
  if (!mpt_finite(eps) || eps < 0.f) return MPT_ERR_ARG;
  if (!mpt_aligned(x, 2) || !mpt_aligned(dy, 2) || !mpt_aligned(dx, 2) || !mpt_aligned(mean, 4) || !mpt_aligned(var, 4) ||
      !mpt_aligned(gamma, 4) || !mpt_aligned(dgamma, 4) || !mpt_aligned(dbeta, 4))
    return MPT_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (C <= 4 * kBlock && bn_vec(x, ldx, C) && bn_vec(dy, lddy, C) && bn_vec(dx, lddx, C)) {
    const BnShape s = bn_shape_pointwise<4>(P, C);
    if (bn_stream(P, C)) hipLaunchKernelGGL((k_bn_bwd_apply<4, true>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, dy, lddy, mean, var, gamma, eps, dgamma, dbeta, dx, lddx);
    else hipLaunchKernelGGL((k_bn_bwd_apply<4, false>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, dy, lddy, mean, var, gamma, eps, dgamma, dbeta, dx, lddx);
  } else if (bn_vec(x, ldx, C) && bn_vec(dy, lddy, C) && bn_vec(dx, lddx, C)) {
    const BnShape s = bn_shape_pointwise<8>(P, C);
    if (bn_stream(P, C)) hipLaunchKernelGGL((k_bn_bwd_apply<8, true>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, dy, lddy, mean, var, gamma, eps, dgamma, dbeta, dx, lddx);
    else hipLaunchKernelGGL((k_bn_bwd_apply<8, false>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, dy, lddy, mean, var, gamma, eps, dgamma, dbeta, dx, lddx);
  } else {
    const BnShape s = bn_shape_pointwise<1>(P, C);
    if (bn_stream(P, C)) hipLaunchKernelGGL((k_bn_bwd_apply<1, true>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, dy, lddy, mean, var, gamma, eps, dgamma, dbeta, dx, lddx);
    else hipLaunchKernelGGL((k_bn_bwd_apply<1, false>), dim3(s.nblk, s.cgy), dim3(kBlock), 0, st, s, x, ldx, dy, lddy, mean, var, gamma, eps, dgamma, dbeta, dx, lddx);
  }
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}
