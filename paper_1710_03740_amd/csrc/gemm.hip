// FP16 contractions with FP32 accumulation and one RNE rounding to FP16 on store
// (paper Sec. 3.3), for the three passes of a layer (Sec. 3.1 / Fig. 1) and for
// the 3x3 convolution as an implicit GEMM.  gfx950 only.
//
// Four kernels compute C[i,j] = sum_r A(i,r) * B(r,j):
//   k_gemm        the general one: any shape, alignment and operand view (plain matrices, gathered image windows,
//                 filter slices), FP16 / FP32 / accumulating stores, split partials;
//   k_gemm_dma64  whole 256 x 256 tiles of aligned operands - plain matrices, or the convolution's gathered image and
//                 filter - streamed global -> LDS in stages of reduction depth 64, one wavefront per SIMD; FP16 store,
//                 or (second instance) FP32 store / accumulate / split partials.  The square 4096^3 workload runs here;
//   k_gemm_dma4   the same in stages of depth 32: 128 x 256 tiles (few-row outputs, split or not) and the convolution's
//                 weight gradient with its per-tap gathered operand;
//   k_gemm_dma    depth 32 with two wavefronts per SIMD: FP16 outputs with odd row strides, FP32 outputs over short
//                 reductions.
// k_split_reduce / k_split_reduce4 add split partials in split order.
//
// k_gemm works on a BM x BN tile per workgroup with v_mfma_f32_32x32x16_f16.  Operands differ only in how a
// tile is fetched:
//   * "RC" operands are contiguous along the reduction index r: a thread fetches
//     16-byte chunks of 8 r-values and stores them to LDS unchanged;
//   * "OC" operands are contiguous along the outer index (i or j): a thread
//     fetches a 4(r) x 8(outer) patch and transposes it in registers on the way
//     to LDS.
// Either way LDS holds [outer][64 r-values] rows of 128 bytes whose 16-byte
// chunks are XOR-swizzled, so MFMA fragments are single ds_read_b128's.
// LDS is double buffered: global loads for tile t+1 are issued before the MFMAs
// of tile t and written to the other buffer after them; one barrier per tile.
#include "mpt_internal.h"
#include <algorithm>
#include <mutex>
#include <type_traits>

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

#ifndef MPT_GEMM_DEPTH_DEFAULT
#define MPT_GEMM_DEPTH_DEFAULT 64  // reduction depth per stage of the streamed 256 x 256 kernel: 64 (k_gemm_dma64) or 32 (k_gemm_dma4)
#endif

namespace {

constexpr int BK = 64;            // reduction depth of one LDS tile
constexpr int ROWB = BK * 2;      // bytes per LDS row

// ---------------------------------------------------------------- exact 32-bit division by an invariant
struct FastDiv {
  uint32_t d, m, s;               // q = (umulhi(m, n) + n') >> s  (round-up method)
  __host__ __device__ FastDiv() : d(1), m(0), s(0) {}
  explicit FastDiv(uint32_t div) : d(div) {
    if (div <= 1) { m = 0; s = 0; d = 1; return; }
    uint32_t l = 0;
    while ((1ull << l) < div) ++l;                                 // l = ceil(log2 d), 1..32
    m = (uint32_t)(((1ull << 32) * ((1ull << l) - div)) / div + 1);
    s = l - 1;
  }
  __device__ __forceinline__ uint32_t div(uint32_t n) const {
    if (d == 1) return n;
    const uint32_t t = __umulhi(m, n);
    return (t + ((n - t) >> 1)) >> s;
  }
  __device__ __forceinline__ void divmod(uint32_t n, uint32_t& q, uint32_t& r) const {
    q = div(n);
    r = n - q * d;
  }
};

// ---------------------------------------------------------------- operand views
// chunk(o, r, nvalid): address of the chunk that starts at outer index o and
// reduction index r, and how many of its 8 elements exist (0 => do not touch).
// RC views: the chunk runs along r.  OC views: the chunk runs along o.

struct MatRC {                     // element (o, r) at base[o*ld + r]
  const uint16_t* base; int64_t ld; int O, R;
  static constexpr bool kRC = true;
  __device__ __forceinline__ const uint16_t* chunk(int o, int r, int& nv) const {
    nv = (o < O) ? min(max(R - r, 0), 8) : 0;
    return base + (int64_t)o * ld + r;
  }
};

struct MatOC {                     // element (o, r) at base[r*ld + o]
  const uint16_t* base; int64_t ld; int O, R;
  static constexpr bool kRC = false;
  __device__ __forceinline__ const uint16_t* chunk(int o, int r, int& nv) const {
    nv = (r < R) ? min(max(O - o, 0), 8) : 0;
    return base + (int64_t)r * ld + o;
  }
};

// Gathered image rows for the 3x3 convolution, stride 1, pad 1.
// Outer index o = flat pixel (n, y, x); reduction index r = tap * Cc + c with
// tap = 3*tr + ts.  Source pixel is (y + sgn*(tr-1), x + sgn*(ts-1)); sgn = +1
// fetches the forward window, sgn = -1 the mirrored window of the input gradient.
struct ImgRC {
  const uint16_t* base; int H, W, Cc, O, R, sgn;
  FastDiv dHW, dW, dC;
  static constexpr bool kRC = true;
  __device__ __forceinline__ const uint16_t* chunk(int o, int r, int& nv) const {
    nv = 0;
    if (o >= O || r >= R) return base;
    uint32_t n, rem, y, x, tap, c;
    dHW.divmod((uint32_t)o, n, rem);
    dW.divmod(rem, y, x);
    dC.divmod((uint32_t)r, tap, c);
    const int tr = (int)tap / 3, ts = (int)tap - 3 * tr;
    const int yy = (int)y + sgn * (tr - 1), xx = (int)x + sgn * (ts - 1);
    if (yy < 0 || yy >= H || xx < 0 || xx >= W) return base;
    nv = 8;
    return base + (((int64_t)n * H + yy) * W + xx) * Cc + c;
  }
};

// Same gather with the roles swapped: reduction index r = flat pixel (n, y, x),
// outer index o = tap * Cc + c (weight-gradient pass reads the forward window).
struct ImgOC {
  const uint16_t* base; int H, W, Cc, O, R;
  FastDiv dHW, dW, dC;
  static constexpr bool kRC = false;
  __device__ __forceinline__ const uint16_t* chunk(int o, int r, int& nv) const {
    nv = 0;
    if (o >= O || r >= R) return base;
    uint32_t n, rem, y, x, tap, c;
    dHW.divmod((uint32_t)r, n, rem);
    dW.divmod(rem, y, x);
    dC.divmod((uint32_t)o, tap, c);
    const int tr = (int)tap / 3, ts = (int)tap - 3 * tr;
    const int yy = (int)y + tr - 1, xx = (int)x + ts - 1;
    if (yy < 0 || yy >= H || xx < 0 || xx >= W) return base;
    nv = 8;
    return base + (((int64_t)n * H + yy) * W + xx) * Cc + c;
  }
};

// Filter w[k][tap][c] read as B(r = tap*Kf + k, o = c) for the input-gradient pass.
struct FilterOC {
  const uint16_t* base; int Cc, Kf, O, R;
  FastDiv dK;
  static constexpr bool kRC = false;
  __device__ __forceinline__ const uint16_t* chunk(int o, int r, int& nv) const {
    nv = 0;
    if (o >= O || r >= R) return base;
    uint32_t tap, k;
    dK.divmod((uint32_t)r, tap, k);
    nv = min(O - o, 8);
    return base + ((int64_t)k * 9 + tap) * Cc + o;
  }
};

// ---------------------------------------------------------------- chunk fetch
// `safe`: an address that can always be read (the view's first element).  The element-wise form has no branch around
// its loads: each reads an existing element (its own, the chunk's last, or `safe`) and the value is kept only if the
// element exists.  Behind branches the loads went out one at a time, each waited for: a 256 x 1024 output over a
// reduction of 10 took 20 us, all of it in two such chunks per operand.
template <bool ALIGNED>
__device__ __forceinline__ uint4v fetch(const uint16_t* p, int nv, const uint16_t* safe) {
  uint4v v = {0u, 0u, 0u, 0u};
  if constexpr (ALIGNED) {
    if (nv == 8) v = *reinterpret_cast<const uint4v*>(p);
  } else {
    const uint16_t* q = nv > 0 ? p : safe;
    const int last = max(nv, 1) - 1;
    uint16_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint16_t x = q[min(i, last)];
      e[i] = (i < nv) ? x : (uint16_t)0;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = (uint32_t)e[2 * i] | ((uint32_t)e[2 * i + 1] << 16);
  }
  return v;
}

// LDS byte offset of 16-byte chunk kc (0..7) of row `row`.
__device__ __forceinline__ int lds_off(int row, int kc) {
  return row * ROWB + (((kc ^ row ^ (row >> 3)) & 7) << 4);
}

// One operand tile in flight: 4 chunks per thread, whatever the flavour.
template <class View, bool ALIGNED, int BO, int NT>
struct TileLoader {
  static_assert(BO * 8 == NT * 4, "4 chunks per thread");
  uint4v reg[4];

  __device__ __forceinline__ void load(const View& v, int o_base, int r_base, int t) {
    if constexpr (View::kRC) {
      const int kc = t & 7, row0 = t >> 3;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = row0 + i * (NT / 8);
        int nv;
        const uint16_t* p = v.chunk(o_base + row, r_base + kc * 8, nv);
        reg[i] = fetch<ALIGNED>(p, nv, v.base);
      }
    } else {
      const int oc = t % (BO / 8), rg = t / (BO / 8);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int nv;
        const uint16_t* p = v.chunk(o_base + oc * 8, r_base + rg * 4 + i, nv);
        reg[i] = fetch<ALIGNED>(p, nv, v.base);
      }
    }
  }

  __device__ __forceinline__ void store(char* lds, int t) const {
    if constexpr (View::kRC) {
      const int kc = t & 7, row0 = t >> 3;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = row0 + i * (NT / 8);
        *reinterpret_cast<uint4v*>(lds + lds_off(row, kc)) = reg[i];
      }
    } else {
      // 4(r) x 8(o) patch -> eight rows of 4 r-values (8 bytes each)
      const int oc = t % (BO / 8), rg = t / (BO / 8);
      const int kc = rg >> 1, half = (rg & 1) << 3;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
        uint2v o2;
        o2[0] = __builtin_amdgcn_perm(reg[1][j >> 1], reg[0][j >> 1], sel);
        o2[1] = __builtin_amdgcn_perm(reg[3][j >> 1], reg[2][j >> 1], sel);
        const int row = oc * 8 + j;
        *reinterpret_cast<uint2v*>(lds + lds_off(row, kc) + half) = o2;
      }
    }
  }
};

// ---------------------------------------------------------------- epilogue description
struct Epilogue {
  void* out;            // uint16_t* (FP16) or float* (FP32 / split partials)
  int64_t ld;
  int mode;             // 0: FP16 store, 1: FP32 store, 2: FP32 accumulate, 3: FP32 partial [split][I][J]
  uint32_t* flag;       // nullable; OR 1 when an FP16/FP32 stored value is Inf/NaN (modes 0..2)
  int act;              // FP16 store only.  0: none; 1: ReLU, store 0 unless the value is > 0;
                        // 2: store 0 unless mask[i][j] > 0 (the ReLU of the layer below, backward)
  const uint16_t* mask; // act == 2: FP16 matrix of the output's shape
  int64_t ldmask;
};

// FP16 bit pattern of a value > 0 (Inf included, NaN not).
__device__ __forceinline__ bool half_bits_positive(uint32_t b) { return (uint16_t)((b & 0xFFFFu) - 1u) < 0x7C00u; }
// The mask values (act == 2) of 4 consecutive outputs of row i starting at column j, n of them inside the matrix
// (n = 0: none, the mask's first element is read instead), packed like the outputs.  No branch around the loads, so a
// caller can fetch the masks of a whole tile first and wait once: fetched one group at a time between the stores, each
// group cost a memory round trip (16 of them made a 256 x 1024 masked store take 17 us).
// `whole`: the caller has checked (uniformly) that every group is 4 wide or absent and 8-byte aligned, so one load
// fetches it; element by element each wavefront instruction touches 32 rows for 2 bytes apiece, and the 64 of them that
// a 128 x 128 tile needs took 8 us.
__device__ __forceinline__ uint2v load_mask4(const Epilogue& ep, int64_t i, int64_t j, int n, bool whole) {
  const uint16_t* m = n > 0 ? ep.mask + i * ep.ldmask + j : ep.mask;
  if (whole) return *reinterpret_cast<const uint2v*>(m);
  const int last = max(n, 1) - 1;
  const uint32_t e0 = m[0], e1 = m[min(1, last)], e2 = m[min(2, last)], e3 = m[min(3, last)];
  return uint2v{e0 | (e1 << 16), e2 | (e3 << 16)};
}
// Pointwise stage of an FP16 store: 4 consecutive outputs (packed in hb); mk = their mask values when act == 2.
__device__ __forceinline__ uint2v apply_act4(uint2v hb, const Epilogue& ep, uint2v mk) {
  if (ep.act == 0) return hb;
  uint32_t keep = 0;
  const uint2v src = ep.act == 1 ? hb : mk;
#pragma unroll
  for (int e = 0; e < 4; ++e) keep |= (uint32_t)half_bits_positive(src[e >> 1] >> ((e & 1) * 16)) << e;
  hb[0] &= ((keep & 1u) ? 0x0000FFFFu : 0u) | ((keep & 2u) ? 0xFFFF0000u : 0u);
  hb[1] &= ((keep & 4u) ? 0x0000FFFFu : 0u) | ((keep & 8u) ? 0xFFFF0000u : 0u);
  return hb;
}

struct Problem {
  int I, J, R;          // output rows, output cols, reduction length
  int tiles_i, tiles_j, splits, ktiles_per_split;
};

// Workgroup id -> (tile_i, tile_j, split).  Consecutive ids land on different XCDs
// (8 of them, round-robin), so ids are first regrouped per XCD and then walked in
// panels of 4 tile-rows so that one XCD's L2 sees a compact block of tiles.
__device__ __forceinline__ void tile_of(const Problem& pb, int wg, int& ti, int& tj, int& sp) {
  const int per_split = pb.tiles_i * pb.tiles_j;
  const int total = per_split * pb.splits;
  const int xcd = wg & 7, local = wg >> 3;
  const int n_per = total >> 3, rem = total & 7;
  int id = xcd * n_per + min(xcd, rem) + local;
  sp = id / per_split;
  id -= sp * per_split;
  constexpr int GM = 4;
  const int panel = id / (GM * pb.tiles_j);
  const int first_i = panel * GM;
  const int rows = min(GM, pb.tiles_i - first_i);
  const int in_panel = id - panel * GM * pb.tiles_j;
  ti = first_i + in_panel % rows;
  tj = in_panel / rows;
}

__device__ __forceinline__ bool half_bits_special(uint32_t b) { return (b & 0x7C00u) == 0x7C00u; }
// Inf/NaN vote over many packed FP16 pairs at two instructions per pair: keep the running maximum of the exponent fields
// of the low and of the high halves (v_pk_max_u16); a field of all ones anywhere shows in the maximum at the end.
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));
struct ExpMax {
  ushort2v m = {0, 0};
  __device__ __forceinline__ void add(uint32_t pair) { m = __builtin_elementwise_max(m, __builtin_bit_cast(ushort2v, pair & 0x7C007C00u)); }
  __device__ __forceinline__ bool special() const { return m[0] == 0x7C00 || m[1] == 0x7C00; }
};

// One output element from its split partials: summed in split order (fixed, so results are reproducible; eight partials
// in flight, since a dependent chain of single loads is bound by the memory latency: 28 splits took 17 us), then stored
// once in the final form.  Returns whether the stored value is Inf / NaN.
__device__ __forceinline__ bool reduce_one(const float* __restrict__ part, int splits, int64_t total, int64_t idx, int64_t i, int64_t j, const Epilogue& ep) {
  float s = part[idx];
  int k = 1;
  for (; k + 8 <= splits; k += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = part[(int64_t)(k + u) * total + idx];
#pragma unroll
    for (int u = 0; u < 8; ++u) s = __fadd_rn(s, v[u]);
  }
  for (; k < splits; ++k) s = __fadd_rn(s, part[(int64_t)k * total + idx]);
  if (ep.mode == 0) {
    const _Float16 h = (_Float16)s;
    uint16_t hb = __builtin_bit_cast(uint16_t, h);
    if (ep.act == 1 && !half_bits_positive(hb)) hb = 0;
    if (ep.act == 2 && !half_bits_positive(ep.mask[i * ep.ldmask + j])) hb = 0;
    reinterpret_cast<uint16_t*>(ep.out)[i * ep.ld + j] = hb;
    return half_bits_special(hb);
  }
  float* o = reinterpret_cast<float*>(ep.out) + i * ep.ld + j;
  if (ep.mode == 2) s = __fadd_rn(*o, s);
  *o = s;
  return (__float_as_uint(s) & 0x7F800000u) == 0x7F800000u;
}

template <class AView, class BView, bool A_ALIGNED, bool B_ALIGNED, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void k_gemm(AView A, BView B, Problem pb, Epilogue ep) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int FM = WM / 32, FN = WN / 32;
  constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB, STAGE = A_BYTES + B_BYTES;
  extern __shared__ __attribute__((aligned(16))) char lds[];

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm = wave / (BN / WN), wn = wave % (BN / WN);
  int ti, tj, sp;
  tile_of(pb, blockIdx.x, ti, tj, sp);
  const int i0 = ti * BM, j0 = tj * BN;
  const int kt_total = (pb.R + BK - 1) / BK;
  const int kt_begin = sp * pb.ktiles_per_split;
  const int kt_end = min(kt_begin + pb.ktiles_per_split, kt_total);

  float16v acc[FM][FN];
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  TileLoader<AView, A_ALIGNED, BM, NT> la;
  TileLoader<BView, B_ALIGNED, BN, NT> lb;

  // Mask values (act == 2) of the whole tile: fetched in one go - ahead of the first operand loads where the registers are there
  // for it (the 256-thread tile), so that both round trips pass together; else before the first store.
  constexpr bool kMasksEarly = NT == 256;
  uint2v mk[FM][FN][4];
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b)
#pragma unroll
      for (int g = 0; g < 4; ++g) mk[a][b][g] = uint2v{0u, 0u};
  auto fetch_masks = [&]() {
    if (!(ep.mode == 0 && ep.act == 2)) return;
    const bool whole = (pb.J % 4) == 0 && (ep.ldmask % 4) == 0 && (reinterpret_cast<uintptr_t>(ep.mask) & 7) == 0;
#pragma unroll
    for (int a = 0; a < FM; ++a) {
      const int i = i0 + wm * WM + a * 32 + (lane & 31);
#pragma unroll
      for (int b = 0; b < FN; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int j = j0 + wn * WN + b * 32 + g * 8 + ((lane >> 5) << 2);
          mk[a][b][g] = load_mask4(ep, i, j, (i < pb.I && j < pb.J) ? min(4, pb.J - j) : 0, whole);
        }
    }
  };
  if constexpr (kMasksEarly) fetch_masks();
  if (kt_begin < kt_end) {
    la.load(A, i0, kt_begin * BK, t);
    lb.load(B, j0, kt_begin * BK, t);
    la.store(lds, t);
    lb.store(lds + A_BYTES, t);
  }
  __syncthreads();

  const int frag_row = lane & 31, frag_kc = lane >> 5;
  int stage = 0;
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const bool more = kt + 1 < kt_end;
    if (more) {
      la.load(A, i0, (kt + 1) * BK, t);
      lb.load(B, j0, (kt + 1) * BK, t);
    }
    const char* sa = lds + stage * STAGE;
    const char* sb = sa + A_BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      half8 fa[FM], fb[FN];
#pragma unroll
      for (int a = 0; a < FM; ++a)
        fa[a] = *reinterpret_cast<const half8*>(sa + lds_off(wm * WM + a * 32 + frag_row, ks * 2 + frag_kc));
#pragma unroll
      for (int b = 0; b < FN; ++b)
        fb[b] = *reinterpret_cast<const half8*>(sb + lds_off(wn * WN + b * 32 + frag_row, ks * 2 + frag_kc));
      // operands swapped: the MFMA sees (B-fragment) x (A-fragment), so each lane ends
      // up owning 4 consecutive output columns j for one output row i.
#pragma unroll
      for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[b], fa[a], acc[a][b], 0, 0, 0);
    }
    if (more) {
      char* dst = lds + (stage ^ 1) * STAGE;
      la.store(dst, t);
      lb.store(dst + A_BYTES, t);
    }
    __syncthreads();
    stage ^= 1;
  }

  // ---- epilogue.  acc[a][b][v]: row i = lane%32, col j = 8*(v/4) + 4*(lane/32) + v%4 of the 32x32 block.
  bool bad = false;
  const int64_t split_off = (ep.mode == 3) ? (int64_t)sp * pb.I * pb.J : 0;
  if constexpr (!kMasksEarly) fetch_masks();
#pragma unroll
  for (int a = 0; a < FM; ++a) {
    const int i = i0 + wm * WM + a * 32 + (lane & 31);
#pragma unroll
    for (int b = 0; b < FN; ++b) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int j = j0 + wn * WN + b * 32 + g * 8 + ((lane >> 5) << 2);
        if (i >= pb.I || j >= pb.J) continue;
        const int nj = min(4, pb.J - j);
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = acc[a][b][g * 4 + e];
        if (ep.mode == 0) {
          uint16_t* o = reinterpret_cast<uint16_t*>(ep.out) + (int64_t)i * ep.ld + j;
          half4 h;
#pragma unroll
          for (int e = 0; e < 4; ++e) h[e] = (_Float16)x[e];
          const uint2v hb = apply_act4(__builtin_bit_cast(uint2v, h), ep, mk[a][b][g]);
          if (ep.flag) {
#pragma unroll
            for (int e = 0; e < 4; ++e) bad |= (e < nj) & half_bits_special(hb[e >> 1] >> ((e & 1) * 16));
          }
          if (nj == 4 && ((reinterpret_cast<uintptr_t>(o) & 7) == 0)) {
            *reinterpret_cast<uint2v*>(o) = hb;
          } else {
            for (int e = 0; e < nj; ++e) o[e] = (uint16_t)(hb[e >> 1] >> ((e & 1) * 16));
          }
        } else {
          float* o = reinterpret_cast<float*>(ep.out) + split_off + (int64_t)i * ep.ld + j;
          if (nj == 4 && (reinterpret_cast<uintptr_t>(o) & 15) == 0) {     // 16 bytes per lane
            float4v v = {x[0], x[1], x[2], x[3]};
            if (ep.mode == 2) {
              const float4v old = *reinterpret_cast<const float4v*>(o);
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] = __fadd_rn(old[e], v[e]);
            }
            if (ep.flag && ep.mode != 3) {
#pragma unroll
              for (int e = 0; e < 4; ++e) bad |= (__float_as_uint(v[e]) & 0x7F800000u) == 0x7F800000u;
            }
            *reinterpret_cast<float4v*>(o) = v;
          } else {
            for (int e = 0; e < nj; ++e) {
              float v = x[e];
              if (ep.mode == 2) v = __fadd_rn(o[e], v);
              if (ep.flag && ep.mode != 3) bad |= (__float_as_uint(v) & 0x7F800000u) == 0x7F800000u;
              o[e] = v;
            }
          }
        }
      }
    }
  }
  if (ep.flag != nullptr && ep.mode != 3) {
    const unsigned long long vote = __builtin_amdgcn_ballot_w64(bad);
    if (vote != 0ull && lane == 0) atomicOr(ep.flag, 1u);
  }
}

// ---------------------------------------------------------------- streamed variant for whole 256x256 tiles of plain matrices
// Same contraction and tile on v_mfma_f32_16x16x32_f16 blocks, but operand slices go global -> LDS with the LDS-direct load
// (global_load_lds_dwordx4: no staging registers), through a ring of four 32 KiB stages of reduction depth 32,
// three of them in flight.  The two wavefronts that share a SIMD run half a stage apart (wavefronts 4-7 take the
// per-stage barrier in the middle of their stage), so one of them always has MFMAs to issue while the other sits
// at the barrier or waits for LDS.  LDS layouts (64 banks of 4 bytes, 16 lanes served together):
//   RC operand: [256 outer][32 r] rows of 64 B; 16-byte chunk c of row o is stored at chunk c ^ ((o >> 1) & 3)
//               (found by measurement to be the conflict-free key when 16 lanes read 16 rows x the same chunk);
//               a fragment is one ds_read_b128 per lane.
//   OC operand: [32 r][256 outer] rows of 512 B; 32-byte unit u of row r is stored at unit u ^ ((r & 3) | ((r >> 1) & 4));
//               a fragment is two ds_read_b64_tr_b16 per lane (the transposing LDS read: within 16 lanes, lane i
//               receives element i of each of the four 32-byte rows that lanes 4j..4j+3 point at; lanes 0-31 and
//               32-63 are served in separate passes, and the key keeps the 8 rows of a pass on distinct banks).
// The swizzles are applied by choosing which global chunk each lane fetches, since an LDS-direct load writes lane l
// at base + 16*l.  Requirements (checked by the host): I, J multiples of 256, R a multiple of 64, 16-byte aligned
// operands, FP16 store or FP32 split partials.
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;
typedef __fp16 fp16x4_t __attribute__((ext_vector_type(4)));

struct DmaMat { const uint16_t* base; int64_t ld; };

// XOR key of reduction row r for the 32-byte units of an OC stage row (see the layout note above).
__device__ __forceinline__ int oc_key(int r) { return (r & 3) | ((r >> 1) & 4); }

template <bool RC>
struct DmaOperand {
  const uint16_t* p0;       // this lane's source for its first 1 KiB block of stage 0
  const uint16_t* p1;       // ... and for its second block
  int64_t step;             // elements to advance per stage
  // o0: first outer index of the workgroup tile; r0: first reduction index of this workgroup's range
  __device__ __forceinline__ void init(const DmaMat& m, int o0, int r0, int wave, int lane) {
    if constexpr (RC) {
      const int row = wave * 32 + (lane >> 2);                       // blocks 2w, 2w+1 hold 16 rows each
      const int chunk = (lane & 3) ^ ((row >> 1) & 3);               // same for row + 16
      p0 = m.base + (int64_t)(o0 + row) * m.ld + r0 + chunk * 8;
      p1 = p0 + 16 * m.ld;
      step = 32;
    } else {
      const int row = wave * 4 + (lane >> 5);                        // blocks 2w, 2w+1 hold 2 reduction rows each
      const int pc = lane & 31;
      const int c0 = 2 * ((pc >> 1) ^ oc_key(row)) + (pc & 1);
      const int c1 = 2 * ((pc >> 1) ^ oc_key(row + 2)) + (pc & 1);
      p0 = m.base + (int64_t)(r0 + row) * m.ld + o0 + c0 * 8;
      p1 = m.base + (int64_t)(r0 + row + 2) * m.ld + o0 + c1 * 8;
      step = 32 * m.ld;
    }
  }
  __device__ __forceinline__ void issue(int stage_rel, char* lds_block, int which) const {
    if (which == 0) __builtin_amdgcn_global_load_lds((global_void_ptr)(p0 + stage_rel * step), (lds_void_ptr)lds_block, 16, 0, 0);
    else __builtin_amdgcn_global_load_lds((global_void_ptr)(p1 + stage_rel * step), (lds_void_ptr)(lds_block + 1024), 16, 0, 0);
  }
};

// LDS reads are issued through inline assembly so that their completion is tracked here, by explicit
// s_waitcnt on the in-order LGKM counter, and not by the compiler, which would otherwise put a full vmcnt(0)
// wait in front of every read that follows an LDS-direct load.
__device__ __forceinline__ uint32_t lds_offset(const char* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}
__device__ __forceinline__ half8 lds_read_b128(uint32_t addr) {
  half8 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
__device__ __forceinline__ uint2v lds_read_tr_b64(uint32_t addr) {
  uint2v v;
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}

// Fragment of 16 outer indices x 32 reduction indices (a whole stage) for v_mfma_f32_16x16x32_f16: lane l holds outer
// index l%16 and reduction indices 8*(l/16) .. +7.  Per-lane byte offsets inside an operand's stage are fixed for the
// whole kernel: RC fragments need one (a 16-byte chunk), OC fragments two (reduction rows +0..3 and +4..7, one
// transposing read each).
template <bool RC, int BO = 256>
struct FragAddr {
  uint32_t off[RC ? 1 : 2];
  __device__ __forceinline__ void init(int outer0, int lane) {
    if constexpr (RC) {
      const int r = outer0 + (lane & 15);
      const int c = lane >> 4;
      off[0] = r * 64 + (((c ^ (r >> 1)) & 3) << 4);
    } else {
      const int unit = outer0 >> 4;
      const int sub = (lane & 3) << 3;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int r = ((lane >> 4) << 3) + 4 * h + ((lane & 15) >> 2);
        off[h] = r * (BO * 2) + ((unit ^ (oc_key(r) & (BO / 16 - 1))) << 5) + sub;
      }
    }
  }
  __device__ __forceinline__ half8 read(uint32_t stage_operand) const {
    if constexpr (RC) {
      return lds_read_b128(stage_operand + off[0]);
    } else {
      const uint2v lo = lds_read_tr_b64(stage_operand + off[0]);
      const uint2v hi = lds_read_tr_b64(stage_operand + off[1]);
      uint4v q = {lo[0], lo[1], hi[0], hi[1]};
      return __builtin_bit_cast(half8, q);
    }
  }
};

// The same fragment addressed without arithmetic in the loop: the lane's absolute LDS address inside the first slot of
// each pair of ring slots sits in a register, and the slot within the pair and the operand's offset inside a stage go
// into the read's immediate offset (16 bits: a pair of slots plus an operand offset stays below 64 KiB).
template <int IMM>
__device__ __forceinline__ half8 lds_read_b128_imm(uint32_t addr) {
  static_assert(IMM >= 0 && IMM < 65536, "LDS immediate offset");
  half8 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(IMM) : "memory");
  return v;
}
template <int IMM>
__device__ __forceinline__ uint2v lds_read_tr_b64_imm(uint32_t addr) {
  static_assert(IMM >= 0 && IMM < 65536, "LDS immediate offset");
  uint2v v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(IMM) : "memory");
  return v;
}
template <bool RC, int BO = 256>
struct FragAddr4 {
  uint32_t at[2][RC ? 1 : 2];
  __device__ __forceinline__ void init(int outer0, int lane, uint32_t lds0, uint32_t pair_bytes) {
    FragAddr<RC, BO> f;
    f.init(outer0, lane);
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int h = 0; h < (RC ? 1 : 2); ++h) at[p][h] = lds0 + p * pair_bytes + f.off[h];
  }
  template <int PAIR, int IMM>
  __device__ __forceinline__ half8 read() const {
    if constexpr (RC) {
      return lds_read_b128_imm<IMM>(at[PAIR][0]);
    } else {
      const uint2v lo = lds_read_tr_b64_imm<IMM>(at[PAIR][0]);
      const uint2v hi = lds_read_tr_b64_imm<IMM>(at[PAIR][1]);
      uint4v q = {lo[0], lo[1], hi[0], hi[1]};
      return __builtin_bit_cast(half8, q);
    }
  }
};

// The compiler takes an inline-assembly LDS read to be complete when the statement ends.  A fragment that nothing
// consumes afterwards (the prefetch past the last stage) would leave its registers free for reuse, for instance as the
// address of the next LDS-direct load, while the data is still on its way and lands on top of the new value.  Passing
// such fragments through this statement after the final wait keeps their registers reserved until then.
__device__ __forceinline__ void keep_until_here(const half8& f) { asm volatile("" ::"v"(f)); }

// Wait until at most NEWER LDS reads issued after these fragments are still outstanding (the LGKM counter is
// in order and 4 bits wide); the fragments pass through the statement so that their consumers stay below it.
template <int NEWER>
__device__ __forceinline__ void wait_frags8(half8 (&f)[4], half8 (&g)[4]) {
  asm volatile("s_waitcnt lgkmcnt(%8)"
               : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(g[0]), "+v"(g[1]), "+v"(g[2]), "+v"(g[3])
               : "n"(NEWER < 15 ? NEWER : 15)
               : "memory");
}
template <int NEWER>
__device__ __forceinline__ void wait_frags4(half8 (&f)[4]) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : "n"(NEWER < 15 ? NEWER : 15) : "memory");
}

// Workgroup tile 256 x 256, 8 wavefronts as 2 x 4, 128 x 64 each = 8 x 4 blocks of v_mfma_f32_16x16x32_f16 (this shape
// moves half the accumulator bytes per FLOP of the 32x32x16 shape, which matters on a power-limited clock).  A stage
// (reduction depth 32) is one MFMA k-step; it is issued as two halves of 16 MFMAs (A blocks 0-3, then 4-7) so that
// the fragments of the other half / the next stage are fetched underneath.
template <bool A_RC, bool B_RC, int NSTAGE>
__global__ __launch_bounds__(512) void k_gemm_dma(DmaMat A, DmaMat B, Problem pb, Epilogue ep) {
  constexpr int AHEAD = NSTAGE - 1, OPERAND = 256 * 64, STAGE = 2 * OPERAND;
  constexpr int RA = 4 * (A_RC ? 1 : 2), RB = 4 * (B_RC ? 1 : 2);      // LDS read instructions per 4 A / 4 B fragments
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  int ti, tj, sp;
  tile_of(pb, blockIdx.x, ti, tj, sp);
  const int i0 = ti * 256, j0 = tj * 256;
  const int st_total = pb.R / 32;
  const int st_begin = sp * pb.ktiles_per_split * 2;
  const int nst = min(pb.ktiles_per_split * 2, st_total - st_begin);   // stages this workgroup reduces over (>= 1)

  float4v acc[8][4];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.f;

  DmaOperand<A_RC> da;
  DmaOperand<B_RC> db;
  da.init(A, i0, st_begin * 32, wave, lane);
  db.init(B, j0, st_begin * 32, wave, lane);
  const int blk = wave * 2048;                                         // this wavefront's two 1 KiB blocks inside an operand stage
  auto issue1 = [&](int s, int q) {                                    // one of the 4 loads of stage s; past the end: refetch the last slice into a free slot
    const int sc = min(s, nst - 1);
    char* st = lds + (s % NSTAGE) * STAGE;
    if (q < 2) da.issue(sc, st + blk, q);
    else db.issue(sc, st + OPERAND + blk, q - 2);
  };
  auto issue = [&](int s) {
#pragma unroll
    for (int q = 0; q < 4; ++q) issue1(s, q);
  };
  FragAddr<A_RC> aa[8];
  FragAddr<B_RC> ab[4];
#pragma unroll
  for (int a = 0; a < 8; ++a) aa[a].init(wm * 128 + a * 16, lane);
#pragma unroll
  for (int b = 0; b < 4; ++b) ab[b].init(wn * 64 + b * 16, lane);
  const uint32_t lds0 = lds_offset(lds);
  half8 fal[4], fah[4], fb[2][4];                                      // A blocks 0-3, A blocks 4-7, B blocks (double buffered)
  auto stage_base = [&](int s) { return lds0 + (uint32_t)((s % NSTAGE) * STAGE); };
  auto read_lo = [&](int s) {                                          // B blocks and A blocks 0-3 of stage s
    const uint32_t st = stage_base(s);
#pragma unroll
    for (int b = 0; b < 4; ++b) fb[s & 1][b] = ab[b].read(st + OPERAND);
#pragma unroll
    for (int a = 0; a < 4; ++a) fal[a] = aa[a].read(st);
  };
  auto read_hi = [&](int s) {                                          // A blocks 4-7 of stage s
    const uint32_t st = stage_base(s);
#pragma unroll
    for (int a = 0; a < 4; ++a) fah[a] = aa[4 + a].read(st);
  };
  // 16 MFMAs; when `load_stage` >= 0, two of the four LDS-direct loads of that stage are issued, one after every
  // eighth MFMA (A's pair in the first half of a stage, B's pair in the second), so that the vector-memory unit
  // drains between them instead of blocking the wavefront on a burst.
  auto mfma_half = [&](half8 (&fa)[4], half8 (&fbv)[4], int abase, int load_stage) {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
#pragma unroll
      for (int b = 0; b < 4; ++b)   // operands swapped: each lane ends up with 4 consecutive output columns of one row
        acc[abase + a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fbv[b], fa[a], acc[abase + a][b], 0, 0, 0);
      if (load_stage >= 0 && (a & 1)) {
        __builtin_amdgcn_sched_barrier(0);
        issue1(load_stage, (abase >> 1) + (a >> 1));
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  // Before the barrier that publishes stage s+2: only loads of the newest stage (s+AHEAD) may still be in flight, and
  // every LDS read of this wavefront has returned.  Wavefronts 0-3 reach their barrier after both halves of the
  // stage (all 4 newest loads issued), wavefronts 4-7 after the first half (2 issued).
  auto publish_end = [&]() { asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(4 * (AHEAD - 2)) : "memory"); };
  auto publish_mid = [&]() { asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(4 * (AHEAD - 2) - 2) : "memory"); };

#pragma unroll
  for (int q = 0; q < AHEAD; ++q) issue(q);
  publish_end();                              // stages 0 and 1 have landed everywhere
  read_lo(0);
  // The loop body is written for an even and an odd stage so that the B double buffer is indexed statically.
  auto one_stage = [&](int s, half8 (&fb_cur)[4]) {
    read_hi(s);
    __builtin_amdgcn_sched_barrier(0);
    wait_frags8<RA>(fal, fb_cur);            // requested half a stage ago; only the A 4-7 reads may still be in flight
    // loads of stage s+AHEAD go into the slot of stage s-1: every wavefront finished reading it before the last barrier it passed
    mfma_half(fal, fb_cur, 0, s + AHEAD);
    __builtin_amdgcn_sched_barrier(0);
    if (wave >= 4) publish_mid();
    __builtin_amdgcn_sched_barrier(0);
    read_lo(s + 1);                          // stage s+1 was published by an earlier barrier; past the end the data is unused
    __builtin_amdgcn_sched_barrier(0);
    wait_frags4<RA + RB>(fah);
    mfma_half(fah, fb_cur, 4, s + AHEAD);
    __builtin_amdgcn_sched_barrier(0);
    if (wave < 4) publish_end();
    __builtin_amdgcn_sched_barrier(0);
  };
  // nst is even (the reduction length is a multiple of 64 and splits are cut at multiples of 64), so the loop is the
  // only copy of the stage code: every prefetched fragment is consumed by the next trip, and none has a dead
  // destination inside the loop (see keep_until_here).
  for (int s = 0; s < nst; s += 2) {
    one_stage(s, fb[0]);
    one_stage(s + 1, fb[1]);
  }
  // drain the tail prefetches before LDS is released
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");

  // ---- epilogue (whole tiles): FP16 store, FP32 store / accumulate (each with optional Inf/NaN vote), or FP32 split partial.
  // acc[a][b][e]: row i = 16a + lane%16, column j = 16b + 4*(lane/16) + e of the wavefront's 128 x 64 block.
  bool bad = false;
  const int64_t split_off = (ep.mode == 3) ? (int64_t)sp * pb.I * pb.J : 0;
#pragma unroll
  for (int a = 0; a < 8; ++a) {
    const int i = i0 + wm * 128 + a * 16 + (lane & 15);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int j = j0 + wn * 64 + b * 16 + ((lane >> 4) << 2);
      if (ep.mode == 0) {
        half4 h;
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = (_Float16)acc[a][b][e];
        const uint2v hb = apply_act4(__builtin_bit_cast(uint2v, h), ep, ep.act == 2 ? load_mask4(ep, i, j, 4, false) : uint2v{0u, 0u});
        if (ep.flag) bad |= half_bits_special(hb[0]) | half_bits_special(hb[0] >> 16) | half_bits_special(hb[1]) | half_bits_special(hb[1] >> 16);
        uint16_t* o = reinterpret_cast<uint16_t*>(ep.out) + (int64_t)i * ep.ld + j;
        if ((reinterpret_cast<uintptr_t>(o) & 7) == 0) {
          *reinterpret_cast<uint2v*>(o) = hb;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (uint16_t)(hb[e >> 1] >> ((e & 1) * 16));
        }
      } else {                                                           // FP32 store, accumulate, or split partial: 16 bytes per lane
        float* o = reinterpret_cast<float*>(ep.out) + split_off + (int64_t)i * ep.ld + j;
        float4v v = acc[a][b];
        if (ep.mode == 2) {
          const float4v old = *reinterpret_cast<const float4v*>(o);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = __fadd_rn(old[e], v[e]);
        }
        if (ep.flag && ep.mode != 3) {
#pragma unroll
          for (int e = 0; e < 4; ++e) bad |= (__float_as_uint(v[e]) & 0x7F800000u) == 0x7F800000u;
        }
        *reinterpret_cast<float4v*>(o) = v;
      }
    }
  }
  if (ep.flag != nullptr && ep.mode != 3) {
    const unsigned long long vote = __builtin_amdgcn_ballot_w64(bad);
    if (vote != 0ull && lane == 0) atomicOr(ep.flag, 1u);
  }
}

// ---------------------------------------------------------------- streamed variant with one wavefront per SIMD
// Same ring, layouts and fragments as k_gemm_dma, but 4 wavefronts as 2 x 2, each owning 128 x 128 of the tile
// (8 x 8 MFMA blocks, 256 accumulator registers): a stage costs 16 fragment reads per 64 MFMAs instead of 12 per 32,
// i.e. two thirds of the LDS read traffic, and only four wavefronts meet at the per-stage barrier.  With a single
// wavefront per SIMD nothing else covers a stall, so everything is software-pipelined inside the wavefront:
// a stage is 8 steps (one A block against the 8 B blocks); step a requests A block a+2 (wrapping into the next stage),
// the steps after the stage's barrier also request the next stage's B blocks, and every step issues one of the
// wavefront's 8 LDS-direct loads (FragSched below says where in a step each request sits, and why).
// The kernel is also instantiated for a 128-row tile (64 x 128 per wavefront, 4 steps per stage).
// An operand of the one-wavefront-per-SIMD kernel is a policy: Src (what the host passes), kRC (layout kind),
// init (per-lane constants for this workgroup's tile) and issue<K> (the K-th LDS-direct load of a stage).
template <bool RC, int BO = 256>
struct DmaOperand4 {
  typedef DmaMat Src;
  static constexpr bool kRC = RC;
  static constexpr int NB = BO / 64;   // 1 KiB blocks per wavefront per stage (the operand stage is BO x 32 halves)
  const uint16_t* p[NB];    // this lane's source for its blocks of stage 0
  int64_t step;             // elements to advance per stage
  __device__ __forceinline__ void init(const DmaMat& m, int o0, int r0, int wave, int lane) {
    if constexpr (RC) {
      const int row = wave * (BO / 4) + (lane >> 2);                 // blocks NB*w .. hold 16 rows each
      const int chunk = (lane & 3) ^ ((row >> 1) & 3);               // same for row + 16k
#pragma unroll
      for (int k = 0; k < NB; ++k) p[k] = m.base + (int64_t)(o0 + row + 16 * k) * m.ld + r0 + chunk * 8;
      step = 32;
    } else {
      constexpr int RPB = 512 / BO;                                  // reduction rows per 1 KiB block (rows of BO*2 bytes)
      constexpr int LPR = 64 / RPB;                                  // lanes per reduction row
      const int pc = lane % LPR;
#pragma unroll
      for (int k = 0; k < NB; ++k) {
        const int row = (wave * NB + k) * RPB + lane / LPR;
        const int c = 2 * ((pc >> 1) ^ (oc_key(row) & (BO / 16 - 1))) + (pc & 1);
        p[k] = m.base + (int64_t)(r0 + row) * m.ld + o0 + c * 8;
      }
      step = 32 * m.ld;
    }
  }
  template <int K>
  __device__ __forceinline__ void issue(int stage_rel, char* lds_blocks) const {
    __builtin_amdgcn_global_load_lds((global_void_ptr)(p[K] + stage_rel * step), (lds_void_ptr)(lds_blocks + K * 1024), 16, 0, 0);
  }
};

// Source of zeros for taps that fall outside the image (an LDS-direct load needs an address to read).
__device__ __attribute__((aligned(64))) const uint32_t k_zero_line[16] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};

// 3x3 convolution, stride 1, pad 1: rows of the implicit matrix are pixels (n, y, x), the reduction index is
// r = tap * Cc + c with tap = 3*tr + ts; the source pixel is (y + sgn*(tr-1), x + sgn*(ts-1)).  Cc is a multiple of
// 32, so a stage of 32 r-values is 32 consecutive channels of one tap: per load a lane needs one bounds test and one
// address.  Reduction-contiguous layout, same LDS image as a plain RC operand.
struct DmaImgSrc {
  const uint16_t* base;
  int H, W, Cc, sgn;
  FastDiv dHW, dW, dSpt;           // divisions by H*W, W and by the stages per tap (Cc / 32)
};
template <int BO>
struct DmaImgRC {
  typedef DmaImgSrc Src;
  static constexpr bool kRC = true;
  static constexpr int NB = BO / 64;
  const uint16_t* base;
  int32_t pix[NB];                 // element offset of the lane's pixel (centre tap) + its 16-byte chunk
  int32_t yx[NB];                  // y << 16 | x
  int H, W, Cc, sgn, stage0;
  FastDiv dSpt;
  int st_dy, st_dx, st_off;        // of the stage being fetched (wavefront-uniform), worked out by the stage's first load
  __device__ __forceinline__ void init(const Src& m, int o0, int r0, int wave, int lane) {
    base = m.base; H = m.H; W = m.W; Cc = m.Cc; sgn = m.sgn; dSpt = m.dSpt; stage0 = r0 >> 5;
    st_dy = st_dx = st_off = 0;
    const int row = wave * (BO / 4) + (lane >> 2);
    const int chunk = (lane & 3) ^ ((row >> 1) & 3);
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      uint32_t n, rem, y, x;
      m.dHW.divmod((uint32_t)(o0 + row + 16 * k), n, rem);
      m.dW.divmod(rem, y, x);
      pix[k] = (int32_t)(((n * (uint32_t)H + y) * (uint32_t)W + x) * (uint32_t)Cc) + chunk * 8;
      yx[k] = (int32_t)((y << 16) | x);
    }
  }
  // A stage's loads are issued in order K = 0, 1, ...: the first works out what the stage has in common, the others
  // reuse it; pixel or line of zeros is a select on the address, not a branch (see DmaImgRC64).
  template <int K>
  __device__ __forceinline__ void issue(int stage_rel, char* lds_blocks) {
    if constexpr (K == 0) {
      uint32_t tap, cs;
      dSpt.divmod((uint32_t)(stage0 + stage_rel), tap, cs);        // wavefront-uniform
      const int tr = (int)tap / 3, ts = (int)tap - 3 * tr;
      st_dy = sgn * (tr - 1); st_dx = sgn * (ts - 1);
      st_off = (st_dy * W + st_dx) * Cc + (int)cs * 32;
    }
    const int yy = (int)((uint32_t)yx[K] >> 16) + st_dy, xx = (yx[K] & 0xFFFF) + st_dx;   // y up to 65535: logical shift
    const bool inside = (unsigned)yy < (unsigned)H && (unsigned)xx < (unsigned)W;
    const uintptr_t there = reinterpret_cast<uintptr_t>(base + (pix[K] + st_off));
    const uintptr_t zeros = reinterpret_cast<uintptr_t>(k_zero_line);
    const uintptr_t mask = inside ? ~(uintptr_t)0 : (uintptr_t)0;
    const uint16_t* p = reinterpret_cast<const uint16_t*>((there & mask) | (zeros & ~mask));
    __builtin_amdgcn_global_load_lds((global_void_ptr)p, (lds_void_ptr)(lds_blocks + K * 1024), 16, 0, 0);
  }
};

// The filter w[k][tap][c] read as B(r = tap * Kf + k, o = c) for the input-gradient pass: outer-contiguous, one
// reduction row (k, tap) is Cc contiguous channels; Kf is a multiple of 32, so a stage stays inside one tap.
struct DmaFilterSrc {
  const uint16_t* base;
  int Cc, Kf;
  FastDiv dSpt;                    // stages per tap = Kf / 32
};
struct DmaFilterOC {
  typedef DmaFilterSrc Src;
  static constexpr bool kRC = false;
  static constexpr int NB = 4;
  const uint16_t* p[NB];           // lane's source for reduction row (k = row, tap = 0) of its blocks
  int Cc, stage0;
  FastDiv dSpt;
  int64_t st_off;                  // element offset of the stage being fetched (wavefront-uniform), set by its first load
  __device__ __forceinline__ void init(const Src& m, int o0, int r0, int wave, int lane) {
    Cc = m.Cc; dSpt = m.dSpt; stage0 = r0 >> 5; st_off = 0;
    const int pc = lane & 31;
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      const int row = (wave * NB + k) * 2 + (lane >> 5);
      const int c = 2 * ((pc >> 1) ^ oc_key(row)) + (pc & 1);
      p[k] = m.base + (int64_t)row * 9 * m.Cc + o0 + c * 8;
    }
  }
  template <int K>
  __device__ __forceinline__ void issue(int stage_rel, char* lds_blocks) {
    if constexpr (K == 0) {
      uint32_t tap, ks;
      dSpt.divmod((uint32_t)(stage0 + stage_rel), tap, ks);
      st_off = ((int64_t)ks * 32 * 9 + tap) * Cc;
    }
    const uint16_t* q = p[K] + st_off;
    __builtin_amdgcn_global_load_lds((global_void_ptr)q, (lds_void_ptr)(lds_blocks + K * 1024), 16, 0, 0);
  }
};

// The image read as B(r = flat pixel (n, y, x), o = tap * Cc + c) for the weight-gradient pass: outer-contiguous, one
// reduction row is the Cc channels of the pixel shifted by the tap.  Cc is a multiple of 256, so a tile column of 256
// outer indices lies inside one tap: the shift is the same for the whole workgroup, and a lane needs per load the
// (y, x) of its pixel for one bounds test (two exact divisions) and one address.
struct DmaImgOCSrc {
  const uint16_t* base;
  int H, W, Cc;
  FastDiv dW, dH;
};
struct DmaImgOC {
  typedef DmaImgOCSrc Src;
  static constexpr bool kRC = false;
  static constexpr int NB = 4;
  const uint16_t* base;
  int H, W, Cc, dy, dx, r0;
  int32_t row[NB];                 // reduction row inside a stage of this lane's piece of block k
  int32_t coff[NB];                // channel offset of its 16-byte chunk (the LDS swizzle depends on the row)
  // The image coordinates (y, x) of the lane's pixel decide only whether the shifted pixel is inside the image (the
  // address is linear in the pixel index).  They are divided out once, for the first stage, and then stepped along:
  // a block's loads are issued stage after stage (the stage index never jumps by more than one, and repeats past
  // the end), and a stage is 32 pixels further.
  int32_t py[NB], px[NB];          // of the stage issued last for block k
  int last[NB];                    // that stage (wavefront-uniform)
  int step_x, step_y;              // 32 % W and (32 / W) % H
  int bad_y, bad_x;                // the one row / column whose shifted pixel falls outside (-1: none), fixed per workgroup
  __device__ __forceinline__ void init(const Src& m, int o0, int r0_, int wave, int lane) {
    base = m.base; H = m.H; W = m.W; Cc = m.Cc; r0 = r0_;
    const int tap = o0 / m.Cc, c0 = o0 - tap * m.Cc;
    const int tr = tap / 3, ts = tap - 3 * tr;
    dy = tr - 1; dx = ts - 1;
    bad_y = dy < 0 ? 0 : (dy > 0 ? m.H - 1 : -1);
    bad_x = dx < 0 ? 0 : (dx > 0 ? m.W - 1 : -1);
    step_x = 32 % m.W;
    step_y = (32 / m.W) % m.H;
    const int pc = lane & 31;
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      row[k] = (wave * NB + k) * 2 + (lane >> 5);
      coff[k] = c0 + (2 * ((pc >> 1) ^ oc_key(row[k])) + (pc & 1)) * 8;
      uint32_t q, x, n, y;
      m.dW.divmod((uint32_t)(r0_ + row[k]), q, x);
      m.dH.divmod(q, n, y);
      py[k] = (int32_t)y; px[k] = (int32_t)x; last[k] = 0;
    }
  }
  template <int K>
  __device__ __forceinline__ void issue(int stage_rel, char* lds_blocks) {
    const int inc = stage_rel - last[K];                             // 0 or 1, wavefront-uniform
    last[K] = stage_rel;
    int x = px[K] + (inc ? step_x : 0);
    const int carry = x >= W ? 1 : 0;
    x -= carry ? W : 0;
    int y = py[K] + (inc ? step_y : 0) + carry;
    y -= y >= H ? H : 0;
    px[K] = x; py[K] = y;
    const bool inside = y != bad_y && x != bad_x;
    const int p = r0 + stage_rel * 32 + row[K];
    const uintptr_t there = reinterpret_cast<uintptr_t>(base + ((int64_t)(p + dy * W + dx) * Cc + coff[K]));
    const uintptr_t zeros = reinterpret_cast<uintptr_t>(k_zero_line);
    const uintptr_t mask = inside ? ~(uintptr_t)0 : (uintptr_t)0;
    const uint16_t* src = reinterpret_cast<const uint16_t*>((there & mask) | (zeros & ~mask));
    __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(lds_blocks + K * 1024), 16, 0, 0);
  }
};

// Fragment-request schedule of the one-wavefront-per-SIMD kernel.  A stage is NA steps of 8 MFMAs; step a requests the
// A block used two steps later and, in the late steps (a >= NA/2, after the stage's barrier), its share of the next
// stage's 8 B blocks.  With a single wavefront per SIMD every instruction that is not an MFMA delays the next MFMA
// unless it sits alone in the gap behind one (measured: 4 VALU operations bunched before a step cost 9 cycles, the
// same 4 placed one per gap cost none; a bunched pair of LDS reads 10 cycles, spread 2-6), so the kernel
// issues its requests one per gap: the A block behind MFMA 0, B blocks behind the odd MFMAs (3, 3, 2 of them in steps
// 4, 5, 6, so that the last one is a whole step old when step 0 needs it), the LDS-direct load behind MFMA 6.  The
// 128-row kernel has only two steps behind its barrier: 6 B blocks behind MFMAs 1-6 of step 2, 2 behind MFMAs 1-2 of
// step 3, the loads behind MFMA 7 (late steps) and MFMAs 2 and 6 (early steps).
template <int NA>
struct FragSched {
  static constexpr int kADist = 2;
  static constexpr bool kSpread = true;
  static constexpr int nb_at(int a) {               // B blocks requested in step a
    if (NA == 4) return a == 2 ? 6 : (a == 3 ? 2 : 0);
    return (a == 4 || a == 5) ? 3 : (a == 6 ? 2 : 0);
  }
  static constexpr int b_gap(int k) { return NA == 4 ? k + 1 : 2 * k + 1; }   // MFMA behind which the step's k-th B request sits
  static constexpr int kLateLoadGap = NA == 4 ? 7 : 6;                        // ... and the late steps' LDS-direct load
  static constexpr int nb_before(int a) { int n = 0; for (int j = 0; j < a; ++j) n += nb_at(j); return n; }
  static constexpr int last_b_step() { int l = 0; for (int j = 0; j < NA; ++j) if (nb_at(j) > 0) l = j; return l; }
  // LDS read instructions issued in step a (ra1 / rb1 instructions per A / B fragment)
  static constexpr int reads(int a, int ra1, int rb1) { return ra1 + nb_at(((a % NA) + NA) % NA) * rb1; }
  // Reads that may still be outstanding when step a's operands are needed (the LDS returns data in order): everything
  // issued after the request of A block a; step 0 also needs the whole B buffer.
  static constexpr int allowed(int a, int ra1, int rb1) {
    if (kSpread) {                                  // requests follow the MFMAs: step a's own come after its wait
      int w = nb_at((((a - kADist) % NA) + NA) % NA) * rb1;
      for (int j = a - kADist + 1; j <= a - 1; ++j) w += reads(j, ra1, rb1);
      if (a == 0) {
        int wb = 0;
        for (int j = last_b_step() + 1; j <= NA - 1; ++j) wb += reads(j, ra1, rb1);
        if (wb < w) w = wb;
      }
      return w;
    }
    int w = 0;                                      // requests precede the step's wait; the B requests precede the A request
    for (int j = a - kADist + 1; j <= a; ++j) w += reads(j, ra1, rb1);
    if (a == 0) {
      int wb = ra1;
      for (int j = last_b_step() + 1; j <= NA; ++j) wb += reads(j, ra1, rb1);
      if (wb < w) w = wb;
    }
    return w;
  }
};

// MFMA with the accumulator pinned, in place, to the accumulation half of the register file: the 256 accumulator
// registers of a 128 x 128 wavefront block fill that half exactly, and left to itself the register allocator shuffles
// them through the other half.  Issued as assembly, the instruction is opaque to the compiler's hazard handling; the
// kernel keeps every reuse of an accumulator at least 7 MFMAs apart and idles 32 cycles before the epilogue reads them.
__device__ __forceinline__ void mfma_acc(float4v& acc, const half8& x, const half8& y) {
  asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(x), "v"(y));
}
template <int NEWER>
__device__ __forceinline__ void wait_frag1(half8& f) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(f) : "n"(NEWER < 15 ? NEWER : 15) : "memory");
}
template <int NEWER>
__device__ __forceinline__ void wait_frags9(half8& f, half8 (&g)[8]) {
  asm volatile("s_waitcnt lgkmcnt(%9)"
               : "+v"(f), "+v"(g[0]), "+v"(g[1]), "+v"(g[2]), "+v"(g[3]), "+v"(g[4]), "+v"(g[5]), "+v"(g[6]), "+v"(g[7])
               : "n"(NEWER < 15 ? NEWER : 15)
               : "memory");
}

// F32OUT selects the epilogue at compile time (both in one kernel spill): false = FP16 store through LDS; true = FP32
// store, accumulate or split partial straight from the accumulators, 16 bytes per lane (used for the convolution's
// weight gradient and for split reductions over 128-row tiles).
template <class AOp, class BOp, int BM, bool F32OUT = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_gemm_dma4(typename AOp::Src A, typename BOp::Src B, Problem pb, Epilogue ep) {
  constexpr bool A_RC = AOp::kRC, B_RC = BOp::kRC;
  // BM = 256: tile 256 x 256, 128 x 128 per wavefront.  BM = 128: tile 128 x 256, 64 x 128 per wavefront, for problems
  // with too few 256-row tiles to occupy the chip (batch-256 recurrent and gate products).
  static_assert(BM == 256 || BM == 128, "tile rows");
  constexpr int NA = BM / 32;                      // A blocks per wavefront = steps per stage
  constexpr int HALF = NA / 2;                     // the barrier sits before step HALF
  constexpr int LA = BM / 64, LB = 4;              // LDS-direct loads per wavefront per stage: A blocks, B blocks
  constexpr int LBQ = LB / HALF;                   // B loads issued per early step
  typedef FragSched<NA> Sched;
  constexpr int AD = Sched::kADist;
  constexpr int NSTAGE = 4, AHEAD = 3, A_BYTES = BM * 64, B_BYTES = 256 * 64, STAGE = A_BYTES + B_BYTES;
  constexpr int RA1 = A_RC ? 1 : 2, RB1 = B_RC ? 1 : 2;               // LDS read instructions per fragment
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  int ti, tj, sp;
  tile_of(pb, blockIdx.x, ti, tj, sp);
  const int i0 = ti * BM, j0 = tj * 256;
  const int st_total = pb.R / 32;
  const int st_begin = sp * pb.ktiles_per_split * 2;
  const int nst = min(pb.ktiles_per_split * 2, st_total - st_begin);   // stages this workgroup reduces over (even, >= 2)

  float4v acc[NA][8];
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.f;

  AOp da;
  BOp db;
  da.init(A, i0, st_begin * 32, wave, lane);
  db.init(B, j0, st_begin * 32, wave, lane);
  // load q (0 .. LA-1: A blocks, then the B blocks) of stage s; past the end: refetch the last slice into a free slot
  auto issue1 = [&](int s, auto qc) {
    constexpr int q = decltype(qc)::value;
    const int sc = min(s, nst - 1);
    char* st = lds + (s % NSTAGE) * STAGE;
    if constexpr (q < LA) da.template issue<q>(sc, st + wave * (LA * 1024));
    else db.template issue<q - LA>(sc, st + A_BYTES + wave * (LB * 1024));
  };
  static_assert(STAGE + A_BYTES < 65536, "the second slot of a pair plus the B offset fits the LDS immediate");
  const uint32_t lds0 = lds_offset(lds);
  FragAddr4<A_RC, BM> aa[NA];
  FragAddr4<B_RC, 256> ab[8];
#pragma unroll
  for (int a = 0; a < NA; ++a) aa[a].init(wm * (BM / 2) + a * 16, lane, lds0, 2 * STAGE);
#pragma unroll
  for (int b = 0; b < 8; ++b) ab[b].init(wn * 128 + b * 16, lane, lds0, 2 * STAGE);
  half8 fa[NA], fb[2][8];                                              // A blocks of the running stage(s); B blocks, double buffered
  auto issue_all = [&](int s, auto lo, auto hi) {                      // loads lo .. hi-1 of stage s
    constexpr int L = decltype(lo)::value, Hh = decltype(hi)::value;
    if constexpr (L + 0 < Hh) issue1(s, std::integral_constant<int, L + 0>{});
    if constexpr (L + 1 < Hh) issue1(s, std::integral_constant<int, L + 1>{});
    if constexpr (L + 2 < Hh) issue1(s, std::integral_constant<int, L + 2>{});
    if constexpr (L + 3 < Hh) issue1(s, std::integral_constant<int, L + 3>{});
    if constexpr (L + 4 < Hh) issue1(s, std::integral_constant<int, L + 4>{});
    if constexpr (L + 5 < Hh) issue1(s, std::integral_constant<int, L + 5>{});
    if constexpr (L + 6 < Hh) issue1(s, std::integral_constant<int, L + 6>{});
    if constexpr (L + 7 < Hh) issue1(s, std::integral_constant<int, L + 7>{});
  };

  // prologue: stages 0 and 1 whole, and the A part of stage 2 (the early steps of stage 0 add its B part)
  issue_all(0, std::integral_constant<int, 0>{}, std::integral_constant<int, LA + LB>{});
  issue_all(1, std::integral_constant<int, 0>{}, std::integral_constant<int, LA + LB>{});
  issue_all(2, std::integral_constant<int, 0>{}, std::integral_constant<int, LA>{});
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(LA) : "memory");     // stages 0 and 1 have landed everywhere
#pragma unroll
  for (int b = 0; b < 8; ++b) fb[0][b] = ab[b].template read<0, A_BYTES>();
#pragma unroll
  for (int a = 0; a < AD; ++a) fa[a] = aa[a].template read<0, 0>();

  // One step: requests, wait for this step's operands, 8 MFMAs with the step's LDS-direct loads among them.
  // LDS reads complete in order, so "A block a has arrived" is "at most W reads issued after it are outstanding"
  // (FragSched::allowed).
  // The ring slot of stage s (s % 4) is a compile-time constant SLOT: the loop below is unrolled over the four slots.
  auto step = [&](int s, auto slotc, auto ac, half8 (&fb_cur)[8], half8 (&fb_nxt)[8]) {
    constexpr int a = decltype(ac)::value, SLOT = decltype(slotc)::value;
    constexpr int SLOT_A = (SLOT + (a + Sched::kADist) / NA) % NSTAGE;  // slot of the A block requested in this step
    constexpr int SLOT_B = (SLOT + 1) % NSTAGE;                         // slot of the next stage's B blocks
    constexpr int PAIR_A = SLOT_A >> 1, IMM_A = (SLOT_A & 1) * STAGE;
    constexpr int PAIR_B = SLOT_B >> 1, IMM_B = (SLOT_B & 1) * STAGE + A_BYTES;
    if constexpr (a == HALF) {
      // Stage s+1 is about to be read and the slot of stage s-1 about to be refilled: every wavefront's loads of
      // stage s+1 must have landed (only the loads of stage s+2 may be in flight) and every wavefront must be
      // past stage s-1, all of whose reads were consumed by MFMAs already issued.
      asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(LA + LB) : "memory");
    }
    constexpr int B0 = Sched::nb_before(a);
    constexpr int na = (a + AD) % NA;
    static_assert(Sched::nb_at(a) == 0 || a >= HALF, "the next stage is published by the barrier before step HALF");
    constexpr bool SPREAD = Sched::kSpread;
    if constexpr (!SPREAD) {
#pragma unroll
      for (int k = 0; k < Sched::nb_at(a); ++k) fb_nxt[B0 + k] = ab[B0 + k].template read<PAIR_B, IMM_B>();
      fa[na] = aa[na].template read<PAIR_A, IMM_A>();                  // the last AD steps read the next stage (published at step HALF)
    }
    __builtin_amdgcn_sched_barrier(0);
    constexpr int W = Sched::allowed(a, RA1, RB1);
    if constexpr (a == 0) wait_frags9<W>(fa[0], fb_cur);
    else wait_frag1<W>(fa[a]);
#pragma unroll
    for (int b = 0; b < 8; ++b) {   // operands swapped: each lane ends up with 4 consecutive output columns of one row
      mfma_acc(acc[a][b], fb_cur[b], fa[a]);
      if constexpr (SPREAD) {       // one request per gap between MFMAs: the A block after MFMA 0, B blocks after the odd ones
        if (b == 0) {
          __builtin_amdgcn_sched_barrier(0);
          fa[na] = aa[na].template read<PAIR_A, IMM_A>();
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int k = 0; k < Sched::nb_at(a); ++k)
          if (b == Sched::b_gap(k)) {
            __builtin_amdgcn_sched_barrier(0);
            fb_nxt[B0 + k] = ab[B0 + k].template read<PAIR_B, IMM_B>();
            __builtin_amdgcn_sched_barrier(0);
          }
      }
      // late steps start stage s+3 (one A block each) into the slot just vacated; early steps finish stage s+2 (B blocks)
      constexpr int L1 = SPREAD ? 6 : 3, L2A = SPREAD ? 2 : 1, L2B = SPREAD ? 6 : 5;   // MFMAs followed by an LDS-direct load
      if constexpr (a >= HALF) {
        if (b == (SPREAD ? Sched::kLateLoadGap : 3)) {
          __builtin_amdgcn_sched_barrier(0);
          issue1(s + AHEAD, std::integral_constant<int, a - HALF>{});
          __builtin_amdgcn_sched_barrier(0);
        }
      } else if constexpr (LBQ == 1) {
        if (b == L1) {
          __builtin_amdgcn_sched_barrier(0);
          issue1(s + AHEAD - 1, std::integral_constant<int, LA + a>{});
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
        if (b == L2A) {
          __builtin_amdgcn_sched_barrier(0);
          issue1(s + AHEAD - 1, std::integral_constant<int, LA + 2 * a>{});
          __builtin_amdgcn_sched_barrier(0);
        }
        if (b == L2B) {
          __builtin_amdgcn_sched_barrier(0);
          issue1(s + AHEAD - 1, std::integral_constant<int, LA + 2 * a + 1>{});
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto one_stage = [&](int s, auto slotc, half8 (&fb_cur)[8], half8 (&fb_nxt)[8]) {
    step(s, slotc, std::integral_constant<int, 0>{}, fb_cur, fb_nxt);
    step(s, slotc, std::integral_constant<int, 1>{}, fb_cur, fb_nxt);
    step(s, slotc, std::integral_constant<int, 2>{}, fb_cur, fb_nxt);
    step(s, slotc, std::integral_constant<int, 3>{}, fb_cur, fb_nxt);
    if constexpr (NA == 8) {
      step(s, slotc, std::integral_constant<int, 4 % NA>{}, fb_cur, fb_nxt);
      step(s, slotc, std::integral_constant<int, 5 % NA>{}, fb_cur, fb_nxt);
      step(s, slotc, std::integral_constant<int, 6 % NA>{}, fb_cur, fb_nxt);
      step(s, slotc, std::integral_constant<int, 7 % NA>{}, fb_cur, fb_nxt);
    }
  };
  // nst is even: the reduction length is a multiple of 64 and splits are cut at multiples of 64
  typedef std::integral_constant<int, 0> S0;
  typedef std::integral_constant<int, 1> S1;
  typedef std::integral_constant<int, 2> S2;
  typedef std::integral_constant<int, 3> S3;
  // Where two paths that end in MFMAs meet (the loop's exit and the two-stage tail), the register allocator may place
  // accumulator copies on the edges; it knows nothing of the latency of an MFMA issued from assembly, so each path
  // first lets its last MFMAs retire (32 idle cycles, only in the loop's last trip).
  int s = 0;
  for (; s + 4 <= nst; s += 4) {
    one_stage(s, S0{}, fb[0], fb[1]);
    one_stage(s + 1, S1{}, fb[1], fb[0]);
    one_stage(s + 2, S2{}, fb[0], fb[1]);
    one_stage(s + 3, S3{}, fb[1], fb[0]);
    if (s + 8 > nst) asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  }
  if (s < nst) {                                                       // two stages left, in slots 0 and 1
    one_stage(s, S0{}, fb[0], fb[1]);
    one_stage(s + 1, S1{}, fb[1], fb[0]);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  }
  // drain the tail prefetches before LDS is released, and let the last MFMAs retire before their results are read
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int a = 0; a < NA; ++a) keep_until_here(fa[a]);
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    keep_until_here(fb[0][b]); keep_until_here(fb[1][b]);
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- epilogue (whole tiles; the host sends only 16-byte aligned outputs with whole 16-byte rows here, and FP16
  // stores only of unsplit problems).
  // acc[a][b][e]: row i = 16a + lane%16, column j = 16b + 4*(lane/16) + e of the wavefront's (BM/2) x 128 block.
  bool bad = false;
  if constexpr (F32OUT) {
    const int64_t split_off = (ep.mode == 3) ? (int64_t)sp * pb.I * pb.J : 0;
    float* out = reinterpret_cast<float*>(ep.out) + split_off + (int64_t)(i0 + wm * (BM / 2) + (lane & 15)) * ep.ld + j0 + wn * 128 + ((lane >> 4) << 2);
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int b = 0; b < 8; ++b) {
        asm volatile("" : "+a"(acc[a][b]) : : "memory");              // one block at a time out of the accumulation registers
        float* o = out + (int64_t)(a * 16) * ep.ld + b * 16;
        float4v v = acc[a][b];
        if (ep.mode == 2) {
          const float4v old = *reinterpret_cast<const float4v*>(o);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = __fadd_rn(old[e], v[e]);
        }
        if (ep.flag && ep.mode != 3) {
#pragma unroll
          for (int e = 0; e < 4; ++e) bad |= (__float_as_uint(v[e]) & 0x7F800000u) == 0x7F800000u;
        }
        *reinterpret_cast<float4v*>(o) = v;
      }
  } else {
    // FP16 store through LDS, so that global stores are whole 256-byte row segments instead of 32-byte pieces:
    // each wavefront rounds its block to FP16 into its own part of the (now idle) ring as [BM/2 rows][256 B],
    // 16-byte unit u of row r kept at unit u ^ (r & 15), then streams it out 16 bytes per lane, 16 lanes per row.
    __syncthreads();                                                   // every wavefront is done reading the ring
    char* mine = lds + wave * (BM / 2 * 256);
    const int li = lane & 15, lg = lane >> 4;
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int b = 0; b < 8; ++b) {
        asm volatile("" : "+a"(acc[a][b]) : : "memory");              // keeps the copy out of the accumulation registers here, one block at a time
        half4 h;
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = (_Float16)acc[a][b][e];
        *reinterpret_cast<half4*>(mine + (a * 16 + li) * 256 + (((2 * b + (lg >> 1)) ^ li) << 4) + (lg & 1) * 8) = h;
      }
    uint16_t* out = reinterpret_cast<uint16_t*>(ep.out) + (int64_t)(i0 + wm * (BM / 2)) * ep.ld + j0 + wn * 128 + li * 8;
    ExpMax emax;
#pragma unroll 8
    for (int it = 0; it < BM / 8; ++it) {
      const int r = it * 4 + lg;
      uint4v q = *reinterpret_cast<const uint4v*>(mine + r * 256 + ((li ^ (r & 15)) << 4));
      if (ep.act == 1) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          q[e] &= (half_bits_positive(q[e]) ? 0x0000FFFFu : 0u) | (half_bits_positive(q[e] >> 16) ? 0xFFFF0000u : 0u);
      } else if (ep.act == 2) {                                        // the host sends only 16-byte aligned masks with ldmask % 8 == 0 here
        const uint4v m = *reinterpret_cast<const uint4v*>(ep.mask + (int64_t)(i0 + wm * (BM / 2) + r) * ep.ldmask + j0 + wn * 128 + li * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          q[e] &= (half_bits_positive(m[e]) ? 0x0000FFFFu : 0u) | (half_bits_positive(m[e] >> 16) ? 0xFFFF0000u : 0u);
      }
      if (ep.flag) {
#pragma unroll
        for (int e = 0; e < 4; ++e) emax.add(q[e]);
      }
      *reinterpret_cast<uint4v*>(out + (int64_t)r * ep.ld) = q;
    }
    bad = emax.special();
  }
  if (ep.flag != nullptr && !(F32OUT && ep.mode == 3)) {
    const unsigned long long vote = __builtin_amdgcn_ballot_w64(bad);
    if (vote != 0ull && lane == 0) atomicOr(ep.flag, 1u);
  }
}

// ---------------------------------------------------------------- one wavefront per SIMD, reduction depth 64 per stage
// The same tile, wavefront blocks, fragment schedule and epilogue as k_gemm_dma4 (BM = 256), with the operand slices
// moved in stages of reduction depth 64: a reduction-contiguous operand is then fetched as whole 128-byte row
// slices, one cache line per 8 lanes, where a depth-32 stage asks the L2 for half lines (twice the requests).
// LDS holds two slots of 32 KiB per operand (A at 0 and 32 KiB, B at 64 and 96 KiB); a slot is one stage:
//   RC operand: [256 outer][128 B]; 16-byte chunk c (0..7, reduction indices 8c..8c+7) of row o at chunk c ^ ((o >> 1) & 7)
//               (16 lanes reading the same chunk of 16 consecutive rows then cover all 64 banks once);
//   OC operand: two depth-32 images of k_gemm_dma4's layout, 16 KiB each.
// A stage is consumed as two half stages of depth 32 (8 steps of 8 MFMAs each, exactly k_gemm_dma4's stage), so the
// fragment requests, waits and their immediates are the same; only the movement differs.  Per stage D (16 steps):
//   step 0   barrier F: every wavefront has finished reading A(D-1); steps 0-3 then fetch A(D+1) into its slot;
//   step 12  wait for all own loads, barrier P: A(D+1) and B(D+1) have landed everywhere, and every wavefront holds
//            the last B fragments of stage D in registers; steps 12-15 then fetch B(D+2) into B(D)'s slot.
// Loads are issued two per step, each alone in a gap between MFMAs; the youngest is 9 steps old when it must have
// landed, as in k_gemm_dma4.  Requirements (host): I, J multiples of 256, R of 64, unsplit FP16 store.
template <bool RC>
struct DmaOperand64 {
  typedef DmaMat Src;
  static constexpr bool kRC = RC;
  static constexpr int NB = 8;       // 1 KiB blocks per wavefront per stage (256 outer x 64 r halves = 32 KiB / 4 wavefronts)
  const uint16_t* p[RC ? 2 : 4];     // RC: lane's source in blocks 0 and 1 (blocks 2j, 2j+1 lie 16j rows further); OC: blocks 0-3 (4-7: 32 r further)
  int64_t ld;
  __device__ __forceinline__ void init(const DmaMat& m, int o0, int wave, int lane) {
    ld = m.ld;
    if constexpr (RC) {
#pragma unroll
      for (int k = 0; k < 2; ++k) {                                  // block k of the wavefront: rows 64w + 8k .. +7, lane -> (row, position)
        const int row = wave * 64 + k * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);             // rows 16 further have the same key
        p[k] = m.base + (int64_t)(o0 + row) * m.ld + chunk * 8;
      }
    } else {
      const int pc = lane & 31;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int row = (wave * 4 + k) * 2 + (lane >> 5);
        const int c = 2 * ((pc >> 1) ^ oc_key(row)) + (pc & 1);
        p[k] = m.base + (int64_t)row * m.ld + o0 + c * 8;
      }
    }
  }
  // K-th load of stage d (reduction indices 64d .. 64d+63) into the operand slot at `slot`
  template <int K>
  __device__ __forceinline__ void issue(int d, char* slot, int wave) const {
    if constexpr (RC) {
      const uint16_t* src = p[K & 1] + ((int64_t)d * 64 + (int64_t)(K >> 1) * 16 * ld);
      __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(slot + (wave * 8 + K) * 1024), 16, 0, 0);
    } else {
      const uint16_t* src = p[K & 3] + (int64_t)(2 * d + (K >> 2)) * 32 * ld;
      __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(slot + (K >> 2) * 16384 + (wave * 4 + (K & 3)) * 1024), 16, 0, 0);
    }
  }
};

// The convolution's gathered image rows (see DmaImgRC) for stages of depth 64: Cc is a multiple of 64, so a stage is
// 64 consecutive channels of one tap, a whole 128-byte line per pixel.  Src::dSpt divides by the stages per tap, Cc / 64.
struct DmaImgRC64 {
  typedef DmaImgSrc Src;
  static constexpr bool kRC = true;
  const uint16_t* base;
  int32_t pix[8];                  // element offset of the lane's pixel (centre tap) + its 16-byte chunk, per block
  int32_t yx[8];                   // y << 16 | x
  int H, W, Cc, sgn;
  FastDiv dSpt;
  int st_dy, st_dx, st_off;        // of the stage being fetched (wavefront-uniform): tap shift, element offset of tap and channel slice
  __device__ __forceinline__ void init(const Src& m, int o0, int wave, int lane) {
    base = m.base; H = m.H; W = m.W; Cc = m.Cc; sgn = m.sgn; dSpt = m.dSpt;
    st_dy = st_dx = st_off = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int row = wave * 64 + k * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      uint32_t n, rem, y, x;
      m.dHW.divmod((uint32_t)(o0 + row), n, rem);
      m.dW.divmod(rem, y, x);
      pix[k] = (int32_t)(((n * (uint32_t)H + y) * (uint32_t)W + x) * (uint32_t)Cc) + chunk * 8;
      yx[k] = (int32_t)((y << 16) | x);
    }
  }
  // The loads of a stage are issued in order K = 0 .. 7; the first one works out what the stage has in common (a
  // dozen dependent scalar instructions, which would otherwise sit in front of every load of a wavefront that has
  // nothing else to issue meanwhile), the others reuse it.  The choice between the pixel and the line of zeros is a
  // select on the address, not a branch.
  template <int K>
  __device__ __forceinline__ void issue(int d, char* slot, int wave) {
    if constexpr (K == 0) {
      uint32_t tap, cs;
      dSpt.divmod((uint32_t)d, tap, cs);                             // wavefront-uniform
      const int tr = (int)tap / 3, ts = (int)tap - 3 * tr;
      st_dy = sgn * (tr - 1); st_dx = sgn * (ts - 1);
      st_off = (st_dy * W + st_dx) * Cc + (int)cs * 64;
    }
    const int yy = (int)((uint32_t)yx[K] >> 16) + st_dy, xx = (yx[K] & 0xFFFF) + st_dx;
    const bool inside = (unsigned)yy < (unsigned)H && (unsigned)xx < (unsigned)W;
    const uintptr_t there = reinterpret_cast<uintptr_t>(base + (pix[K] + st_off));
    const uintptr_t zeros = reinterpret_cast<uintptr_t>(k_zero_line);
    const uintptr_t mask = inside ? ~(uintptr_t)0 : (uintptr_t)0;
    const uint16_t* p = reinterpret_cast<const uint16_t*>((there & mask) | (zeros & ~mask));
    __builtin_amdgcn_global_load_lds((global_void_ptr)p, (lds_void_ptr)(slot + (wave * 8 + K) * 1024), 16, 0, 0);
  }
};

// The filter read outer-contiguous for the input-gradient pass (see DmaFilterOC), stages of depth 64: Kf is a multiple
// of 64, so a stage is 64 consecutive k of one tap; Src::dSpt divides by the stages per tap, Kf / 64.
struct DmaFilterOC64 {
  typedef DmaFilterSrc Src;
  static constexpr bool kRC = false;
  const uint16_t* p[4];            // lane's source for reduction row (k = row, tap = 0) of blocks 0-3 (4-7: 32 k further)
  int Cc;
  FastDiv dSpt;
  int64_t st_off;                  // element offset of the stage being fetched (wavefront-uniform), set by its first load
  __device__ __forceinline__ void init(const Src& m, int o0, int wave, int lane) {
    Cc = m.Cc; dSpt = m.dSpt; st_off = 0;
    const int pc = lane & 31;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int row = (wave * 4 + k) * 2 + (lane >> 5);
      const int c = 2 * ((pc >> 1) ^ oc_key(row)) + (pc & 1);
      p[k] = m.base + (int64_t)row * 9 * m.Cc + o0 + c * 8;
    }
  }
  template <int K>
  __device__ __forceinline__ void issue(int d, char* slot, int wave) {
    if constexpr (K == 0) {
      uint32_t tap, ks;
      dSpt.divmod((uint32_t)d, tap, ks);
      st_off = ((int64_t)((int)ks * 64) * 9 + tap) * Cc;
    }
    const uint16_t* q = p[K & 3] + (st_off + (int64_t)((K >> 2) * 32 * 9) * Cc);
    __builtin_amdgcn_global_load_lds((global_void_ptr)q, (lds_void_ptr)(slot + (K >> 2) * 16384 + (wave * 4 + (K & 3)) * 1024), 16, 0, 0);
  }
};

// Fragment addresses for the depth-64 slots: two registers per fragment.  RC: the lane's address for the first and
// the second half stage (they differ by an XOR, not by a constant); the slot goes into the immediate.  OC: the two
// transposing reads of a fragment; slot and half stage go into the immediate.
template <bool RC>
struct FragAddr64 {
  uint32_t at[2];
  __device__ __forceinline__ void init(int outer0, int lane, uint32_t operand0) {
    if constexpr (RC) {
      const int r = outer0 + (lane & 15), c = lane >> 4;
#pragma unroll
      for (int kh = 0; kh < 2; ++kh) at[kh] = operand0 + r * 128 + ((((kh << 2) | c) ^ ((r >> 1) & 7)) << 4);
    } else {
      FragAddr<false, 256> f;
      f.init(outer0, lane);
      at[0] = operand0 + f.off[0];
      at[1] = operand0 + f.off[1];
    }
  }
  template <int SLOT4>                                               // SLOT4 = 2 * slot + half stage
  __device__ __forceinline__ half8 read() const {
    if constexpr (RC) {
      return lds_read_b128_imm<(SLOT4 >> 1) * 32768>(at[SLOT4 & 1]);
    } else {
      constexpr int IMM = (SLOT4 >> 1) * 32768 + (SLOT4 & 1) * 16384;
      const uint2v lo = lds_read_tr_b64_imm<IMM>(at[0]);
      const uint2v hi = lds_read_tr_b64_imm<IMM>(at[1]);
      uint4v q = {lo[0], lo[1], hi[0], hi[1]};
      return __builtin_bit_cast(half8, q);
    }
  }
};

template <class AOp, class BOp, bool F32OUT = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_gemm_dma64(typename AOp::Src A, typename BOp::Src B, Problem pb, Epilogue ep) {
  constexpr bool A_RC = AOp::kRC, B_RC = BOp::kRC;
  constexpr int NA = 8, HALF = 4, BM = 256;
  typedef FragSched<NA> Sched;
  constexpr int AD = Sched::kADist;
  constexpr int OPSLOT = 32768, B_BASE = 2 * OPSLOT;
  constexpr int RA1 = A_RC ? 1 : 2, RB1 = B_RC ? 1 : 2;
  static_assert(Sched::kSpread && AD == 2, "the request schedule this kernel was written for");
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  int ti, tj, sp;
  tile_of(pb, blockIdx.x, ti, tj, sp);
  const int i0 = ti * BM, j0 = tj * 256;
  const int d0 = sp * pb.ktiles_per_split;                             // first stage of this workgroup's share of the reduction
  const int nd = min(pb.ktiles_per_split, pb.R / 64 - d0);             // its stages (>= 1: the host plans no empty split)
  const int nst = 2 * nd;                                              // half stages

  AOp da;
  BOp db;
  da.init(A, i0, wave, lane);
  db.init(B, j0, wave, lane);
  // load K of stage d of A / B into slot `sl`; past the end: refetch the last stage into a slot nobody reads
  auto issueA = [&](int d, int sl, auto kc) { da.template issue<decltype(kc)::value>(d0 + min(d, nd - 1), lds + sl * OPSLOT, wave); };
  auto issueB = [&](int d, int sl, auto kc) { db.template issue<decltype(kc)::value>(d0 + min(d, nd - 1), lds + B_BASE + sl * OPSLOT, wave); };
  auto issueA8 = [&](int d, int sl) {
    issueA(d, sl, std::integral_constant<int, 0>{}); issueA(d, sl, std::integral_constant<int, 1>{});
    issueA(d, sl, std::integral_constant<int, 2>{}); issueA(d, sl, std::integral_constant<int, 3>{});
    issueA(d, sl, std::integral_constant<int, 4>{}); issueA(d, sl, std::integral_constant<int, 5>{});
    issueA(d, sl, std::integral_constant<int, 6>{}); issueA(d, sl, std::integral_constant<int, 7>{});
  };
  auto issueB8 = [&](int d, int sl) {
    issueB(d, sl, std::integral_constant<int, 0>{}); issueB(d, sl, std::integral_constant<int, 1>{});
    issueB(d, sl, std::integral_constant<int, 2>{}); issueB(d, sl, std::integral_constant<int, 3>{});
    issueB(d, sl, std::integral_constant<int, 4>{}); issueB(d, sl, std::integral_constant<int, 5>{});
    issueB(d, sl, std::integral_constant<int, 6>{}); issueB(d, sl, std::integral_constant<int, 7>{});
  };
  // prologue: stage 0 whole and the B part of stage 1 (steps 0-3 of stage 0 add its A part); the loads go out first so
  // that the set-up below runs under their latency
  issueA8(0, 0);
  issueB8(0, 0);
  issueB8(1, 1);

  float4v acc[NA][8];
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.f;
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) asm volatile("" : "+a"(acc[a][b]));      // cleared here, under the loads' latency, not behind the barrier
  const uint32_t lds0 = lds_offset(lds);
  FragAddr64<A_RC> aa[NA];
  FragAddr64<B_RC> ab[8];
#pragma unroll
  for (int a = 0; a < NA; ++a) aa[a].init(wm * 128 + a * 16, lane, lds0);
#pragma unroll
  for (int b = 0; b < 8; ++b) ab[b].init(wn * 128 + b * 16, lane, lds0 + B_BASE);
  half8 fa[NA], fb[2][8];

  asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");          // stage 0 has landed everywhere (the 8 loads of B(1) may be in flight)
#pragma unroll
  for (int b = 0; b < 8; ++b) fb[0][b] = ab[b].template read<0>();
#pragma unroll
  for (int a = 0; a < AD; ++a) fa[a] = aa[a].template read<0>();

  // One step of half stage s (SLOT4 = s % 4 = 2 * slot + half): as in k_gemm_dma4, plus this kernel's barriers and loads.
  auto step = [&](int s, auto slotc, auto ac, half8 (&fb_cur)[8], half8 (&fb_nxt)[8]) {
    constexpr int a = decltype(ac)::value, SLOT4 = decltype(slotc)::value;
    constexpr int KH = SLOT4 & 1, SL = SLOT4 >> 1;
    constexpr int SLOT4_A = (SLOT4 + (a + AD) / NA) % 4;               // half stage of the A block requested in this step
    constexpr int SLOT4_B = (SLOT4 + 1) % 4;                           // half stage of the B blocks requested in this step
    if constexpr (KH == 1 && a == HALF) {
      // P: the B requests of this step and the A requests of steps 6, 7 read stage D+1, whose loads (A: steps 0-3 of
      // this stage, B: steps 12-15 of the last one) are all of this wavefront's loads in flight.
      asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    }
    constexpr int B0 = Sched::nb_before(a);
    constexpr int na = (a + AD) % NA;
    __builtin_amdgcn_sched_barrier(0);
    constexpr int W = Sched::allowed(a, RA1, RB1);
    if constexpr (a == 0) wait_frags9<W>(fa[0], fb_cur);
    else wait_frag1<W>(fa[a]);
    if constexpr (KH == 0 && a == 0) {
      // F: this wavefront's reads of stage D-1 have all returned (the LDS returns data in order and the fragments
      // just waited for were requested after them); once every wavefront is here, A(D-1)'s slot may be refilled.
      asm volatile("s_barrier" ::: "memory");
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      mfma_acc(acc[a][b], fb_cur[b], fa[a]);
      if (b == 0) {
        __builtin_amdgcn_sched_barrier(0);
        fa[na] = aa[na].template read<SLOT4_A>();
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int k = 0; k < Sched::nb_at(a); ++k)
        if (b == Sched::b_gap(k)) {
          __builtin_amdgcn_sched_barrier(0);
          fb_nxt[B0 + k] = ab[B0 + k].template read<SLOT4_B>();
          __builtin_amdgcn_sched_barrier(0);
        }
      // two loads per step in gaps that carry no fragment request: behind MFMAs 2 and 6
      if constexpr (KH == 0 && a < HALF) {                             // A(D+1) into the other A slot
        if (b == 2) {
          __builtin_amdgcn_sched_barrier(0);
          issueA((s >> 1) + 1, 1 - SL, std::integral_constant<int, 2 * a>{});
          __builtin_amdgcn_sched_barrier(0);
        }
        if (b == 6) {
          __builtin_amdgcn_sched_barrier(0);
          issueA((s >> 1) + 1, 1 - SL, std::integral_constant<int, 2 * a + 1>{});
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if constexpr (KH == 1 && a >= HALF) {                            // B(D+2) into this stage's B slot
        if (b == 2) {
          __builtin_amdgcn_sched_barrier(0);
          issueB((s >> 1) + 2, SL, std::integral_constant<int, 2 * (a - HALF)>{});
          __builtin_amdgcn_sched_barrier(0);
        }
        if (b == 6) {
          __builtin_amdgcn_sched_barrier(0);
          issueB((s >> 1) + 2, SL, std::integral_constant<int, 2 * (a - HALF) + 1>{});
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto half_stage = [&](int s, auto slotc, half8 (&fb_cur)[8], half8 (&fb_nxt)[8]) {
    step(s, slotc, std::integral_constant<int, 0>{}, fb_cur, fb_nxt);
    step(s, slotc, std::integral_constant<int, 1>{}, fb_cur, fb_nxt);
    step(s, slotc, std::integral_constant<int, 2>{}, fb_cur, fb_nxt);
    step(s, slotc, std::integral_constant<int, 3>{}, fb_cur, fb_nxt);
    step(s, slotc, std::integral_constant<int, 4>{}, fb_cur, fb_nxt);
    step(s, slotc, std::integral_constant<int, 5>{}, fb_cur, fb_nxt);
    step(s, slotc, std::integral_constant<int, 6>{}, fb_cur, fb_nxt);
    step(s, slotc, std::integral_constant<int, 7>{}, fb_cur, fb_nxt);
  };
  typedef std::integral_constant<int, 0> S0;
  typedef std::integral_constant<int, 1> S1;
  typedef std::integral_constant<int, 2> S2;
  typedef std::integral_constant<int, 3> S3;
  // accumulator copies on the edges where the loop's exit and the one-stage tail meet: see k_gemm_dma4
  int s = 0;
  for (; s + 4 <= nst; s += 4) {
    half_stage(s, S0{}, fb[0], fb[1]);
    half_stage(s + 1, S1{}, fb[1], fb[0]);
    half_stage(s + 2, S2{}, fb[0], fb[1]);
    half_stage(s + 3, S3{}, fb[1], fb[0]);
    if (s + 8 > nst) asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  }
  if (s < nst) {                                                       // one stage left, in slot 0
    half_stage(s, S0{}, fb[0], fb[1]);
    half_stage(s + 1, S1{}, fb[1], fb[0]);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  }
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int a = 0; a < NA; ++a) keep_until_here(fa[a]);
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    keep_until_here(fb[0][b]); keep_until_here(fb[1][b]);
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- epilogue: k_gemm_dma4's two forms (whole tiles, 16-byte aligned rows): FP32 straight from the accumulators
  // (store, accumulate, or this split's partial), or the FP16 store through LDS
  bool bad = false;
  if constexpr (F32OUT) {
    const int64_t split_off = (ep.mode == 3) ? (int64_t)sp * pb.I * pb.J : 0;
    float* out = reinterpret_cast<float*>(ep.out) + split_off + (int64_t)(i0 + wm * (BM / 2) + (lane & 15)) * ep.ld + j0 + wn * 128 + ((lane >> 4) << 2);
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int b = 0; b < 8; ++b) {
        asm volatile("" : "+a"(acc[a][b]) : : "memory");              // one block at a time out of the accumulation registers
        float* o = out + (int64_t)(a * 16) * ep.ld + b * 16;
        float4v v = acc[a][b];
        if (ep.mode == 2) {
          const float4v old = *reinterpret_cast<const float4v*>(o);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = __fadd_rn(old[e], v[e]);
        }
        if (ep.flag && ep.mode != 3) {
#pragma unroll
          for (int e = 0; e < 4; ++e) bad |= (__float_as_uint(v[e]) & 0x7F800000u) == 0x7F800000u;
        }
        *reinterpret_cast<float4v*>(o) = v;
      }
    if (ep.flag != nullptr && ep.mode != 3) {
      const unsigned long long vote = __builtin_amdgcn_ballot_w64(bad);
      if (vote != 0ull && lane == 0) atomicOr(ep.flag, 1u);
    }
    return;
  }
  __syncthreads();
  char* mine = lds + wave * (BM / 2 * 256);
  const int li = lane & 15, lg = lane >> 4;
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      asm volatile("" : "+a"(acc[a][b]) : : "memory");
      half4 h;
#pragma unroll
      for (int e = 0; e < 4; ++e) h[e] = (_Float16)acc[a][b][e];
      *reinterpret_cast<half4*>(mine + (a * 16 + li) * 256 + (((2 * b + (lg >> 1)) ^ li) << 4) + (lg & 1) * 8) = h;
    }
  uint16_t* out = reinterpret_cast<uint16_t*>(ep.out) + (int64_t)(i0 + wm * (BM / 2)) * ep.ld + j0 + wn * 128 + li * 8;
  ExpMax emax;
#pragma unroll 8
  for (int it = 0; it < BM / 8; ++it) {
    const int r = it * 4 + lg;
    uint4v q = *reinterpret_cast<const uint4v*>(mine + r * 256 + ((li ^ (r & 15)) << 4));
    if (ep.act == 1) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        q[e] &= (half_bits_positive(q[e]) ? 0x0000FFFFu : 0u) | (half_bits_positive(q[e] >> 16) ? 0xFFFF0000u : 0u);
    } else if (ep.act == 2) {
      const uint4v m = *reinterpret_cast<const uint4v*>(ep.mask + (int64_t)(i0 + wm * (BM / 2) + r) * ep.ldmask + j0 + wn * 128 + li * 8);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        q[e] &= (half_bits_positive(m[e]) ? 0x0000FFFFu : 0u) | (half_bits_positive(m[e] >> 16) ? 0xFFFF0000u : 0u);
    }
    if (ep.flag) {
#pragma unroll
      for (int e = 0; e < 4; ++e) emax.add(q[e]);
    }
    // nontemporal: the tile is not read again by this kernel, and lines that do not linger in the L2 need no write-back when
    // the kernel ends (measured, interleaved with the cached form: 1 - 4 us per launch at 4096^3)
    __builtin_nontemporal_store(q, reinterpret_cast<uint4v*>(out + (int64_t)r * ep.ld));
  }
  bad = emax.special();
  if (ep.flag != nullptr) {
    const unsigned long long vote = __builtin_amdgcn_ballot_w64(bad);
    if (vote != 0ull && lane == 0) atomicOr(ep.flag, 1u);
  }
}

// Sum split partials in split order, then store once.  A pass of its own on purpose: folded into the producing kernel
// (the workgroup that stores a tile's last partial adds the tile up) it left the additions to a handful of workgroups,
// each bound by the latency of its own loads: 16 splits of a 256 x 1024 output took 184 us instead of 14.
__global__ __launch_bounds__(256) void k_split_reduce(const float* __restrict__ part, int splits, int I, int J, Epilogue ep) {
  const int64_t total = (int64_t)I * J;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  bool bad = false;
  if (idx < total) {
    const int64_t i = idx / J, j = idx - i * J;
    bad = reduce_one(part, splits, total, idx, i, j, ep);
  }
  if (ep.flag != nullptr) {
    const unsigned long long vote = __builtin_amdgcn_ballot_w64(bad);
    if (vote != 0ull && (threadIdx.x & 63) == 0) atomicOr(ep.flag, 1u);
  }
}

// The same reduction four adjacent columns per thread, for outputs whose rows hold a whole number of such groups at
// 16-byte (FP32) / 8-byte (FP16, mask) aligned addresses - the host checks that: 16 bytes per lane from each partial,
// one 8- or 16-byte store.  Each element's additions are those of reduce_one, in the same order.
__global__ __launch_bounds__(256) void k_split_reduce4(const float* __restrict__ part, int splits, int I, int J, Epilogue ep) {
  const int64_t total = (int64_t)I * J, total4 = total >> 2;
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  bool bad = false;
  if (q < total4) {
    const float4v* p4 = reinterpret_cast<const float4v*>(part);
    float4v s = p4[q];
    int k = 1;
    for (; k + 8 <= splits; k += 8) {
      float4v v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p4[(int64_t)(k + u) * total4 + q];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) s[e] = __fadd_rn(s[e], v[u][e]);
    }
    for (; k < splits; ++k) {
      const float4v v = p4[(int64_t)k * total4 + q];
#pragma unroll
      for (int e = 0; e < 4; ++e) s[e] = __fadd_rn(s[e], v[e]);
    }
    const int64_t idx = q << 2, i = idx / J, j = idx - i * J;
    if (ep.mode == 0) {
      half4 h;
#pragma unroll
      for (int e = 0; e < 4; ++e) h[e] = (_Float16)s[e];
      const uint2v mk = ep.act == 2 ? *reinterpret_cast<const uint2v*>(ep.mask + i * ep.ldmask + j) : uint2v{0u, 0u};
      const uint2v hb = apply_act4(__builtin_bit_cast(uint2v, h), ep, mk);
      bad = half_bits_special(hb[0]) | half_bits_special(hb[0] >> 16) | half_bits_special(hb[1]) | half_bits_special(hb[1] >> 16);
      *reinterpret_cast<uint2v*>(reinterpret_cast<uint16_t*>(ep.out) + i * ep.ld + j) = hb;
    } else {
      float4v* o = reinterpret_cast<float4v*>(reinterpret_cast<float*>(ep.out) + i * ep.ld + j);
      if (ep.mode == 2) {
        const float4v old = *o;
#pragma unroll
        for (int e = 0; e < 4; ++e) s[e] = __fadd_rn(old[e], s[e]);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) bad |= (__float_as_uint(s[e]) & 0x7F800000u) == 0x7F800000u;
      *o = s;
    }
  }
  if (ep.flag != nullptr) {
    const unsigned long long vote = __builtin_amdgcn_ballot_w64(bad);
    if (vote != 0ull && (threadIdx.x & 63) == 0) atomicOr(ep.flag, 1u);
  }
}

// Launches the reduction of `splits` partial outputs [split][I][J] at `ws` into the final form `ep`.
void launch_split_reduce(hipStream_t s, const void* ws, int splits, int I, int J, const Epilogue& ep) {
  const int64_t total = (int64_t)I * J;
  const bool out_ok = ep.mode == 0 ? ((ep.ld % 4) == 0 && mpt_aligned(ep.out, 8) && (ep.act != 2 || ((ep.ldmask % 4) == 0 && mpt_aligned(ep.mask, 8))))
                                   : ((ep.ld % 4) == 0 && mpt_aligned(ep.out, 16));
  if ((J % 4) == 0 && mpt_aligned(ws, 16) && out_ok)
    hipLaunchKernelGGL(k_split_reduce4, dim3((unsigned)((total / 4 + 255) / 256)), dim3(256), 0, s, reinterpret_cast<const float*>(ws), splits, I, J, ep);
  else
    hipLaunchKernelGGL(k_split_reduce, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, reinterpret_cast<const float*>(ws), splits, I, J, ep);
}

// ---------------------------------------------------------------- host-side planning
struct Plan {
  bool big;             // 256x256 tiles (8 wavefronts) or 128x128 (4 wavefronts)
  int splits, ktiles_per_split, tiles_i, tiles_j;
};

constexpr int kCUs = 256;

Plan make_plan(int64_t I, int64_t J, int64_t R, bool allow_split) {
  static const int force_tile = MPT_TUNABLE("MPT_GEMM_TILE", 0);      // 128 / 256 force a tile size (tuning builds only)
  static const int force_split = MPT_TUNABLE("MPT_GEMM_SPLITS", 0);   // >0 forces a split count (tuning builds only)
  Plan p;
  const int64_t t256 = ((I + 255) / 256) * ((J + 255) / 256);
  p.big = t256 >= kCUs / 2;
  if (allow_split && !p.big) {
    // with a workspace, splitting the reduction can fill the chip with 256 x 256 tiles too (measured: the batch-256
    // gate product's activation gradient 83 -> 58 us, the convolution's weight gradient 195 -> 140 us)
    const int64_t kt64 = (R + BK - 1) / BK;
    int64_t sp = kCUs / t256;
    if (sp > kt64 / 8) sp = kt64 / 8;
    if (sp > 64) sp = 64;
    if (sp >= 1 && t256 * sp >= kCUs / 2) p.big = true;
  }
  if (force_tile == 128) p.big = false;
  if (force_tile == 256) p.big = true;
  const int tile = p.big ? 256 : 128;
  p.tiles_i = (int)((I + tile - 1) / tile);
  p.tiles_j = (int)((J + tile - 1) / tile);
  const int64_t tiles = (int64_t)p.tiles_i * p.tiles_j;
  const int kt = (int)((R + BK - 1) / BK);
  int splits = 1;
  if (allow_split && tiles < kCUs) {
    splits = (int)(kCUs / tiles);
    // keep >= 8 k-tiles per split; a short reduction (the latency-bound layers of a small network, one memory round
    // trip per k-tile) may go down to 2 per split, up to 8 splits
    int max_by_depth = kt / 8;
    const int short_r = kt / 2 < 8 ? kt / 2 : 8;
    if (max_by_depth < short_r) max_by_depth = short_r;
    if (max_by_depth < 1) max_by_depth = 1;
    if (splits > max_by_depth) splits = max_by_depth;
    if (splits > 64) splits = 64;
  }
  if (allow_split && force_split > 0) splits = force_split < kt ? force_split : kt;
  if (splits < 1) splits = 1;
  p.ktiles_per_split = (kt + splits - 1) / splits;
  p.splits = (kt + p.ktiles_per_split - 1) / p.ktiles_per_split;   // no empty split
  return p;
}

size_t plan_ws_bytes(const Plan& p, int64_t I, int64_t J) {
  return p.splits > 1 ? (size_t)p.splits * (size_t)I * (size_t)J * sizeof(float) : 0;
}

// A second way to split: 128 x 256 tiles of the streamed kernel, for outputs whose row count is an odd multiple of 128
// (256-row tiles would compute a padded half tile: 128 x 4096 x 4096 forward 27.5 -> 18.8 us) and whose time the memory
// traffic decides: few tiles and an arithmetic intensity (every operand and the result once) below the ridge of
// 2.5 PFLOP/s / 8 TB/s.  (For row counts that are multiples of 256 it measured within 2 % of the 256-row plans either
// way - gate input gradient 55.8 against 55.5 us, projection 22.7 against 23.2 - and is used only as noted below.)
// Depends on the shape only, so that the workspace size can be asked for beforehand.
bool plan_split128(int64_t I, int64_t J, int64_t R, Plan& p) {
  if ((I % 128) || (J % 256) || (R % 64)) return false;
  const int64_t t128 = (I / 128) * (J / 256), kt = R / 64;
  // rows a multiple of 256: only the smallest outputs over the longest reductions, where 256-row tiles would need 64
  // splits (256 x 1024 over 32768: 40.5 -> 34.1 us; 256 x 2048 over 32768 is 3 us slower this way, over 8192 the same)
  if ((I % 256) == 0 && !(t128 <= 8 && kt / 8 >= kCUs / t128)) return false;
  if (t128 >= kCUs * 3 / 4) return false;
  int64_t splits = kCUs / t128;
  if (splits > kt / 8) splits = kt / 8;                               // at least 8 stages of 64 per workgroup
  if (splits > 64) splits = 64;
  if (splits < 2 || t128 * splits < kCUs * 3 / 8) return false;
  const double flops = 2.0 * (double)I * (double)J * (double)R, bytes = 2.0 * ((double)I * R + (double)R * J + (double)I * J);
  if (flops >= 312.5 * bytes) return false;
  p.big = false;
  p.tiles_i = (int)(I / 128);
  p.tiles_j = (int)(J / 256);
  p.ktiles_per_split = (int)((kt + splits - 1) / splits);
  p.splits = (int)((kt + p.ktiles_per_split - 1) / p.ktiles_per_split);   // no empty split
  return p.splits >= 2;
}

template <class AView, class BView, bool A_ALIGNED, bool B_ALIGNED>
int launch_tiles(hipStream_t s, const AView& A, const BView& B, const Plan& pl, int I, int J, int R, const Epilogue& ep) {
  Problem pb{I, J, R, pl.tiles_i, pl.tiles_j, pl.splits, pl.ktiles_per_split};
  const unsigned grid = (unsigned)((int64_t)pl.tiles_i * pl.tiles_j * pl.splits);
  if (pl.big) {
    auto k = k_gemm<AView, BView, A_ALIGNED, B_ALIGNED, 256, 256, 128, 64>;
    constexpr int lds = 2 * (256 + 256) * ROWB;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, lds), true);
    (void)once;
    hipLaunchKernelGGL(k, dim3(grid), dim3(512), lds, s, A, B, pb, ep);
  } else {
    auto k = k_gemm<AView, BView, A_ALIGNED, B_ALIGNED, 128, 128, 64, 64>;
    constexpr int lds = 2 * (128 + 128) * ROWB;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, lds), true);
    (void)once;
    hipLaunchKernelGGL(k, dim3(grid), dim3(256), lds, s, A, B, pb, ep);
  }
  MPT_LAUNCH_CHECK();
  return MPT_OK;
}

// Plain-matrix views can take the streamed kernel.
template <class V> struct DmaKind { static constexpr bool ok = false; static constexpr bool rc = true; };
template <> struct DmaKind<MatRC> { static constexpr bool ok = true; static constexpr bool rc = true; };
template <> struct DmaKind<MatOC> { static constexpr bool ok = true; static constexpr bool rc = false; };

template <class AView, class BView>
bool try_launch_dma(hipStream_t s, const AView& A, const BView& B, bool aligned, const Plan& pl, int I, int J, int R, const Epilogue& ep, int& status) {
  if constexpr (DmaKind<AView>::ok && DmaKind<BView>::ok) {
    static const bool enabled = MPT_TUNABLE("MPT_GEMM_STREAMED", 1) != 0;
    if (!enabled || !aligned || !pl.big || (I % 256) || (J % 256) || (R % 64)) return false;
    if (ep.mode != 0 && ((ep.ld % 4) || !mpt_aligned(ep.out, 16))) return false;      // FP32 outputs go out 16 bytes per lane
    // FP16 stores of unsplit problems into 16-byte aligned rows take the one-wavefront-per-SIMD kernel (same speed at one
    // tile per CU, about 5 % faster over several); split partials and odd output strides take k_gemm_dma.
    static const int nwaves = MPT_TUNABLE("MPT_GEMM_WAVES", 4);           // 8 forces k_gemm_dma (tuning builds only)
    const bool four = nwaves == 4 && ep.mode == 0 && pl.splits == 1 && (ep.ld % 8) == 0 && mpt_aligned(ep.out, 16) &&
                      (ep.act != 2 || ((ep.ldmask % 8) == 0 && mpt_aligned(ep.mask, 16)));
    auto k4 = k_gemm_dma<DmaKind<AView>::rc, DmaKind<BView>::rc, 4>;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k4), hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 32768), true);
    (void)once;
#ifdef MPT_TUNING
    static const int nstage = MPT_TUNABLE("MPT_GEMM_STAGES", 4);          // 4 or 5 ring slots of 32 KiB
    auto k5 = k_gemm_dma<DmaKind<AView>::rc, DmaKind<BView>::rc, 5>;
    auto kw4 = k_gemm_dma4<DmaOperand4<DmaKind<AView>::rc, 256>, DmaOperand4<DmaKind<BView>::rc, 256>, 256>;
    static bool once_t = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k5), hipFuncAttributeMaxDynamicSharedMemorySize, 5 * 32768),
                          (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kw4), hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 32768), true);
    (void)once_t;
#endif
    Problem pb{I, J, R, pl.tiles_i, pl.tiles_j, pl.splits, pl.ktiles_per_split};
    const unsigned grid = (unsigned)((int64_t)pl.tiles_i * pl.tiles_j * pl.splits);
    auto k64 = k_gemm_dma64<DmaOperand64<DmaKind<AView>::rc>, DmaOperand64<DmaKind<BView>::rc>>;
    auto k64f = k_gemm_dma64<DmaOperand64<DmaKind<AView>::rc>, DmaOperand64<DmaKind<BView>::rc>, true>;
    static bool once64 = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k64), hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 32768),
                          (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k64f), hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 32768), true);
    (void)once64;
    static const int depth32_f32 = MPT_TUNABLE("MPT_GEMM_F32_DEPTH32", 0);   // 1: FP32 outputs on k_gemm_dma (tuning builds only)
#ifdef MPT_TUNING
    static const int depth = MPT_TUNABLE("MPT_GEMM_DEPTH", MPT_GEMM_DEPTH_DEFAULT);   // 32: k_gemm_dma4
    if (four && depth != 64) {
      hipLaunchKernelGGL(kw4, dim3(grid), dim3(256), 4 * 32768, s, DmaMat{A.base, A.ld}, DmaMat{B.base, B.ld}, pb, ep);
    } else if (!four && nstage == 5) {
      hipLaunchKernelGGL(k5, dim3(grid), dim3(512), 5 * 32768, s, DmaMat{A.base, A.ld}, DmaMat{B.base, B.ld}, pb, ep);
    } else
#endif
    if (four) {
      hipLaunchKernelGGL(k64, dim3(grid), dim3(256), 4 * 32768, s, DmaMat{A.base, A.ld}, DmaMat{B.base, B.ld}, pb, ep);
    } else if (ep.mode != 0 && depth32_f32 == 0 && pl.ktiles_per_split >= 8) {
      // FP32 outputs (store, accumulate, split partials; 16 bytes per lane, checked above) on the same kernel, unless
      // the reduction is short: over 4 stages k_gemm_dma's two wavefronts per SIMD cover the fill and the write-out of
      // each other (projection weight gradient 8192 x 1024 x 256, accumulated: 24.5 us there, 28.4 us here)
      hipLaunchKernelGGL(k64f, dim3(grid), dim3(256), 4 * 32768, s, DmaMat{A.base, A.ld}, DmaMat{B.base, B.ld}, pb, ep);
    } else {
      hipLaunchKernelGGL(k4, dim3(grid), dim3(512), 4 * 32768, s, DmaMat{A.base, A.ld}, DmaMat{B.base, B.ld}, pb, ep);
    }
    status = hipGetLastError() == hipSuccess ? MPT_OK : MPT_ERR_HIP;
    return true;
  } else {
    return false;
  }
}

// Problems with few 256-row tiles but many 128 x 256 ones (a batch-256 product against a wide weight matrix): one
// unsplit launch of the 128-row variant of the one-wavefront-per-SIMD kernel fills the chip where 256 x 256 tiles
// leave half of it idle; a workspace, if given, is not needed then.
template <class AView, class BView>
bool try_launch_dma128(hipStream_t s, const AView& A, const BView& B, bool aligned, int I, int J, int R, const Epilogue& ep, int& status) {
  if constexpr (DmaKind<AView>::ok && DmaKind<BView>::ok) {
    static const bool enabled = MPT_TUNABLE("MPT_GEMM_STREAMED", 1) != 0 && MPT_TUNABLE("MPT_GEMM_WAVES", 4) == 4 &&
                                MPT_TUNABLE("MPT_GEMM_TILE128", 1) != 0;
    if (!enabled || !aligned || (I % 128) || (J % 256) || (R % 64) || ep.mode != 0) return false;
    if ((ep.ld % 8) || !mpt_aligned(ep.out, 16) || (ep.act == 2 && ((ep.ldmask % 8) || !mpt_aligned(ep.mask, 16)))) return false;
    const int64_t t256 = ((int64_t)(I + 255) / 256) * (J / 256), t128 = (int64_t)(I / 128) * (J / 256);
    if (t256 >= kCUs * 3 / 4 || t128 < kCUs * 3 / 8) return false;
    auto k = k_gemm_dma4<DmaOperand4<DmaKind<AView>::rc, 128>, DmaOperand4<DmaKind<BView>::rc, 256>, 128>;
    constexpr int lds = 4 * (128 + 256) * 64;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, lds), true);
    (void)once;
    Problem pb{I, J, R, I / 128, J / 256, 1, R / 64};
    hipLaunchKernelGGL(k, dim3((unsigned)t128), dim3(256), lds, s, DmaMat{A.base, A.ld}, DmaMat{B.base, B.ld}, pb, ep);
    status = hipGetLastError() == hipSuccess ? MPT_OK : MPT_ERR_HIP;
    return true;
  } else {
    return false;
  }
}

// The split 128-row plan on the streamed kernel's FP32 epilogue: partials [split][I][J] into the workspace.
template <class AView, class BView>
bool try_launch_split128(hipStream_t s, const AView& A, const BView& B, bool aligned, const Plan& p, int I, int J, int R, float* ws, int& status) {
  if constexpr (DmaKind<AView>::ok && DmaKind<BView>::ok) {
    static const bool enabled = MPT_TUNABLE("MPT_GEMM_STREAMED", 1) != 0 && MPT_TUNABLE("MPT_GEMM_SPLIT128", 1) != 0;
    if (!enabled || !aligned || !mpt_aligned(ws, 16)) return false;
    auto k = k_gemm_dma4<DmaOperand4<DmaKind<AView>::rc, 128>, DmaOperand4<DmaKind<BView>::rc, 256>, 128, true>;
    constexpr int lds = 4 * (128 + 256) * 64;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, lds), true);
    (void)once;
    Problem pb{I, J, R, p.tiles_i, p.tiles_j, p.splits, p.ktiles_per_split};
    Epilogue part{ws, J, 3, nullptr, 0, nullptr, 0};
    hipLaunchKernelGGL(k, dim3((unsigned)((int64_t)p.tiles_i * p.tiles_j * p.splits)), dim3(256), lds, s, DmaMat{A.base, A.ld}, DmaMat{B.base, B.ld}, pb, part);
    status = hipGetLastError() == hipSuccess ? MPT_OK : MPT_ERR_HIP;
    return true;
  } else {
    return false;
  }
}

// Run one contraction: single pass, or split partials + ordered reduction.
template <class AView, class BView>
int run(hipStream_t s, const AView& A, const BView& B, bool a_aligned, bool b_aligned, int I, int J, int R, Epilogue ep, void* ws, size_t ws_bytes) {
  const bool aligned = a_aligned && b_aligned;
  const Plan pl = make_plan(I, J, R, ws != nullptr);
  if (ws != nullptr && ws_bytes < plan_ws_bytes(pl, I, J)) return MPT_ERR_WORKSPACE;
  int st = MPT_OK;
  // Few 256-row tiles but many 128 x 256 ones: the unsplit 128-row launch, unless a workspace is there, the reduction is
  // long and splitting it over 256-row tiles occupies at least a quarter more CUs (time-batched products of a recurrent
  // layer: 5120 x 1024 over 32768 has 160 tiles of 128 rows, but 80 x 3 of 256: 613 -> 318 us; over 8192: 99 -> 82 us).
  // The split writes and reads back 67 MB of partials whatever the shape, about 20 us: below a reduction length of 8192
  // that costs more than the idle CUs do (2048 x 2048 over 1024: 16 us unsplit, 33 us split; over 4096: 47 us either way;
  // over 8192: 88 against 70 us).
  const int64_t t128 = (int64_t)(I / 128) * (J / 256);
  const bool rather_split = ws != nullptr && pl.big && pl.splits > 1 && R >= 8192 && (int64_t)pl.tiles_i * pl.tiles_j * pl.splits * 4 >= t128 * 5;
  if (!rather_split && try_launch_dma128(s, A, B, aligned, I, J, R, ep, st)) return st;
  Plan p128;
  if (ws != nullptr && plan_split128(I, J, R, p128) && ws_bytes >= plan_ws_bytes(p128, I, J) &&
      try_launch_split128(s, A, B, aligned, p128, I, J, R, reinterpret_cast<float*>(ws), st)) {
    if (st != MPT_OK) return st;
    launch_split_reduce(s, ws, p128.splits, I, J, ep);
    MPT_LAUNCH_CHECK();
    return MPT_OK;
  }
  Epilogue first = ep;
  if (pl.splits > 1) {
    first.out = ws; first.ld = J; first.mode = 3; first.flag = nullptr;
  }
  if (!try_launch_dma(s, A, B, aligned, pl, I, J, R, first, st))
    st = a_aligned ? (b_aligned ? launch_tiles<AView, BView, true, true>(s, A, B, pl, I, J, R, first)
                                : launch_tiles<AView, BView, true, false>(s, A, B, pl, I, J, R, first))
                   : (b_aligned ? launch_tiles<AView, BView, false, true>(s, A, B, pl, I, J, R, first)
                                : launch_tiles<AView, BView, false, false>(s, A, B, pl, I, J, R, first));
  if (st != MPT_OK) return st;
  if (pl.splits > 1) {
    launch_split_reduce(s, ws, pl.splits, I, J, ep);
    MPT_LAUNCH_CHECK();
  }
  return MPT_OK;
}

bool dims_ok(int64_t a, int64_t b, int64_t c) {
  const int64_t lim = 0x7FFFFFFF - 512;
  return a >= 1 && b >= 1 && c >= 1 && a <= lim && b <= lim && c <= lim;
}
// A plain matrix can use 16-byte chunk loads when its base and row stride keep every chunk aligned
// and its contiguous extent is a whole number of chunks.
bool mat_fast(const void* p, int64_t ld, int64_t contiguous_extent) {
  return mpt_aligned(p, 16) && (ld % 8) == 0 && (contiguous_extent % 8) == 0;
}

}  // namespace

// ---------------------------------------------------------------- C ABI: GEMMs
extern "C" size_t mpt_gemm_workspace_bytes(int op, int64_t M, int64_t N, int64_t K) {
  if (!dims_ok(M, N, K)) return 0;
  int64_t I, J, R;
  switch (op) {
    case MPT_OP_FWD: I = M; J = N; R = K; break;
    case MPT_OP_DGRAD: I = M; J = K; R = N; break;
    case MPT_OP_WGRAD: I = K; J = N; R = M; break;
    default: return 0;
  }
  // the larger of what the two ways of splitting need: which one runs also depends on the operands' alignment
  size_t need = plan_ws_bytes(make_plan(I, J, R, true), I, J);
  Plan p128;
  if (plan_split128(I, J, R, p128)) need = std::max(need, plan_ws_bytes(p128, I, J));
  return need;
}

namespace {
int gemm_fwd_impl(void* stream, int64_t M, int64_t N, int64_t K, const uint16_t* X, int64_t ldx, const uint16_t* W, int64_t ldw,
                  uint16_t* Y, int64_t ldy, int act, void* ws, size_t ws_bytes) {
  if (X == nullptr || W == nullptr || Y == nullptr) return MPT_ERR_NULL;
  if (!dims_ok(M, N, K) || ldx < K || ldw < N || ldy < N) return MPT_ERR_SHAPE;
  if (!mpt_aligned(X, 2) || !mpt_aligned(W, 2) || !mpt_aligned(Y, 2) || (ws && !mpt_aligned(ws, 16))) return MPT_ERR_ALIGN;
  MatRC A{X, ldx, (int)M, (int)K};
  MatOC B{W, ldw, (int)N, (int)K};
  Epilogue ep{Y, ldy, 0, nullptr, act, nullptr, 0};
  return run(static_cast<hipStream_t>(stream), A, B, mat_fast(X, ldx, K), mat_fast(W, ldw, N), (int)M, (int)N, (int)K, ep, ws, ws_bytes);
}

int gemm_dgrad_impl(void* stream, int64_t M, int64_t N, int64_t K, const uint16_t* dY, int64_t ldy, const uint16_t* W, int64_t ldw,
                    const uint16_t* H, int64_t ldh, bool masked, uint16_t* dX, int64_t ldx, void* ws, size_t ws_bytes) {
  if (dY == nullptr || W == nullptr || dX == nullptr || (masked && H == nullptr)) return MPT_ERR_NULL;
  if (!dims_ok(M, N, K) || ldy < N || ldw < N || ldx < K || (masked && ldh < K)) return MPT_ERR_SHAPE;
  if (!mpt_aligned(dY, 2) || !mpt_aligned(W, 2) || !mpt_aligned(dX, 2) || (masked && !mpt_aligned(H, 2)) || (ws && !mpt_aligned(ws, 16)))
    return MPT_ERR_ALIGN;
  MatRC A{dY, ldy, (int)M, (int)N};
  MatRC B{W, ldw, (int)K, (int)N};
  Epilogue ep{dX, ldx, 0, nullptr, masked ? 2 : 0, masked ? H : nullptr, masked ? ldh : 0};
  return run(static_cast<hipStream_t>(stream), A, B, mat_fast(dY, ldy, N), mat_fast(W, ldw, N), (int)M, (int)K, (int)N, ep, ws, ws_bytes);
}
}  // namespace

extern "C" int mpt_gemm_fwd(void* stream, int64_t M, int64_t N, int64_t K, const uint16_t* X, int64_t ldx,
                            const uint16_t* W, int64_t ldw, uint16_t* Y, int64_t ldy, void* ws, size_t ws_bytes) {
  return gemm_fwd_impl(stream, M, N, K, X, ldx, W, ldw, Y, ldy, 0, ws, ws_bytes);
}

extern "C" int mpt_gemm_fwd_relu(void* stream, int64_t M, int64_t N, int64_t K, const uint16_t* X, int64_t ldx,
                                 const uint16_t* W, int64_t ldw, uint16_t* H, int64_t ldh, void* ws, size_t ws_bytes) {
  return gemm_fwd_impl(stream, M, N, K, X, ldx, W, ldw, H, ldh, 1, ws, ws_bytes);
}

extern "C" int mpt_gemm_dgrad(void* stream, int64_t M, int64_t N, int64_t K, const uint16_t* dY, int64_t ldy,
                              const uint16_t* W, int64_t ldw, uint16_t* dX, int64_t ldx, void* ws, size_t ws_bytes) {
  return gemm_dgrad_impl(stream, M, N, K, dY, ldy, W, ldw, nullptr, 0, false, dX, ldx, ws, ws_bytes);
}

extern "C" int mpt_gemm_dgrad_relu(void* stream, int64_t M, int64_t N, int64_t K, const uint16_t* dY, int64_t ldy,
                                   const uint16_t* W, int64_t ldw, const uint16_t* H, int64_t ldh, uint16_t* dX, int64_t ldx,
                                   void* ws, size_t ws_bytes) {
  return gemm_dgrad_impl(stream, M, N, K, dY, ldy, W, ldw, H, ldh, true, dX, ldx, ws, ws_bytes);
}

extern "C" int mpt_gemm_wgrad(void* stream, int64_t M, int64_t N, int64_t K, const uint16_t* X, int64_t ldx,
                              const uint16_t* dY, int64_t ldy, void* dW, int64_t lddw, int out_fp32, int accumulate,
                              uint32_t* flag, void* ws, size_t ws_bytes) {
  if (X == nullptr || dY == nullptr || dW == nullptr) return MPT_ERR_NULL;
  if (!dims_ok(M, N, K) || ldx < K || ldy < N || lddw < N) return MPT_ERR_SHAPE;
  if (accumulate && !out_fp32) return MPT_ERR_ARG;
  if (!mpt_aligned(X, 2) || !mpt_aligned(dY, 2) || !mpt_aligned(dW, out_fp32 ? 4 : 2) || (flag && !mpt_aligned(flag, 4)) ||
      (ws && !mpt_aligned(ws, 16)))
    return MPT_ERR_ALIGN;
  MatOC A{X, ldx, (int)K, (int)M};
  MatOC B{dY, ldy, (int)N, (int)M};
  Epilogue ep{dW, lddw, out_fp32 ? (accumulate ? 2 : 1) : 0, flag, 0, nullptr, 0};
  return run(static_cast<hipStream_t>(stream), A, B, mat_fast(X, ldx, K), mat_fast(dY, ldy, N), (int)K, (int)N, (int)M, ep, ws, ws_bytes);
}

// ---------------------------------------------------------------- weight gradient for callers that cannot allocate
// The split partials of mpt_gemm_wgrad normally live in a workspace the caller allocates.  This array stands in for
// it: device memory that exists from the moment the code object is loaded, one copy per GPU, kept until the process
// ends.  In host code the array's name is not a device address; the address is looked up once per device with
// hipGetSymbolAddress and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[MPT_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];            // per device; written once under the mutex
std::mutex g_scratch_mutex;

int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MPT_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return MPT_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MPT_OK;
}
}  // namespace

extern "C" int mpt_gemm_wgrad_static(void* stream, int64_t M, int64_t N, int64_t K, const uint16_t* X, int64_t ldx,
                                     const uint16_t* dY, int64_t ldy, void* dW, int64_t lddw, int out_fp32, int accumulate,
                                     uint32_t* flag) {
  if (X == nullptr || dY == nullptr || dW == nullptr) return MPT_ERR_NULL;
  if (!dims_ok(M, N, K) || ldx < K || ldy < N || lddw < N) return MPT_ERR_SHAPE;
  if (accumulate && !out_fp32) return MPT_ERR_ARG;
  // the split this shape would use must fit the array; nothing is launched otherwise
  if (mpt_gemm_workspace_bytes(MPT_OP_WGRAD, M, N, K) > (size_t)MPT_STATIC_SCRATCH_BYTES) return MPT_ERR_WORKSPACE;
  void* ws = nullptr;
  const int st = static_scratch(&ws);
  if (st != MPT_OK) return st;
  return mpt_gemm_wgrad(stream, M, N, K, X, ldx, dY, ldy, dW, lddw, out_fp32, accumulate, flag, ws, (size_t)MPT_STATIC_SCRATCH_BYTES);
}

// ---------------------------------------------------------------- C ABI: 3x3 convolution
namespace {
bool conv_ok(int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Kf) {
  const int64_t lim = 0x7FFFFFFF - 512;
  if (Nb < 1 || H < 1 || W < 1 || C < 1 || Kf < 1) return false;
  if ((C % 8) != 0 || (Kf % 8) != 0) return false;
  if (Nb * H * W > lim || 9 * C > lim || 9 * Kf > lim) return false;
  if (Nb * H * W * C > (int64_t)1 << 40 || Nb * H * W * Kf > (int64_t)1 << 40) return false;
  return true;
}
}  // namespace

extern "C" size_t mpt_conv3x3_workspace_bytes(int op, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Kf) {
  if (!conv_ok(Nb, H, W, C, Kf)) return 0;
  const int64_t P = Nb * H * W;
  int64_t I, J, R;
  switch (op) {
    case MPT_OP_FWD: I = P; J = Kf; R = 9 * C; break;
    case MPT_OP_DGRAD: I = P; J = C; R = 9 * Kf; break;
    case MPT_OP_WGRAD: I = Kf; J = 9 * C; R = P; break;
    default: return 0;
  }
  return plan_ws_bytes(make_plan(I, J, R, true), I, J);
}

namespace {
// Whole-tile convolutions (pixel count a multiple of the tile rows, 256 output channels per tile column, input
// channels a multiple of 64) take the streamed one-wavefront-per-SIMD kernel with a gathered A operand.
template <class BOp, class BOp64>
bool try_launch_conv_dma(hipStream_t s, const uint16_t* img, int64_t H, int64_t W, int64_t Cin, int sgn, const typename BOp::Src& B,
                         const typename BOp64::Src& B64, int64_t P, int64_t J, uint16_t* out, int& status) {
  static const bool enabled = MPT_TUNABLE("MPT_GEMM_STREAMED", 1) != 0 && MPT_TUNABLE("MPT_CONV_STREAMED", 1) != 0;
  if (!enabled || (J % 256) || (Cin % 64) || H >= 65536 || W >= 65536 || P * Cin >= (1LL << 31) || P * J >= (1LL << 31)) return false;
  const int R = (int)(9 * Cin);
  const DmaImgSrc A{img, (int)H, (int)W, (int)Cin, sgn, FastDiv((uint32_t)(H * W)), FastDiv((uint32_t)W), FastDiv((uint32_t)(Cin / 32))};
  Epilogue ep{out, J, 0, nullptr, 0, nullptr, 0};
  const int64_t t256 = (P / 256) * (J / 256), t128 = (P / 128) * (J / 256);
#ifdef MPT_TUNING
  static const int depth = MPT_TUNABLE("MPT_GEMM_DEPTH", MPT_GEMM_DEPTH_DEFAULT);
#else
  constexpr int depth = 64;
#endif
  if (depth == 64 && (P % 256) == 0 && t256 >= kCUs * 3 / 8) {
    auto k = k_gemm_dma64<DmaImgRC64, BOp64>;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 32768), true);
    (void)once;
    const DmaImgSrc A64{img, (int)H, (int)W, (int)Cin, sgn, FastDiv((uint32_t)(H * W)), FastDiv((uint32_t)W), FastDiv((uint32_t)(Cin / 64))};
    Problem pb{(int)P, (int)J, R, (int)(P / 256), (int)(J / 256), 1, R / 64};
    hipLaunchKernelGGL(k, dim3((unsigned)t256), dim3(256), 4 * 32768, s, A64, B64, pb, ep);
#ifdef MPT_TUNING
  } else if ((P % 256) == 0 && t256 >= kCUs * 3 / 8) {
    auto k = k_gemm_dma4<DmaImgRC<256>, BOp, 256>;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 32768), true);
    (void)once;
    Problem pb{(int)P, (int)J, R, (int)(P / 256), (int)(J / 256), 1, R / 64};
    hipLaunchKernelGGL(k, dim3((unsigned)t256), dim3(256), 4 * 32768, s, A, B, pb, ep);
#endif
  } else if ((P % 128) == 0 && t128 >= kCUs * 3 / 8) {
    auto k = k_gemm_dma4<DmaImgRC<128>, BOp, 128>;
    constexpr int lds = 4 * (128 + 256) * 64;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, lds), true);
    (void)once;
    Problem pb{(int)P, (int)J, R, (int)(P / 128), (int)(J / 256), 1, R / 64};
    hipLaunchKernelGGL(k, dim3((unsigned)t128), dim3(256), lds, s, A, B, pb, ep);
  } else {
    return false;
  }
  status = hipGetLastError() == hipSuccess ? MPT_OK : MPT_ERR_HIP;
  return true;
}
}  // namespace

extern "C" int mpt_conv3x3_fwd(void* stream, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Kf, const uint16_t* x,
                               const uint16_t* w, uint16_t* y, void* ws, size_t ws_bytes) {
  if (x == nullptr || w == nullptr || y == nullptr) return MPT_ERR_NULL;
  if (!conv_ok(Nb, H, W, C, Kf)) return MPT_ERR_SHAPE;
  if (!mpt_aligned(x, 16) || !mpt_aligned(w, 16) || !mpt_aligned(y, 16) || (ws && !mpt_aligned(ws, 16))) return MPT_ERR_ALIGN;
  {
    int st = MPT_OK;                 // the workspace, if any, is not needed on this path (its size was not checked: nothing is written to it)
    if (ws == nullptr || ws_bytes >= mpt_conv3x3_workspace_bytes(MPT_OP_FWD, Nb, H, W, C, Kf))
      if (try_launch_conv_dma<DmaOperand4<true, 256>, DmaOperand64<true>>(static_cast<hipStream_t>(stream), x, H, W, C, +1, DmaMat{w, 9 * C}, DmaMat{w, 9 * C},
                                                                          Nb * H * W, Kf, y, st)) return st;
  }
  const int P = (int)(Nb * H * W), R = (int)(9 * C);
  ImgRC A{x, (int)H, (int)W, (int)C, P, R, +1, FastDiv((uint32_t)(H * W)), FastDiv((uint32_t)W), FastDiv((uint32_t)C)};
  MatRC B{w, 9 * C, (int)Kf, R};
  Epilogue ep{y, Kf, 0, nullptr, 0, nullptr, 0};
  return run(static_cast<hipStream_t>(stream), A, B, true, true, P, (int)Kf, R, ep, ws, ws_bytes);
}

extern "C" int mpt_conv3x3_dgrad(void* stream, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Kf, const uint16_t* dy,
                                 const uint16_t* w, uint16_t* dx, void* ws, size_t ws_bytes) {
  if (dy == nullptr || w == nullptr || dx == nullptr) return MPT_ERR_NULL;
  if (!conv_ok(Nb, H, W, C, Kf)) return MPT_ERR_SHAPE;
  if (!mpt_aligned(dy, 16) || !mpt_aligned(w, 16) || !mpt_aligned(dx, 16) || (ws && !mpt_aligned(ws, 16))) return MPT_ERR_ALIGN;
  {
    int st = MPT_OK;
    if (ws == nullptr || ws_bytes >= mpt_conv3x3_workspace_bytes(MPT_OP_DGRAD, Nb, H, W, C, Kf))
      if (try_launch_conv_dma<DmaFilterOC, DmaFilterOC64>(static_cast<hipStream_t>(stream), dy, H, W, Kf, -1,
                                                          DmaFilterSrc{w, (int)C, (int)Kf, FastDiv((uint32_t)(Kf / 32))},
                                                          DmaFilterSrc{w, (int)C, (int)Kf, FastDiv((uint32_t)(Kf / 64))}, Nb * H * W, C, dx, st)) return st;
  }
  const int P = (int)(Nb * H * W), R = (int)(9 * Kf);
  ImgRC A{dy, (int)H, (int)W, (int)Kf, P, R, -1, FastDiv((uint32_t)(H * W)), FastDiv((uint32_t)W), FastDiv((uint32_t)Kf)};
  FilterOC B{w, (int)C, (int)Kf, (int)C, R, FastDiv((uint32_t)Kf)};
  Epilogue ep{dx, C, 0, nullptr, 0, nullptr, 0};
  return run(static_cast<hipStream_t>(stream), A, B, true, true, P, (int)C, R, ep, ws, ws_bytes);
}

namespace {
// Weight gradient of a whole-tile convolution (output channels and input channels multiples of 256, pixel count a
// multiple of 64) on the streamed kernel: A = dy as a plain outer-contiguous matrix, B = the image gathered per tap.
// The reduction over the pixels is long and the output small, so it is normally split through the workspace.
bool try_launch_conv_wgrad_dma(hipStream_t s, const uint16_t* x, const uint16_t* dy, int64_t H, int64_t W, int64_t C, int64_t Kf, int64_t P,
                               const Epilogue& ep, void* ws, size_t ws_bytes, int& status) {
  static const bool enabled = MPT_TUNABLE("MPT_GEMM_STREAMED", 1) != 0 && MPT_TUNABLE("MPT_CONV_STREAMED", 1) != 0;
  const int64_t J = 9 * C;
  if (!enabled || (Kf % 256) || (C % 256) || (P % 64) || P * C >= (1LL << 31) || P * Kf >= (1LL << 31)) return false;
  const Plan pl = make_plan(Kf, J, P, ws != nullptr);
  if (!pl.big) return false;
  if (ws != nullptr && ws_bytes < plan_ws_bytes(pl, Kf, J)) { status = MPT_ERR_WORKSPACE; return true; }
  const DmaImgOCSrc B{x, (int)H, (int)W, (int)C, FastDiv((uint32_t)W), FastDiv((uint32_t)H)};
  Problem pb{(int)Kf, (int)J, (int)P, pl.tiles_i, pl.tiles_j, pl.splits, pl.ktiles_per_split};
  const unsigned grid = (unsigned)((int64_t)pl.tiles_i * pl.tiles_j * pl.splits);
  if (pl.splits > 1) {
    auto k = k_gemm_dma4<DmaOperand4<false, 256>, DmaImgOC, 256, true>;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 32768), true);
    (void)once;
    Epilogue first = ep;
    first.out = ws; first.ld = J; first.mode = 3; first.flag = nullptr;
    hipLaunchKernelGGL(k, dim3(grid), dim3(256), 4 * 32768, s, DmaMat{dy, Kf}, B, pb, first);
    if (hipGetLastError() != hipSuccess) { status = MPT_ERR_HIP; return true; }
    launch_split_reduce(s, ws, pl.splits, (int)Kf, (int)J, ep);
  } else {
    auto k = k_gemm_dma4<DmaOperand4<false, 256>, DmaImgOC, 256, false>;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 32768), true);
    (void)once;
    hipLaunchKernelGGL(k, dim3(grid), dim3(256), 4 * 32768, s, DmaMat{dy, Kf}, B, pb, ep);
  }
  status = hipGetLastError() == hipSuccess ? MPT_OK : MPT_ERR_HIP;
  return true;
}
}  // namespace

extern "C" int mpt_conv3x3_wgrad(void* stream, int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Kf, const uint16_t* x,
                                 const uint16_t* dy, uint16_t* dw, uint32_t* flag, void* ws, size_t ws_bytes) {
  if (x == nullptr || dy == nullptr || dw == nullptr) return MPT_ERR_NULL;
  if (!conv_ok(Nb, H, W, C, Kf)) return MPT_ERR_SHAPE;
  if (!mpt_aligned(x, 16) || !mpt_aligned(dy, 16) || !mpt_aligned(dw, 16) || (flag && !mpt_aligned(flag, 4)) ||
      (ws && !mpt_aligned(ws, 16)))
    return MPT_ERR_ALIGN;
  {
    int st = MPT_OK;
    const Epilogue epw{dw, 9 * C, 0, flag, 0, nullptr, 0};
    if (try_launch_conv_wgrad_dma(static_cast<hipStream_t>(stream), x, dy, H, W, C, Kf, Nb * H * W, epw, ws, ws_bytes, st)) return st;
  }
  const int P = (int)(Nb * H * W), J = (int)(9 * C);
  MatOC A{dy, Kf, (int)Kf, P};
  ImgOC B{x, (int)H, (int)W, (int)C, J, P, FastDiv((uint32_t)(H * W)), FastDiv((uint32_t)W), FastDiv((uint32_t)C)};
  Epilogue ep{dw, J, 0, flag, 0, nullptr, 0};
  return run(static_cast<hipStream_t>(stream), A, B, true, true, (int)Kf, J, P, ep, ws, ws_bytes);
}
