// gfx950 kernels of the paged multi-LoRA delta (Sec. II-A Eq. 1 over the page pool of Sec. III-C;
// Sec. IV "Memory Manager": kernels that read adapter weights from non-contiguous pages).
//
// Work decomposition: one work item = one 64-lane wavefront = one workgroup.  Items come from the
// batch translation (tokens grouped by adapter), so every weight byte a batch needs is fetched
// from HBM once per group of tokens, not once per token.
//
//   shrink, vector-ALU item : up to 8 rows of A x up to 4 tokens.  Lanes stride along d_in with
//                             16-byte loads, accumulate in fp32 and finish with a wavefront
//                             reduction.
//   shrink, matrix-core item: 16 rows of A x up to 64 tokens, v_mfma_f32_16x16x32 (bf16 / f16).
//   expand, vector-ALU item : all rows of B x 64 lanes x 16 bytes of columns x up to 4 tokens;
//                             no reduction, read-modify-write of y.
//   expand, matrix-core item: all rows of B x 128 columns x up to 64 tokens; v is split into a
//                             high and a low half so that fp32 v loses nothing that matters.
//
// Address translation: virtual byte o of an adapter is at slab + pt[o >> log2P] * P + (o & (P-1)).
// A 16-byte vector never straddles a page (all offsets are multiples of 16).  Each item stages the
// page-table entries it can touch in LDS first, so the translation in the inner loop is an LDS
// read, and the reduction order depends on virtual offsets only (evicting and reloading an adapter
// onto other pages gives bit-identical results).
#include "plora_internal.h"

namespace plora {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

template <int DT> struct Elt { static constexpr int B = 2, VEC = 8; };
template <> struct Elt<2> { static constexpr int B = 4, VEC = 4; };

__device__ __forceinline__ uint4 ld16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void st16(void* p, uint4 q) { *reinterpret_cast<uint4*>(p) = q; }

__device__ __forceinline__ float half_bits_to_float(uint32_t h) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}

template <int DT>
__device__ __forceinline__ void unpack(const uint4 q, float* f) {
  if constexpr (DT == 2) {
    f[0] = __uint_as_float(q.x); f[1] = __uint_as_float(q.y); f[2] = __uint_as_float(q.z); f[3] = __uint_as_float(q.w);
  } else if constexpr (DT == 1) {
    f[0] = __uint_as_float(q.x << 16); f[1] = __uint_as_float(q.x & 0xffff0000u);
    f[2] = __uint_as_float(q.y << 16); f[3] = __uint_as_float(q.y & 0xffff0000u);
    f[4] = __uint_as_float(q.z << 16); f[5] = __uint_as_float(q.z & 0xffff0000u);
    f[6] = __uint_as_float(q.w << 16); f[7] = __uint_as_float(q.w & 0xffff0000u);
  } else {
    f[0] = half_bits_to_float(q.x & 0xffffu); f[1] = half_bits_to_float(q.x >> 16);
    f[2] = half_bits_to_float(q.y & 0xffffu); f[3] = half_bits_to_float(q.y >> 16);
    f[4] = half_bits_to_float(q.z & 0xffffu); f[5] = half_bits_to_float(q.z >> 16);
    f[6] = half_bits_to_float(q.w & 0xffffu); f[7] = half_bits_to_float(q.w >> 16);
  }
}

// fp32 -> element, round to nearest even.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}

template <int DT>
__device__ __forceinline__ uint4 pack(const float* f) {
  uint4 q;
  if constexpr (DT == 2) {
    q.x = __float_as_uint(f[0]); q.y = __float_as_uint(f[1]); q.z = __float_as_uint(f[2]); q.w = __float_as_uint(f[3]);
  } else if constexpr (DT == 1) {
    q.x = f32_to_bf16_bits(f[0]) | (f32_to_bf16_bits(f[1]) << 16);
    q.y = f32_to_bf16_bits(f[2]) | (f32_to_bf16_bits(f[3]) << 16);
    q.z = f32_to_bf16_bits(f[4]) | (f32_to_bf16_bits(f[5]) << 16);
    q.w = f32_to_bf16_bits(f[6]) | (f32_to_bf16_bits(f[7]) << 16);
  } else {
    q.x = f32_to_f16_bits(f[0]) | (f32_to_f16_bits(f[1]) << 16);
    q.y = f32_to_f16_bits(f[2]) | (f32_to_f16_bits(f[3]) << 16);
    q.z = f32_to_f16_bits(f[4]) | (f32_to_f16_bits(f[5]) << 16);
    q.w = f32_to_f16_bits(f[6]) | (f32_to_f16_bits(f[7]) << 16);
  }
  return q;
}

__device__ __forceinline__ float wave_sum(float s) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
  return s;
}

__device__ __forceinline__ int imin(int a, int b) { return a < b ? a : b; }

// ------------------------------------------------------------------------------------------
// shrink, vector-ALU item
// ------------------------------------------------------------------------------------------
template <int DT, int NT>
__device__ __forceinline__ void shrink_valu_body(const LaunchArgs& a, const SegRec sg, const ItemRec it, const SlotRec sl,
                                                 const uint8_t* __restrict__ x, float* __restrict__ v,
                                                 int32_t* lds_pt) {
  constexpr int EB = Elt<DT>::B, VEC = Elt<DT>::VEC;
  const int lane = threadIdx.x;
  const int r = sg.rank;
  const int d_in = sl.d_in;
  const int vs = a.v_stride;
  int64_t tok[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) tok[i] = a.perm[sg.tok_start + it.tok0 + imin(i, it.ntok - 1)];

  if (it.j0 == 0) {  // the first row block of a token group also clears the unused tail of v
#pragma unroll
    for (int i = 0; i < NT; ++i)
      if (i < it.ntok)
        for (int j = r + lane; j < vs; j += kWave) v[tok[i] * vs + j] = 0.f;
  }
  if (r == 0) return;

  const int nrows = imin(kShrinkRows, r - it.j0);
  const uint64_t rowb = (uint64_t)d_in * EB;
  const uint64_t base = (uint64_t)r * EB * (uint64_t)sl.cum + (uint64_t)it.j0 * rowb;
  const int lp = a.log2_page;
  const uint64_t pmask = ((uint64_t)1 << lp) - 1;
  const uint32_t win0 = (uint32_t)(base >> lp);
  const uint32_t win_n = (uint32_t)((base + (uint64_t)nrows * rowb - 1) >> lp) - win0 + 1;
  const int32_t* ptg = a.pt + sg.pt_off + win0;
  for (uint32_t i = lane; i < win_n; i += kWave) lds_pt[i] = ptg[i];
  __syncthreads();

  float acc[kShrinkRows][NT];
#pragma unroll
  for (int jj = 0; jj < kShrinkRows; ++jj)
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[jj][i] = 0.f;

  for (int k0 = 0; k0 < d_in; k0 += kWave * VEC) {
    const int k = k0 + lane * VEC;
    const bool ok = k < d_in;
    const int kk = ok ? k : 0;
    uint4 wq[kShrinkRows];
#pragma unroll
    for (int jj = 0; jj < kShrinkRows; ++jj) {
      const int jr = imin(jj, nrows - 1);
      const uint64_t voff = base + (uint64_t)jr * rowb + (uint64_t)kk * EB;
      const uint64_t pg = (uint64_t)(uint32_t)lds_pt[(uint32_t)(voff >> lp) - win0];
      wq[jj] = ld16(a.slab + (pg << lp) + (voff & pmask));
    }
    float xf[NT][VEC];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      uint4 xq = ld16(x + ((uint64_t)tok[i] * d_in + kk) * EB);
      if (!ok) xq = make_uint4(0, 0, 0, 0);
      unpack<DT>(xq, xf[i]);
    }
#pragma unroll
    for (int jj = 0; jj < kShrinkRows; ++jj) {
      float wf[VEC];
      unpack<DT>(wq[jj], wf);
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[jj][i] = __builtin_fmaf(wf[e], xf[i][e], acc[jj][i]);
    }
  }
#pragma unroll
  for (int jj = 0; jj < kShrinkRows; ++jj)
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const float s = wave_sum(acc[jj][i]);
      if (lane == 0 && jj < nrows && i < it.ntok) v[tok[i] * vs + it.j0 + jj] = s;
    }
}

template <int DT>
__global__ __launch_bounds__(kWave) void k_shrink_valu(const LaunchArgs a, const SlotPtrs p) {
  __shared__ int32_t lds_pt[kPtWindow];
  const ItemRec it = a.items[blockIdx.x];
  const SegRec sg = a.segs[it.seg];
  const int q = blockIdx.z;
  const SlotRec sl = a.slots[a.slot0 + q];
  const uint8_t* x = (const uint8_t*)p.a[q];
  float* v = (float*)p.b[q];
  if (it.ntok <= 1) shrink_valu_body<DT, 1>(a, sg, it, sl, x, v, lds_pt);
  else if (it.ntok == 2) shrink_valu_body<DT, 2>(a, sg, it, sl, x, v, lds_pt);
  else shrink_valu_body<DT, kValuTok>(a, sg, it, sl, x, v, lds_pt);
}

// ------------------------------------------------------------------------------------------
// expand, vector-ALU item
// ------------------------------------------------------------------------------------------
// Stages, for every row j of B, the physical pages that hold the first and the last byte of the
// item's piece of that row (an item's piece of a row is at most 4096 bytes, a page at least that).
__device__ __forceinline__ void stage_row_pages(const LaunchArgs& a, const SegRec& sg, uint64_t base, uint64_t rowb,
                                                uint32_t piece_bytes, int2* lds_pg) {
  const int lp = a.log2_page;
  const int32_t* ptg = a.pt + sg.pt_off;
  for (int j = threadIdx.x; j < sg.rank; j += kWave) {
    const uint64_t vo = base + (uint64_t)j * rowb;
    const uint32_t q0 = (uint32_t)(vo >> lp);
    const uint32_t q1 = imin((int)((vo + piece_bytes - 1) >> lp), sg.n_pt - 1);
    lds_pg[j] = make_int2(ptg[q0], ptg[q1]);
  }
  __syncthreads();
}

template <int DT, int NT>
__device__ __forceinline__ void expand_valu_body(const LaunchArgs& a, const SegRec sg, const ItemRec it, const SlotRec sl,
                                                 const float* __restrict__ v, uint8_t* __restrict__ y, int2* lds_pg) {
  constexpr int EB = Elt<DT>::B, VEC = Elt<DT>::VEC;
  const int lane = threadIdx.x;
  const int r = sg.rank;
  const int d_out = sl.d_out;
  const int n0w = blockIdx.y * (kWave * VEC);
  if (n0w >= d_out || r == 0) return;
  const int n = n0w + lane * VEC;
  const bool ok = n < d_out;
  const uint32_t lane_b = ok ? lane * 16 : 0;
  const int vs = a.v_stride;
  const int lp = a.log2_page;
  const uint32_t pmask = (1u << lp) - 1;  // pages are at most 2^31 bytes
  const uint64_t rowb = (uint64_t)d_out * EB;
  const uint64_t base = (uint64_t)r * EB * ((uint64_t)sl.cum + (uint64_t)sl.d_in) + (uint64_t)n0w * EB;
  stage_row_pages(a, sg, base, rowb, kWave * 16, lds_pg);

  const float* vrow[NT];
  int64_t tok[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    tok[i] = a.perm[sg.tok_start + it.tok0 + imin(i, it.ntok - 1)];
    vrow[i] = v + tok[i] * vs;
  }
  float acc[NT][VEC];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[i][e] = 0.f;

  constexpr int U = 8;
  int j = 0;
  for (; j + U <= r; j += U) {
    uint4 wq[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t vo = base + (uint64_t)(j + u) * rowb;
      const uint32_t inpage = ((uint32_t)vo & pmask) + lane_b;
      const int2 pp = lds_pg[j + u];
      const uint64_t pg = (uint64_t)(uint32_t)((inpage >> lp) ? pp.y : pp.x);
      wq[u] = ld16(a.slab + (pg << lp) + (inpage & pmask));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float wf[VEC];
      unpack<DT>(wq[u], wf);
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        const float vj = vrow[i][j + u];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[i][e] = __builtin_fmaf(vj, wf[e], acc[i][e]);
      }
    }
  }
  for (; j < r; ++j) {
    const uint64_t vo = base + (uint64_t)j * rowb;
    const uint32_t inpage = ((uint32_t)vo & pmask) + lane_b;
    const int2 pp = lds_pg[j];
    const uint64_t pg = (uint64_t)(uint32_t)((inpage >> lp) ? pp.y : pp.x);
    float wf[VEC];
    unpack<DT>(ld16(a.slab + (pg << lp) + (inpage & pmask)), wf);
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const float vj = vrow[i][j];
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[i][e] = __builtin_fmaf(vj, wf[e], acc[i][e]);
    }
  }
  if (!ok) return;
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    if (i < it.ntok) {
      uint8_t* yp = y + ((uint64_t)tok[i] * d_out + n) * EB;
      float yf[VEC];
      unpack<DT>(ld16(yp), yf);
#pragma unroll
      for (int e = 0; e < VEC; ++e) yf[e] = yf[e] + sg.scale * acc[i][e];
      st16(yp, pack<DT>(yf));
    }
  }
}

template <int DT>
__global__ __launch_bounds__(kWave) void k_expand_valu(const LaunchArgs a, const SlotPtrs p) {
  __shared__ int2 lds_pg[kMaxRank];
  const ItemRec it = a.items[blockIdx.x];
  const SegRec sg = a.segs[it.seg];
  const int q = blockIdx.z;
  const SlotRec sl = a.slots[a.slot0 + q];
  const float* v = (const float*)p.a[q];
  uint8_t* y = (uint8_t*)p.b[q];
  if (it.ntok <= 1) expand_valu_body<DT, 1>(a, sg, it, sl, v, y, lds_pg);
  else if (it.ntok == 2) expand_valu_body<DT, 2>(a, sg, it, sl, v, y, lds_pg);
  else expand_valu_body<DT, kValuTok>(a, sg, it, sl, v, y, lds_pg);
}

// ------------------------------------------------------------------------------------------
// matrix-core items (bf16 / f16 only)
// ------------------------------------------------------------------------------------------
// v_mfma_f32_16x16x32: lane l holds, of the M x K operand, row l%16 and the 8 K-values of group
// l/16; of the K x N operand, column l%16 and the same 8 K-values; of the 16x16 result, column
// l%16 and rows 4*(l/16) .. +3.
template <int DT>
__device__ __forceinline__ f32x4 mfma16(const uint4 a, const uint4 b, const f32x4 c) {
  if constexpr (DT == 1)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// shrink: D[token, row] += X[token, k] * A[row, k].  Within each run of 64 k-values lane group g
// takes k = 16 g .. 16 g + 15 as two 8-wide halves, so a wavefront reads whole 128-byte lines of
// every row; the order of the contraction index is free as long as both operands agree.
template <int DT, int MT>
__device__ __forceinline__ void shrink_mfma_body(const LaunchArgs& a, const SegRec sg, const ItemRec it, const SlotRec sl,
                                                 const uint8_t* __restrict__ x, float* __restrict__ v,
                                                 int32_t* lds_pt) {
  constexpr int EB = 2;
  const int lane = threadIdx.x;
  const int g = lane >> 4, c = lane & 15;
  const int r = sg.rank;
  const int d_in = sl.d_in;
  const int vs = a.v_stride;
  const int lp = a.log2_page;
  const uint64_t pmask = ((uint64_t)1 << lp) - 1;

  if (it.j0 == 0) {  // clear v[t, r .. v_stride) for the item's tokens
    for (int i = 0; i < it.ntok; ++i) {
      const int64_t t = a.perm[sg.tok_start + it.tok0 + i];
      for (int j = r + lane; j < vs; j += kWave) v[t * vs + j] = 0.f;
    }
  }
  const int nrows = imin(kMfmaRows, r - it.j0);
  const uint64_t rowb = (uint64_t)d_in * EB;
  const uint64_t base = (uint64_t)r * EB * (uint64_t)sl.cum + (uint64_t)it.j0 * rowb;
  const uint32_t win0 = (uint32_t)(base >> lp);
  const uint32_t win_n = (uint32_t)((base + (uint64_t)nrows * rowb - 1) >> lp) - win0 + 1;
  const int32_t* ptg = a.pt + sg.pt_off + win0;
  for (uint32_t i = lane; i < win_n; i += kWave) lds_pt[i] = ptg[i];
  __syncthreads();

  const uint64_t wrow = base + (uint64_t)imin(c, nrows - 1) * rowb;
  const uint8_t* xrow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int64_t t = a.perm[sg.tok_start + it.tok0 + imin(mt * 16 + c, it.ntok - 1)];
    xrow[mt] = x + (uint64_t)t * d_in * EB;
  }
  f32x4 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int k0 = 0; k0 < d_in; k0 += 64) {
    const int k = k0 + g * 16;
    const bool ok0 = k < d_in, ok1 = k + 8 < d_in;
    const int ka = ok0 ? k : 0, kb = ok1 ? k + 8 : 0;
    const uint64_t vo0 = wrow + (uint64_t)ka * EB, vo1 = wrow + (uint64_t)kb * EB;
    const uint64_t p0 = (uint64_t)(uint32_t)lds_pt[(uint32_t)(vo0 >> lp) - win0];
    const uint64_t p1 = (uint64_t)(uint32_t)lds_pt[(uint32_t)(vo1 >> lp) - win0];
    uint4 w0 = ld16(a.slab + (p0 << lp) + (vo0 & pmask));
    uint4 w1 = ld16(a.slab + (p1 << lp) + (vo1 & pmask));
    if (!ok0) w0 = make_uint4(0, 0, 0, 0);
    if (!ok1) w1 = make_uint4(0, 0, 0, 0);
    uint4 x0[MT], x1[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      x0[mt] = ld16(xrow[mt] + (uint64_t)ka * EB);
      x1[mt] = ld16(xrow[mt] + (uint64_t)kb * EB);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      acc[mt] = mfma16<DT>(x0[mt], w0, acc[mt]);
      acc[mt] = mfma16<DT>(x1[mt], w1, acc[mt]);
    }
  }
  // result: lane holds weight row it.j0 + c for tokens 4 g .. 4 g + 3 of every tile
  if (c < nrows) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ti = mt * 16 + g * 4 + i;
        if (ti < it.ntok) {
          const int64_t t = a.perm[sg.tok_start + it.tok0 + ti];
          v[t * vs + it.j0 + c] = acc[mt][i];
        }
      }
  }
}

template <int DT>
__global__ __launch_bounds__(kWave) void k_shrink_mfma(const LaunchArgs a, const SlotPtrs p) {
  __shared__ int32_t lds_pt[kPtWindow];
  const ItemRec it = a.items[blockIdx.x];
  const SegRec sg = a.segs[it.seg];
  const int q = blockIdx.z;
  const SlotRec sl = a.slots[a.slot0 + q];
  const uint8_t* x = (const uint8_t*)p.a[q];
  float* v = (float*)p.b[q];
  if (it.ntok <= 16) shrink_mfma_body<DT, 1>(a, sg, it, sl, x, v, lds_pt);
  else if (it.ntok <= 32) shrink_mfma_body<DT, 2>(a, sg, it, sl, x, v, lds_pt);
  else shrink_mfma_body<DT, 4>(a, sg, it, sl, x, v, lds_pt);
}

// Splits 8 fp32 values into a high and a low 16-bit part: hi = round(v), lo = round(v - hi).
template <int DT>
__device__ __forceinline__ void split_hi_lo(const float* f, uint4& hi, uint4& lo) {
  uint32_t h[8], l[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    if constexpr (DT == 1) {
      h[e] = f32_to_bf16_bits(f[e]);
      l[e] = f32_to_bf16_bits(f[e] - __uint_as_float(h[e] << 16));
    } else {
      h[e] = f32_to_f16_bits(f[e]);
      l[e] = f32_to_f16_bits(f[e] - half_bits_to_float(h[e]));
    }
  }
  hi = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
  lo = make_uint4(l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16));
}

// expand: D[token, col] += V[token, j] * B[j, col], K = 32 rows of B per step.  Lane (g, c) loads
// the 8x8 block rows 8 g .. 8 g + 7 x columns 8 c .. 8 c + 7 (16 bytes per row), transposes it in
// registers into eight 8-value K-vectors, one per column offset cc, and issues eight MFMAs whose
// result column l%16 stands for the real column 8 c + cc.  A lane therefore ends up with 8
// consecutive columns of y for each of its 4 token rows: one 16-byte read-modify-write each.
template <int DT, int MT>
__device__ __forceinline__ void expand_mfma_body(const LaunchArgs& a, const SegRec sg, const ItemRec it, const SlotRec sl,
                                                 const float* __restrict__ v, uint8_t* __restrict__ y, int2* lds_pg) {
  constexpr int EB = 2;
  const int lane = threadIdx.x;
  const int g = lane >> 4, c = lane & 15;
  const int r = sg.rank;
  const int d_out = sl.d_out;
  const int n0w = blockIdx.y * kMfmaCols;
  if (n0w >= d_out) return;
  const int n = n0w + 8 * c;
  const bool ok = n < d_out;
  const uint32_t lane_b = ok ? c * 16 : 0;
  const int vs = a.v_stride;
  const int lp = a.log2_page;
  const uint32_t pmask = (1u << lp) - 1;
  const uint64_t rowb = (uint64_t)d_out * EB;
  const uint64_t base = (uint64_t)r * EB * ((uint64_t)sl.cum + (uint64_t)sl.d_in) + (uint64_t)n0w * EB;
  stage_row_pages(a, sg, base, rowb, kMfmaCols * EB, lds_pg);

  const float* vrow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int64_t t = a.perm[sg.tok_start + it.tok0 + imin(mt * 16 + c, it.ntok - 1)];
    vrow[mt] = v + t * vs;
  }
  f32x4 acc[MT][8];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) acc[mt][cc] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int jb = 0; jb < r; jb += 32) {
    uint4 wr[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      const int j = jb + 8 * g + jj;
      const int je = imin(j, r - 1);
      const uint64_t vo = base + (uint64_t)je * rowb;
      const uint32_t inpage = ((uint32_t)vo & pmask) + lane_b;
      const int2 pp = lds_pg[je];
      const uint64_t pg = (uint64_t)(uint32_t)((inpage >> lp) ? pp.y : pp.x);
      wr[jj] = ld16(a.slab + (pg << lp) + (inpage & pmask));
      if (j >= r) wr[jj] = make_uint4(0, 0, 0, 0);
    }
    // in-register transpose: wk[cc] = the 8 rows' values of column cc
    uint4 wk[8];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const uint32_t r0 = (&wr[0].x)[d], r1 = (&wr[1].x)[d], r2 = (&wr[2].x)[d], r3 = (&wr[3].x)[d];
      const uint32_t r4 = (&wr[4].x)[d], r5 = (&wr[5].x)[d], r6 = (&wr[6].x)[d], r7 = (&wr[7].x)[d];
      wk[2 * d] = make_uint4(__builtin_amdgcn_perm(r1, r0, 0x05040100u), __builtin_amdgcn_perm(r3, r2, 0x05040100u),
                             __builtin_amdgcn_perm(r5, r4, 0x05040100u), __builtin_amdgcn_perm(r7, r6, 0x05040100u));
      wk[2 * d + 1] = make_uint4(__builtin_amdgcn_perm(r1, r0, 0x07060302u), __builtin_amdgcn_perm(r3, r2, 0x07060302u),
                                 __builtin_amdgcn_perm(r5, r4, 0x07060302u), __builtin_amdgcn_perm(r7, r6, 0x07060302u));
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float vf[8];
      const int j8 = jb + 8 * g;
      if (j8 + 8 <= r && (vs & 3) == 0) {
        const float4 va = *reinterpret_cast<const float4*>(vrow[mt] + j8);
        const float4 vb = *reinterpret_cast<const float4*>(vrow[mt] + j8 + 4);
        vf[0] = va.x; vf[1] = va.y; vf[2] = va.z; vf[3] = va.w; vf[4] = vb.x; vf[5] = vb.y; vf[6] = vb.z; vf[7] = vb.w;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) vf[e] = (j8 + e < r) ? vrow[mt][j8 + e] : 0.f;
      }
      uint4 hi, lo;
      split_hi_lo<DT>(vf, hi, lo);
#pragma unroll
      for (int cc = 0; cc < 8; ++cc) {
        acc[mt][cc] = mfma16<DT>(hi, wk[cc], acc[mt][cc]);
        acc[mt][cc] = mfma16<DT>(lo, wk[cc], acc[mt][cc]);
      }
    }
  }
  if (!ok) return;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ti = mt * 16 + g * 4 + i;
      if (ti < it.ntok) {
        const int64_t t = a.perm[sg.tok_start + it.tok0 + ti];
        uint8_t* yp = y + ((uint64_t)t * d_out + n) * EB;
        float yf[8];
        unpack<DT>(ld16(yp), yf);
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) yf[cc] = yf[cc] + sg.scale * acc[mt][cc][i];
        st16(yp, pack<DT>(yf));
      }
    }
}

template <int DT>
__global__ __launch_bounds__(kWave) void k_expand_mfma(const LaunchArgs a, const SlotPtrs p) {
  __shared__ int2 lds_pg[kMaxRank];
  const ItemRec it = a.items[blockIdx.x];
  const SegRec sg = a.segs[it.seg];
  const int q = blockIdx.z;
  const SlotRec sl = a.slots[a.slot0 + q];
  const float* v = (const float*)p.a[q];
  uint8_t* y = (uint8_t*)p.b[q];
  if (it.ntok <= 16) expand_mfma_body<DT, 1>(a, sg, it, sl, v, y, lds_pg);
  else if (it.ntok <= 32) expand_mfma_body<DT, 2>(a, sg, it, sl, v, y, lds_pg);
  else expand_mfma_body<DT, 4>(a, sg, it, sl, v, y, lds_pg);
}

}  // namespace

hipError_t launch_shrink(int dtype, int kind, const LaunchArgs& a, const SlotPtrs& p, int n_slots, hipStream_t st) {
  if (a.n_items <= 0 || n_slots <= 0) return hipSuccess;
  const dim3 grid(a.n_items, 1, n_slots), block(kWave);
  if (kind == 0) {
    if (dtype == 0) hipLaunchKernelGGL(k_shrink_valu<0>, grid, block, 0, st, a, p);
    else if (dtype == 1) hipLaunchKernelGGL(k_shrink_valu<1>, grid, block, 0, st, a, p);
    else hipLaunchKernelGGL(k_shrink_valu<2>, grid, block, 0, st, a, p);
  } else {
    if (dtype == 0) hipLaunchKernelGGL(k_shrink_mfma<0>, grid, block, 0, st, a, p);
    else if (dtype == 1) hipLaunchKernelGGL(k_shrink_mfma<1>, grid, block, 0, st, a, p);
    else return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_expand(int dtype, int kind, const LaunchArgs& a, const SlotPtrs& p, int n_slots, int max_chunks,
                         hipStream_t st) {
  if (a.n_items <= 0 || n_slots <= 0 || max_chunks <= 0) return hipSuccess;
  const dim3 grid(a.n_items, max_chunks, n_slots), block(kWave);
  if (kind == 0) {
    if (dtype == 0) hipLaunchKernelGGL(k_expand_valu<0>, grid, block, 0, st, a, p);
    else if (dtype == 1) hipLaunchKernelGGL(k_expand_valu<1>, grid, block, 0, st, a, p);
    else hipLaunchKernelGGL(k_expand_valu<2>, grid, block, 0, st, a, p);
  } else {
    if (dtype == 0) hipLaunchKernelGGL(k_expand_mfma<0>, grid, block, 0, st, a, p);
    else if (dtype == 1) hipLaunchKernelGGL(k_expand_mfma<1>, grid, block, 0, st, a, p);
    else return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace plora
