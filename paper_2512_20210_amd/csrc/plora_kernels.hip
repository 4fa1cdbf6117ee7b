// gfx950 kernels of the paged multi-LoRA delta (Sec. II-A Eq. 1 over the page pool of Sec. III-C;
// Sec. IV "Memory Manager": kernels that read adapter weights from non-contiguous pages).
//
// Work decomposition.  Items come from the batch translation (tokens grouped by adapter), so every
// weight byte a batch needs is fetched from HBM once per group of tokens, not once per token.  The
// work list of a launch is a sequence of blocks of 4 records, one 256-thread workgroup per block:
// either one matrix-core item that the 4 wavefronts share, or up to 4 vector-ALU items, one per
// wavefront.
//
//   shrink, vector-ALU item : up to 8 rows of A x up to 4 tokens.  Lanes stride along d_in with
//                             16-byte loads, accumulate in fp32 (packed dot products for 16-bit
//                             elements) and finish with one transposing wavefront reduction
//                             of all their sums.
//   shrink, matrix-core item: 32 rows of A x up to 32 tokens, v_mfma_f32_16x16x32 (bf16 / f16), by
//                             4 wavefronts that split d_in; operands staged in LDS, one or two
//                             runs of 64 k-values in flight per wavefront (two kernels).
//   expand, vector-ALU item : all rows of B x 64 lanes x 16 bytes of columns x up to 4 tokens;
//                             no reduction, read-modify-write of y.
//   expand, matrix-core item: all rows of B x 512 columns; up to 16 tokens: every wavefront its own
//                             128 columns, B transposed in registers; 17 to 64 tokens (only in
//                             batches with many large groups, kernel k_expand_panel): B stationary
//                             in LDS, one 16-token tile per wavefront.  v is split into a high and a
//                             low half so that fp32 v loses nothing that matters.
//
// One more launch form uses the vector-ALU records alone: the cooperative kernels for calls too small
// to fill the machine (one record per 256-thread workgroup whose wavefronts split the record's chain
// of loads).  k_scatter_pages moves a blob that
// arrived contiguous in a staging buffer into its pages (staged loads).
//
// Uniform values stay scalar: grid coordinates, slot record, work record (one 32-byte scalar load)
// and wavefront index live in scalar registers, so everything derived from them costs no vector
// registers and no vector memory round trips at the head of a workgroup.
//
// Cache policy: y (read once, written once) goes through streaming loads and stores, and so do the
// weights of items whose rows no other item reads; x, v, page tables and weights that the token
// groups of one adapter share stay ordinary accesses.
//
// Address translation: virtual byte o of an adapter is at slab + pt[o >> log2P] * P + (o & (P-1)).
// A 16-byte vector never straddles a page (all offsets are multiples of 16).  Each item stages the
// page-table entries it can touch in LDS first, so the translation in the inner loop is an LDS
// read, and the reduction order depends on virtual offsets only (evicting and reloading an adapter
// onto other pages gives bit-identical results).
//
// Latency: an item's record is self-contained (one 32-byte read), everything that depends only on
// it (page-table entries, x / v / y rows) is requested at once, and the inner loops over whole
// 64-lane chunks carry no predicates, so that all loads of an iteration are in flight together; a
// ragged last chunk goes through a predicated copy of the same code.
#include "plora_internal.h"
#include <hip/hip_ext.h>

#include <mutex>
#include <type_traits>

namespace plora {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

template <int DT> struct Elt { static constexpr int B = 2, VEC = 8; };
template <> struct Elt<2> { static constexpr int B = 4, VEC = 4; };

__device__ __forceinline__ uint4 ld16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
// Minimum workgroups per CU the compiler must leave room for (bounds the VGPR budget).
constexpr int kWgPerCu = 3;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
// Weights that are read once per batch by this item alone are fetched with streaming loads: they
// then do not push the re-used x / v rows, page-table entries and other items' shared weight rows out
// of the caches.  Weights that a neighbouring item reads again stay ordinary loads.
template <bool NT>
__device__ __forceinline__ uint4 ldw16(const void* p) {
  if constexpr (NT) {
    const u32x4_t q = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(q.x, q.y, q.z, q.w);
  } else {
    return *reinterpret_cast<const uint4*>(p);
  }
}
// A work record at a wavefront-uniform position, fetched as eight whole dwords (one scalar load) and
// taken apart in registers: field-by-field reads of its 16-bit members would be separate vector loads,
// the later ones issued only after the first has been tested.
__device__ __forceinline__ ItemRec load_item(const ItemRec* __restrict__ rec) {
  const uint32_t* w = reinterpret_cast<const uint32_t*>(rec);
  uint32_t d[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) d[i] = w[i];
  ItemRec it;
  it.kind = (int16_t)(d[0] & 0xffffu);
  it.ntok = (int16_t)(d[0] >> 16);
  it.rank = (int16_t)(d[1] & 0xffffu);
  it.j0 = (int16_t)(d[1] >> 16);
  it.scale = __uint_as_float(d[2]);
  it.pt_off = (int32_t)d[3];
#pragma unroll
  for (int i = 0; i < 4; ++i) it.tok[i] = (int32_t)d[4 + i];
  return it;
}
// Index of the wavefront in its workgroup, as a scalar.
__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }
// Record flag (bit 8 of a non-negative kind): no other item of the batch reads this item's weights.
__device__ __forceinline__ int item_kind(const ItemRec& it) { return it.kind < 0 ? -1 : (it.kind & 0xff); }
__device__ __forceinline__ bool item_once(const ItemRec& it) {
  return it.kind >= 0 && (it.kind & kItemOnce) != 0;
}
// Record flag: the adapter lies on consecutive physical pages from page pt_off on, so its page-table
// entries follow from their index and need not be fetched (one dependent trip to memory less at the
// head of the item).
__device__ __forceinline__ bool item_contig(const ItemRec& it) { return it.kind >= 0 && (it.kind & kItemContig) != 0; }
// y is read once and written once per step: streaming (non-temporal) loads and stores, so that its
// lines neither stay in the caches nor wait there to be written back during the next kernel.
__device__ __forceinline__ uint4 ldy16(const void* p) {
  const u32x4_t q = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(q.x, q.y, q.z, q.w);
}
__device__ __forceinline__ void sty16(void* p, uint4 q) {
  u32x4_t t; t.x = q.x; t.y = q.y; t.z = q.z; t.w = q.w;
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t*>(p));
}

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

// fp32 -> element, round to nearest even.  The update of y is written as an explicit fused multiply-add
// (y + scale * sum with one rounding in fp32) and then rounded once to the element type.
// Two fp32 -> one register of two bf16, round to nearest even, in one instruction (v_cvt_pk_bf16_f32).
typedef __bf16 bf16x2_cvt_t __attribute__((ext_vector_type(2)));
typedef float f32x2_cvt_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
  const f32x2_cvt_t f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_cvt_t));
}
// (The value passes through an opaque register first: left to itself the compiler folds this conversion
// into the fused multiply-add that produced the value for some elements - one rounding, straight to fp16 -
// and not for others, differently from one kernel to the next.  Every element is rounded the same way:
// to fp32 by the arithmetic, then once to fp16.)
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
  asm("" : "+v"(f));
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}

template <int DT>
__device__ __forceinline__ uint4 pack(const float* f) {
  uint4 q;
  if constexpr (DT == 2) {
    q.x = __float_as_uint(f[0]); q.y = __float_as_uint(f[1]); q.z = __float_as_uint(f[2]); q.w = __float_as_uint(f[3]);
  } else if constexpr (DT == 1) {
    q.x = f32x2_to_bf16x2(f[0], f[1]); q.y = f32x2_to_bf16x2(f[2], f[3]);
    q.z = f32x2_to_bf16x2(f[4], f[5]); q.w = f32x2_to_bf16x2(f[6], f[7]);
  } else {
    q.x = f32_to_f16_bits(f[0]) | (f32_to_f16_bits(f[1]) << 16);
    q.y = f32_to_f16_bits(f[2]) | (f32_to_f16_bits(f[3]) << 16);
    q.z = f32_to_f16_bits(f[4]) | (f32_to_f16_bits(f[5]) << 16);
    q.w = f32_to_f16_bits(f[6]) | (f32_to_f16_bits(f[7]) << 16);
  }
  return q;
}

// a.lo * b.lo + a.hi * b.hi + c for a pair of 16-bit elements per register, summed in fp32.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
template <int DT>
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
  if constexpr (DT == 1)
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
  else
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, a), __builtin_bit_cast(f16x2_t, b), c, false);
}

// Sums each of a[0 .. N) over the 64 lanes of the wavefront and returns, in lane l, the total of
// a[l >> (6 - log2 N)].  While more than one value is left, a lane keeps the half of them that its
// lane bit M selects and hands the other half to its partner, so N values cost N - 1 + (6 - log2 N)
// exchanges instead of 6 N, and the totals end up spread over the lanes (one store writes them all).
// a[] is used as working space.
template <int N, int M>
__device__ __forceinline__ float wave_sums_step(float* a, int lane) {
  if constexpr (N > 1) {
    const bool up = (lane & M) != 0;
#pragma unroll
    for (int j = 0; j < N / 2; ++j) {
      const float keep = up ? a[j + N / 2] : a[j];
      const float give = up ? a[j] : a[j + N / 2];
      a[j] = keep + __shfl_xor(give, M, 64);
    }
    return wave_sums_step<N / 2, M / 2>(a, lane);
  } else if constexpr (M >= 1) {
    a[0] += __shfl_xor(a[0], M, 64);
    return wave_sums_step<1, M / 2>(a, lane);
  } else {
    return a[0];
  }
}
template <int N>
__device__ __forceinline__ float wave_sums(float* a, int lane) {
  static_assert(N == 4 || N == 8 || N == 16 || N == 32, "a power of two of values, at most one per two lanes");
  return wave_sums_step<N, 32>(a, lane);
}
template <int N>
constexpr int wave_sums_shift() { return N == 32 ? 1 : N == 16 ? 2 : N == 8 ? 3 : 4; }

__device__ __forceinline__ int imin(int a, int b) { return a < b ? a : b; }

// v handed from shrink tasks to expand tasks inside one launch (k_delta_queue) crosses from one XCD's L2
// to another's: there every access to v is a device-scope access (written through to, and read from,
// the level all XCDs share), which costs little for so small an array and needs no cache flushes.
// The separate kernels use ordinary accesses (the kernel boundary orders them).
template <bool COH>
__device__ __forceinline__ void st_v(float* p, float x) {
  if constexpr (COH) __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = x;
}
template <bool COH>
__device__ __forceinline__ float ld_v(const float* p) {
  if constexpr (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return *p;
}

// Orders one wavefront's LDS writes before its later LDS reads (any lane).  LDS instructions of a
// wavefront execute in order, so only the compiler has to be kept from moving them: no s_barrier,
// which lets the wavefronts of a 256-thread workgroup run independent vector-ALU items.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

// ------------------------------------------------------------------------------------------
// shrink, vector-ALU item
// ------------------------------------------------------------------------------------------
template <int DT, int NT, int ROWS, bool TAIL, bool NTW>
__device__ __forceinline__ void shrink_valu_chunk(const LaunchArgs& a, const uint8_t* __restrict__ x, const int64_t* tok,
                                                  const int32_t* lds_pt, uint32_t win0, uint64_t base, uint64_t rowb,
                                                  int nrows, int d_in, int k0, float (*acc)[NT]) {
  constexpr int EB = Elt<DT>::B, VEC = Elt<DT>::VEC;
  const int lp = a.log2_page;
  const uint64_t pmask = ((uint64_t)1 << lp) - 1;
  const int k = k0 + lane_id() * VEC;
  const bool ok = !TAIL || k < d_in;
  const int kk = ok ? k : 0;
  uint4 xq[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) xq[i] = ld16(x + ((uint64_t)tok[i] * d_in + kk) * EB);
  uint4 wq[ROWS];
#pragma unroll
  for (int jj = 0; jj < ROWS; ++jj) {
    const int jr = imin(jj, nrows - 1);
    const uint64_t voff = base + (uint64_t)jr * rowb + (uint64_t)kk * EB;
    const uint64_t pg = (uint64_t)(uint32_t)lds_pt[(uint32_t)(voff >> lp) - win0];
    wq[jj] = ldw16<NTW>(a.slab + (pg << lp) + (voff & pmask));
  }
#pragma unroll
  for (int i = 0; i < NT; ++i)
    if (TAIL && !ok) xq[i] = make_uint4(0, 0, 0, 0);
  if constexpr (DT == 2) {
    float xf[NT][VEC];
#pragma unroll
    for (int i = 0; i < NT; ++i) unpack<DT>(xq[i], xf[i]);
#pragma unroll
    for (int jj = 0; jj < ROWS; ++jj) {
      float wf[VEC];
      unpack<DT>(wq[jj], wf);
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[jj][i] = __builtin_fmaf(wf[e], xf[i][e], acc[jj][i]);
    }
  } else {
    // 16-bit elements: two products per instruction straight from the packed pairs, fp32 sum
#pragma unroll
    for (int jj = 0; jj < ROWS; ++jj)
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        float s = acc[jj][i];
        s = dot2<DT>(wq[jj].x, xq[i].x, s);
        s = dot2<DT>(wq[jj].y, xq[i].y, s);
        s = dot2<DT>(wq[jj].z, xq[i].z, s);
        s = dot2<DT>(wq[jj].w, xq[i].w, s);
        acc[jj][i] = s;
      }
  }
}

template <int DT, int NT, int ROWS, bool NTW, bool COH>
__device__ __forceinline__ void shrink_valu_body(const LaunchArgs& a, const ItemRec it, const SlotRec sl,
                                                 const uint8_t* __restrict__ x, float* __restrict__ v,
                                                 int32_t* lds_pt) {
  constexpr int EB = Elt<DT>::B, VEC = Elt<DT>::VEC;
  const int lane = lane_id();
  const int r = it.rank;
  const int d_in = sl.d_in;
  const int vs = a.v_stride;
  int64_t tok[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) tok[i] = it.tok[i];

  const int nrows = imin(ROWS, r - it.j0);
  const uint64_t rowb = (uint64_t)d_in * EB;
  const uint64_t base = (uint64_t)r * EB * (uint64_t)sl.cum + (uint64_t)it.j0 * rowb;
  const int lp = a.log2_page;
  const uint32_t win0 = (uint32_t)(base >> lp);
  if (r > 0) {
    const uint32_t win_n = (uint32_t)((base + (uint64_t)nrows * rowb - 1) >> lp) - win0 + 1;
    const int32_t* ptg = a.pt + it.pt_off + win0;
    const bool contig = item_contig(it);
    const int32_t page0 = it.pt_off + (int32_t)win0;
    for (uint32_t i = lane; i < win_n; i += kWave) lds_pt[i] = contig ? page0 + (int32_t)i : ptg[i];
  }
  if (it.j0 == 0) {  // the first row block of a token group also clears the unused tail of v
#pragma unroll
    for (int i = 0; i < NT; ++i)
      if (i < it.ntok)
        for (int j = r + lane; j < vs; j += kWave) st_v<COH>(v + tok[i] * vs + j, 0.f);
  }
  if (r == 0) return;
  wave_sync();

  float acc[ROWS][NT];
#pragma unroll
  for (int jj = 0; jj < ROWS; ++jj)
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[jj][i] = 0.f;

  constexpr int CH = kWave * VEC;
  const int full = d_in / CH * CH;
  for (int k0 = 0; k0 < full; k0 += CH)
    shrink_valu_chunk<DT, NT, ROWS, false, NTW>(a, x, tok, lds_pt, win0, base, rowb, nrows, d_in, k0, acc);
  if (full < d_in) shrink_valu_chunk<DT, NT, ROWS, true, NTW>(a, x, tok, lds_pt, win0, base, rowb, nrows, d_in, full, acc);

  // lane 2^sh * (jj * NT + i) ends up with the total of acc[jj][i] and stores it
  constexpr int sh = wave_sums_shift<ROWS * NT>();
  const float total = wave_sums<ROWS * NT>(&acc[0][0], lane);
  const int idx = lane >> sh, jj = idx / NT, i = idx % NT;
  const int ti = i == 1 ? it.tok[1] : i == 2 ? it.tok[2] : i == 3 ? it.tok[3] : it.tok[0];
  if ((lane & ((1 << sh) - 1)) == 0 && jj < nrows && i < it.ntok) st_v<COH>(v + (int64_t)ti * vs + it.j0 + jj, total);
}

template <int DT, bool COH = false>
__device__ __forceinline__ void shrink_valu_item(const LaunchArgs& a, const ItemRec& it, const SlotRec& sl,
                                                 const uint8_t* x, float* v, int32_t* lds_pt) {
  if (item_once(it)) {
    if (it.ntok <= 1) shrink_valu_body<DT, 1, kShrinkRows, true, COH>(a, it, sl, x, v, lds_pt);
    else if (it.ntok == 2) shrink_valu_body<DT, 2, kShrinkRows, true, COH>(a, it, sl, x, v, lds_pt);
    else shrink_valu_body<DT, kValuTok, kShrinkRows, true, COH>(a, it, sl, x, v, lds_pt);
  } else {
    if (it.ntok <= 1) shrink_valu_body<DT, 1, kShrinkRows, false, COH>(a, it, sl, x, v, lds_pt);
    else if (it.ntok == 2) shrink_valu_body<DT, 2, kShrinkRows, false, COH>(a, it, sl, x, v, lds_pt);
    else shrink_valu_body<DT, kValuTok, kShrinkRows, false, COH>(a, it, sl, x, v, lds_pt);
  }
}

// ------------------------------------------------------------------------------------------
// expand, vector-ALU item
// ------------------------------------------------------------------------------------------
// Number of page-table entries of a rank-r adapter.
__device__ __forceinline__ int table_len(const LaunchArgs& a, int r, int eb) {
  const uint64_t S = (uint64_t)r * eb * (uint64_t)a.elems_per_rank;
  return (int)((S + (((uint64_t)1 << a.log2_page) - 1)) >> a.log2_page);
}

// Stages, for every row j of B, the physical pages that hold the first and the last byte of the
// item's piece of that row (a piece is 1024 bytes, a page at least 4096).  No barrier here: the
// caller issues its other loads first and then calls wave_sync().
__device__ __forceinline__ void stage_row_pages(const LaunchArgs& a, const ItemRec& it, int n_pt, uint64_t base,
                                                uint64_t rowb, uint32_t piece_bytes, int2* lds_pg) {
  const int lp = a.log2_page;
  const int32_t* ptg = a.pt + it.pt_off;
  const bool contig = item_contig(it);
  for (int j = lane_id(); j < it.rank; j += kWave) {
    const uint64_t vo = base + (uint64_t)j * rowb;
    const uint32_t q0 = (uint32_t)(vo >> lp);
    const uint32_t q1 = imin((int)((vo + piece_bytes - 1) >> lp), n_pt - 1);
    lds_pg[j] = contig ? make_int2(it.pt_off + (int)q0, it.pt_off + (int)q1) : make_int2(ptg[q0], ptg[q1]);
  }
}

template <int DT, int NT, bool NTW, bool COH>
__device__ __forceinline__ void expand_valu_body(const LaunchArgs& a, const ItemRec it, const SlotRec sl,
                                                 const float* __restrict__ v, uint8_t* __restrict__ y, int2* lds_pg,
                                                 int chunk, float* lds_v = nullptr) {
  constexpr int EB = Elt<DT>::B, VEC = Elt<DT>::VEC;
  const int lane = lane_id();
  const int r = it.rank;
  const int d_out = sl.d_out;
  const int n0w = chunk * (kWave * VEC);
  if (n0w >= d_out || r == 0) return;
  const int n = n0w + lane * VEC;
  const bool ok = n < d_out;
  const uint32_t lane_b = ok ? lane * 16 : 0;
  const int vs = a.v_stride;
  const int lp = a.log2_page;
  const uint32_t pmask = (1u << lp) - 1;  // pages are at most 2^30 bytes
  const uint64_t rowb = (uint64_t)d_out * EB;
  const uint64_t base = (uint64_t)r * EB * ((uint64_t)sl.cum + (uint64_t)sl.d_in) + (uint64_t)n0w * EB;
  stage_row_pages(a, it, table_len(a, r, EB), base, rowb, kWave * 16, lds_pg);

  const float* vrow[NT];
  uint8_t* yp[NT];
  uint4 yq[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    vrow[i] = v + (int64_t)it.tok[i] * vs;
    yp[i] = y + ((uint64_t)it.tok[i] * d_out + (ok ? n : n0w)) * EB;
    yq[i] = ldy16(yp[i]);  // requested now, used after the loop
  }
  if constexpr (COH) {
    // the tokens' rows of v come through device-scope loads (a trip past the L2 each): all of them are
    // requested here at once and parked in LDS (row i at lds_v + i * r), the loop below reads them from there
#pragma unroll
    for (int i = 0; i < NT; ++i)
      for (int j = lane; j < r; j += kWave) lds_v[i * r + j] = ld_v<true>(vrow[i] + j);
  }
  wave_sync();
  float acc[NT][VEC];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[i][e] = 0.f;

  constexpr int U = kExpandU;
  int j = 0;
  for (; j + U <= r; j += U) {
    uint4 wq[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t vo = base + (uint64_t)(j + u) * rowb;
      const uint32_t inpage = ((uint32_t)vo & pmask) + lane_b;
      const int2 pp = lds_pg[j + u];
      const uint64_t pg = (uint64_t)(uint32_t)((inpage >> lp) ? pp.y : pp.x);
      wq[u] = ldw16<NTW>(a.slab + (pg << lp) + (inpage & pmask));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float wf[VEC];
      unpack<DT>(wq[u], wf);
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        const float vj = COH ? lds_v[i * r + j + u] : vrow[i][j + u];
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
    unpack<DT>(ldw16<NTW>(a.slab + (pg << lp) + (inpage & pmask)), wf);
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const float vj = COH ? lds_v[i * r + j] : vrow[i][j];
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[i][e] = __builtin_fmaf(vj, wf[e], acc[i][e]);
    }
  }
  if (!ok) return;
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    if (i < it.ntok) {
      float yf[VEC];
      unpack<DT>(yq[i], yf);
#pragma unroll
      for (int e = 0; e < VEC; ++e) yf[e] = __builtin_fmaf(it.scale, acc[i][e], yf[e]);
      sty16(yp[i], pack<DT>(yf));
    }
  }
}

template <int DT, bool COH = false>
__device__ __forceinline__ void expand_valu_item(const LaunchArgs& a, const ItemRec& it, const SlotRec& sl,
                                                 const float* v, uint8_t* y, int2* lds_pg, int chunk, float* lds_v = nullptr) {
  if (item_once(it)) {
    if (it.ntok <= 1) expand_valu_body<DT, 1, true, COH>(a, it, sl, v, y, lds_pg, chunk, lds_v);
    else if (it.ntok == 2) expand_valu_body<DT, 2, true, COH>(a, it, sl, v, y, lds_pg, chunk, lds_v);
    else expand_valu_body<DT, kValuTok, true, COH>(a, it, sl, v, y, lds_pg, chunk, lds_v);
  } else {
    if (it.ntok <= 1) expand_valu_body<DT, 1, false, COH>(a, it, sl, v, y, lds_pg, chunk, lds_v);
    else if (it.ntok == 2) expand_valu_body<DT, 2, false, COH>(a, it, sl, v, y, lds_pg, chunk, lds_v);
    else expand_valu_body<DT, kValuTok, false, COH>(a, it, sl, v, y, lds_pg, chunk, lds_v);
  }
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

// shrink, matrix-core item: D[token, row] += X[token, k] * A[row, k] for 32 tokens x 32 rows, by a
// workgroup of 4 wavefronts that split the contraction (each takes every 4th run of 64 k-values'
// worth of work as one contiguous quarter of d_in) and add their partial sums in a fixed order at
// the end.  MFMA operands want "one row per lane", which as a global load would touch 16 cache
// lines per instruction; instead each wavefront fetches its 32 x 128-byte tiles of A and x with
// row-contiguous 16-byte loads (8 lanes per row), parks them in its own LDS region and reads the
// operands back in MFMA layout.  The next tiles are requested before the current ones are
// multiplied.
#define SM_SYNC() __syncthreads()
constexpr int kSmTok = 32, kSmRows = 32, kSmPitch = 144;  // 128 data bytes + 16 pad per LDS row
static_assert(kMfmaTokS == kSmTok && kMfmaRows == kSmRows, "host work items must match the kernel's tile");

template <int DT, bool NTW, int DEPTH, bool COH = false>
__device__ __forceinline__ void shrink_mfma4_body(const LaunchArgs& a, const ItemRec it, const SlotRec sl,
                                                  const uint8_t* __restrict__ x, float* __restrict__ v,
                                                  uint8_t (*tile)[2][kSmRows * kSmPitch], int32_t* lds_pt) {
  constexpr int EB = 2;

  const int tid = threadIdx.x, wave = wave_id(), lane = tid & 63;
  const int g = lane >> 4, c = lane & 15;   // MFMA coordinates
  const int lr = lane >> 3, lp8 = lane & 7; // staging coordinates: row within a group of 8, 16-byte piece
  const int r = it.rank, d_in = sl.d_in, vs = a.v_stride, lp = a.log2_page;
  const uint64_t pmask = ((uint64_t)1 << lp) - 1;
  const int32_t* perm = a.perm + it.tok[0];

  const int nrows = imin(kSmRows, r - it.j0);
  const uint64_t rowb = (uint64_t)d_in * EB;
  const uint64_t base = (uint64_t)r * EB * (uint64_t)sl.cum + (uint64_t)it.j0 * rowb;
  const uint32_t win0 = (uint32_t)(base >> lp);
  const uint32_t win_n = (uint32_t)((base + (uint64_t)nrows * rowb - 1) >> lp) - win0 + 1;
  const int32_t* ptg = a.pt + it.pt_off + win0;
  {
    const bool contig = item_contig(it);
    const int32_t page0 = it.pt_off + (int32_t)win0;
    for (uint32_t i = tid; i < win_n; i += 256) lds_pt[i] = contig ? page0 + (int32_t)i : ptg[i];
  }

  uint64_t wrow[4];          // virtual offsets of the 4 rows of A this lane stages
  const uint8_t* xrow[4];    // and of its 4 token rows
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    wrow[i] = base + (uint64_t)imin(lr + 8 * i, nrows - 1) * rowb;
    xrow[i] = x + (uint64_t)perm[imin(lr + 8 * i, it.ntok - 1)] * rowb;
  }
  if (it.j0 == 0) {  // clear v[t, r .. v_stride) for the item's tokens
    for (int i = wave; i < it.ntok; i += 4) {
      const int64_t t = perm[i];
      for (int j = r + lane; j < vs; j += kWave) st_v<COH>(v + t * vs + j, 0.f);
    }
  }
  __syncthreads();

  // this wavefront's quarter of the contraction, in runs of 64 k-values
  const int nrun = (d_in + 63) >> 6;
  const int per = (nrun + 3) >> 2;
  const int mine = (nrun - wave + 3) >> 2;  // runs wave, wave + 4, ...
#define SM_RUN(i) ((i) * 4 + wave)

  f32x4 acc[2][2];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

  uint8_t* tw = tile[wave][0];
  uint8_t* tx = tile[wave][1];
  // Loads of a run of 64 k-values into registers (always issued: callers clamp the run, so that the
  // compiler can count the loads in flight), their way into LDS, and the products from there.
  auto fetch = [&](int run, uint4 (&wq)[4], uint4 (&xq)[4]) -> bool {
    const int k = run * 64 + lp8 * 8;
    const bool ok = k < d_in;  // past a ragged end the lane reads k = 0 and stages zeros
    const uint64_t kb = (uint64_t)(ok ? k : 0) * EB;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint64_t vo = wrow[i] + kb;
      const uint64_t pg = (uint64_t)(uint32_t)lds_pt[(uint32_t)(vo >> lp) - win0];
      wq[i] = ldw16<NTW>(a.slab + (pg << lp) + (vo & pmask));
      xq[i] = ld16(xrow[i] + kb);
    }
    return ok;
  };
  // (selects, not a branch around stores of zeros: a branch that touches registers with loads in
  // flight makes the compiler wait for every load there, also the other run's)
  auto keep_if = [](const uint4 q, bool ok) { return make_uint4(ok ? q.x : 0u, ok ? q.y : 0u, ok ? q.z : 0u, ok ? q.w : 0u); };
  auto stage = [&](const uint4 (&wq)[4], const uint4 (&xq)[4], bool ok) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *reinterpret_cast<uint4*>(tw + (lr + 8 * i) * kSmPitch + lp8 * 16) = keep_if(wq[i], ok);
      *reinterpret_cast<uint4*>(tx + (lr + 8 * i) * kSmPitch + lp8 * 16) = keep_if(xq[i], ok);
    }
  };
  auto multiply = [&]() {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint4 wo[2], xo[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        wo[t] = *reinterpret_cast<const uint4*>(tw + (16 * t + c) * kSmPitch + h * 64 + g * 16);
        xo[t] = *reinterpret_cast<const uint4*>(tx + (16 * t + c) * kSmPitch + h * 64 + g * 16);
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = mfma16<DT>(xo[mt], wo[nt], acc[mt][nt]);
    }
  };
  if constexpr (DEPTH == 2) {
    // two runs in flight: while one is multiplied, the next two are on their way
    uint4 wq0[4], xq0[4], wq1[4], xq1[4];
    bool ok0 = false, ok1 = false;
    if (mine > 0) {
      ok0 = fetch(SM_RUN(0), wq0, xq0);
      __builtin_amdgcn_sched_barrier(0);  // first run's loads first: its wait then leaves the second run's in flight
      ok1 = fetch(SM_RUN(imin(1, mine - 1)), wq1, xq1);  // (unconditional, so that the loop sees one state of loads in flight)
      __builtin_amdgcn_sched_barrier(0);
    }
    int i = 0;
    for (; i + 3 < mine; i += 2) {  // whole pairs with two more runs to request: every trip leaves the same loads in flight
      stage(wq0, xq0, ok0);
      SM_SYNC();
      ok0 = fetch(SM_RUN(i + 2), wq0, xq0);
      multiply();
      SM_SYNC();
      __builtin_amdgcn_sched_barrier(0);  // keeps the other pair's work (and with it its wait) below this point
      stage(wq1, xq1, ok1);
      SM_SYNC();
      ok1 = fetch(SM_RUN(i + 3), wq1, xq1);
      multiply();
      SM_SYNC();
      __builtin_amdgcn_sched_barrier(0);
    }
    const int rem = mine - i;  // 0 (no run at all) .. 3 left, the first two of them requested
    if (rem >= 1) {
      stage(wq0, xq0, ok0);
      SM_SYNC();
      if (rem == 3) ok0 = fetch(SM_RUN(i + 2), wq0, xq0);
      multiply();
      SM_SYNC();
    }
    if (rem >= 2) {
      stage(wq1, xq1, ok1);
      SM_SYNC();
      multiply();
      SM_SYNC();
    }
    if (rem == 3) {
      stage(wq0, xq0, ok0);
      SM_SYNC();
      multiply();
      SM_SYNC();
    }
  } else {
    uint4 wq[4], xq[4];
    bool ok = false;
    if (mine > 0) ok = fetch(SM_RUN(0), wq, xq);
    for (int i = 0; i < mine; ++i) {
      stage(wq, xq, ok);
      SM_SYNC();
      if (i + 1 < mine) ok = fetch(SM_RUN(i + 1), wq, xq);  // in flight while this run is multiplied
      multiply();
      SM_SYNC();
    }
  }
  // every wavefront passes 2 * per barriers: those with fewer runs (or none) catch up here
  for (int run = mine; run < per; ++run) { __syncthreads(); __syncthreads(); }
#undef SM_RUN
#undef SM_SYNC

  // add the 4 partial sums in wavefront order: thread (w, lane) finishes tile (mt, nt) = (w >> 1, w & 1)
  float* red = reinterpret_cast<float*>(&tile[0][0][0]);  // 4 x 64 x 16 floats = 16 KiB, tiles are free now
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
      *reinterpret_cast<f32x4*>(red + ((wave * 64 + lane) * 4 + mt * 2 + nt) * 4) = acc[mt][nt];
  __syncthreads();
  const int mt = wave >> 1, nt = wave & 1;
  f32x4 sum = *reinterpret_cast<const f32x4*>(red + ((0 * 64 + lane) * 4 + wave) * 4);
#pragma unroll
  for (int w = 1; w < 4; ++w) {
    const f32x4 t = *reinterpret_cast<const f32x4*>(red + ((w * 64 + lane) * 4 + wave) * 4);
    sum[0] += t[0]; sum[1] += t[1]; sum[2] += t[2]; sum[3] += t[3];
  }
  // lane (g, c) of a result tile: row 16 nt + c of A, tokens 16 mt + 4 g .. + 3
  if (16 * nt + c < nrows) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ti = 16 * mt + 4 * g + i;
      if (ti < it.ntok) st_v<COH>(v + (int64_t)perm[ti] * vs + it.j0 + 16 * nt + c, sum[i]);
    }
  }
}

// Splits 8 fp32 values into a high and a low 16-bit part: hi = round(v), lo = round(v - hi).
template <int DT>
__device__ __forceinline__ void split_hi_lo(const float* f, uint4& hi, uint4& lo) {
  uint32_t hp[4], lp[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    if constexpr (DT == 1) {
      hp[e] = f32x2_to_bf16x2(f[2 * e], f[2 * e + 1]);
      lp[e] = f32x2_to_bf16x2(f[2 * e] - __uint_as_float(hp[e] << 16), f[2 * e + 1] - __uint_as_float(hp[e] & 0xffff0000u));
    } else {
      const uint32_t h0 = f32_to_f16_bits(f[2 * e]), h1 = f32_to_f16_bits(f[2 * e + 1]);
      hp[e] = h0 | (h1 << 16);
      lp[e] = f32_to_f16_bits(f[2 * e] - half_bits_to_float(h0)) | (f32_to_f16_bits(f[2 * e + 1] - half_bits_to_float(h1)) << 16);
    }
  }
  hi = make_uint4(hp[0], hp[1], hp[2], hp[3]);
  lo = make_uint4(lp[0], lp[1], lp[2], lp[3]);
}

// fp16 only: fp32 v does not fit fp16's exponent range in general (|v| > 65504 would become inf, tiny
// rows would land among the subnormals), so every token's row of v goes into the matrix cores
// multiplied by a power of two that brings its largest magnitude into [1, 2), and the row's sums are
// multiplied back in fp32 afterwards; both multiplications are exact.  Lane (g, c) looks at the
// values of operand row c it will load later (8 of every 32, from 8 g) and the four lane groups
// combine.  Returns the biased exponent e of the row's largest magnitude, clamped to [1, 253]:
// scale = 2^(127 - e), inverse = 2^(e - 127).  bf16 shares fp32's exponent range and needs none of this.
template <bool COH>
__device__ __forceinline__ uint32_t row_exponent(const float* vrow, int r, int g) {
  float m = 0.f;
  for (int j = 8 * g; j < r; j += 32)
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (j + e < r) m = fmaxf(m, fabsf(ld_v<COH>(vrow + j + e)));
  m = fmaxf(m, __shfl_xor(m, 16, 64));
  m = fmaxf(m, __shfl_xor(m, 32, 64));
  uint32_t ex = (__float_as_uint(m) >> 23) & 0xffu;
  if (ex == 0 || ex == 255) ex = 127;  // zero / subnormal rows, and rows with inf or NaN: unscaled
  return ex > 253u ? 253u : ex;
}
__device__ __forceinline__ float exp_scale(uint32_t ex) { return __uint_as_float((254u - ex) << 23); }
__device__ __forceinline__ float exp_inverse(uint32_t ex) { return __uint_as_float(ex << 23); }

// One K-step (32 rows of B) of the matrix-core expand for one 128-column pass.
template <int DT, int MT, bool TAIL, bool NTW, bool COH>
__device__ __forceinline__ void expand_mfma_kstep(const LaunchArgs& a, const int2* lds_pg, const float* const* vrow,
                                                  uint64_t base, uint64_t rowb, uint32_t lane_b, int r, int jb,
                                                  const float* rs, f32x4 (*acc)[8]) {
  const int g = lane_id() >> 4;
  const int lp = a.log2_page;
  const uint32_t pmask = (1u << lp) - 1;
  const int vs = a.v_stride;
  const int j8 = jb + 8 * g;
  float vf[MT][8];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if (COH) {
#pragma unroll
      for (int e = 0; e < 8; ++e) vf[mt][e] = (!TAIL || j8 + e < r) ? ld_v<COH>(vrow[mt] + j8 + e) : 0.f;
    } else if ((!TAIL || j8 + 8 <= r) && (vs & 3) == 0) {
      const float4 va = *reinterpret_cast<const float4*>(vrow[mt] + j8);
      const float4 vb = *reinterpret_cast<const float4*>(vrow[mt] + j8 + 4);
      vf[mt][0] = va.x; vf[mt][1] = va.y; vf[mt][2] = va.z; vf[mt][3] = va.w;
      vf[mt][4] = vb.x; vf[mt][5] = vb.y; vf[mt][6] = vb.z; vf[mt][7] = vb.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) vf[mt][e] = (j8 + e < r) ? vrow[mt][j8 + e] : 0.f;
    }
  }
  uint4 wr[8];
  if (!TAIL || j8 < r) {  // lanes whose 8 rows all lie past the rank request nothing (r <= 24: whole lane groups)
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      const int j = j8 + jj;
      const int je = TAIL ? imin(j, r - 1) : j;
      const uint64_t vo = base + (uint64_t)je * rowb;
      const uint32_t inpage = ((uint32_t)vo & pmask) + lane_b;
      const int2 pp = lds_pg[je];
      const uint64_t pg = (uint64_t)(uint32_t)((inpage >> lp) ? pp.y : pp.x);
      wr[jj] = ldw16<NTW>(a.slab + (pg << lp) + (inpage & pmask));
    }
  }
  if (TAIL) {
#pragma unroll
    for (int jj = 0; jj < 8; ++jj)
      if (j8 + jj >= r) wr[jj] = make_uint4(0, 0, 0, 0);
  }
  uint4 vhi[MT], vlo[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if constexpr (DT == 0) {
#pragma unroll
      for (int e = 0; e < 8; ++e) vf[mt][e] *= rs[mt];
    }
    split_hi_lo<DT>(vf[mt], vhi[mt], vlo[mt]);
  }
  // in-register transpose, two column offsets at a time: the 8 rows' values of one column
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t r0 = (&wr[0].x)[d], r1 = (&wr[1].x)[d], r2 = (&wr[2].x)[d], r3 = (&wr[3].x)[d];
    const uint32_t r4 = (&wr[4].x)[d], r5 = (&wr[5].x)[d], r6 = (&wr[6].x)[d], r7 = (&wr[7].x)[d];
    const uint4 wlo = make_uint4(__builtin_amdgcn_perm(r1, r0, 0x05040100u), __builtin_amdgcn_perm(r3, r2, 0x05040100u),
                                 __builtin_amdgcn_perm(r5, r4, 0x05040100u), __builtin_amdgcn_perm(r7, r6, 0x05040100u));
    const uint4 whi = make_uint4(__builtin_amdgcn_perm(r1, r0, 0x07060302u), __builtin_amdgcn_perm(r3, r2, 0x07060302u),
                                 __builtin_amdgcn_perm(r5, r4, 0x07060302u), __builtin_amdgcn_perm(r7, r6, 0x07060302u));
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      acc[mt][2 * d] = mfma16<DT>(vhi[mt], wlo, acc[mt][2 * d]);
      acc[mt][2 * d] = mfma16<DT>(vlo[mt], wlo, acc[mt][2 * d]);
      acc[mt][2 * d + 1] = mfma16<DT>(vhi[mt], whi, acc[mt][2 * d + 1]);
      acc[mt][2 * d + 1] = mfma16<DT>(vlo[mt], whi, acc[mt][2 * d + 1]);
    }
  }
}

// Column-split form for items of at most 32 tokens: every wavefront takes its own 128 columns of the
// 512-column chunk and all MT token tiles, loads its tile of B straight into registers (each tile is
// used by one wavefront only, so nothing is shared and there is no barrier after the page staging),
// transposes and multiplies.
template <int DT, int MT, bool NTW, bool COH>
__device__ __forceinline__ void expand_mfma_cols_body(const LaunchArgs& a, const ItemRec it, const SlotRec sl,
                                                      const float* __restrict__ v, uint8_t* __restrict__ y,
                                                      const int2* lds_pg, int chunk, uint64_t base, uint64_t rowb) {
  constexpr int EB = 2;
  const int wave = wave_id(), lane = lane_id();
  const int g = lane >> 4, c = lane & 15;
  const int r = it.rank, d_out = sl.d_out, vs = a.v_stride;
  const int n0 = chunk * 512 + wave * kMfmaCols;
  if (n0 >= d_out) return;
  const int n = n0 + 8 * c;
  const bool ok = n < d_out;
  const uint32_t lane_b = ok ? (uint32_t)(wave * kMfmaCols * EB + c * 16) : 0;
  const int32_t* perm = a.perm + it.tok[0];
  const float* vrow[MT];
  int64_t trow[MT][4];
  float rs[MT], inv[MT][4];  // fp16: power-of-two scale of operand row c, inverse for this lane's result rows
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int tc = perm[imin(mt * 16 + c, it.ntok - 1)];
    vrow[mt] = v + (int64_t)tc * vs;
#pragma unroll
    for (int i = 0; i < 4; ++i) trow[mt][i] = __shfl(tc, g * 4 + i, 64);
    rs[mt] = 1.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) inv[mt][i] = 1.f;
    if constexpr (DT == 0) {
      const uint32_t ex = row_exponent<COH>(vrow[mt], r, g);
      rs[mt] = exp_scale(ex);
#pragma unroll
      for (int i = 0; i < 4; ++i) inv[mt][i] = exp_inverse((uint32_t)__shfl((int)ex, g * 4 + i, 64));
    }
  }
  f32x4 acc[MT][8];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) acc[mt][cc] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int nn = ok ? n : n0;
  uint4 yq[MT][4];  // requested now, used after the loop
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 4; ++i) yq[mt][i] = ldy16(y + ((uint64_t)trow[mt][i] * d_out + nn) * EB);
  int jb = 0;
  for (; jb + 32 <= r; jb += 32) expand_mfma_kstep<DT, MT, false, NTW, COH>(a, lds_pg, vrow, base, rowb, lane_b, r, jb, rs, acc);
  if (jb < r) expand_mfma_kstep<DT, MT, true, NTW, COH>(a, lds_pg, vrow, base, rowb, lane_b, r, jb, rs, acc);
  if (!ok) return;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (mt * 16 + g * 4 + i < it.ntok) {
        float yf[8];
        unpack<DT>(yq[mt][i], yf);
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) {
          if constexpr (DT == 0) yf[cc] = __builtin_fmaf(it.scale, inv[mt][i] * acc[mt][cc][i], yf[cc]);
          else yf[cc] = __builtin_fmaf(it.scale, acc[mt][cc][i], yf[cc]);
        }
        sty16(y + ((uint64_t)trow[mt][i] * d_out + n) * EB, pack<DT>(yf));
      }
    }
  }
}

// Page pairs of every row's 1 KiB piece of the 512-column chunk, staged in LDS by all 256 threads
// (a piece may straddle one page boundary).
__device__ __forceinline__ void expand_stage_pages(const LaunchArgs& a, const ItemRec& it, int2* lds_pg, uint64_t base,
                                                   uint64_t rowb, int EB) {
  const int r = it.rank, lp = a.log2_page;
  const int n_pt = table_len(a, r, EB);
  const int32_t* ptg = a.pt + it.pt_off;
  const bool contig = item_contig(it);
  for (int j = threadIdx.x; j < r; j += 256) {
    const uint64_t vo = base + (uint64_t)j * rowb;
    const uint32_t q0 = (uint32_t)(vo >> lp);
    const uint32_t q1 = imin((int)((vo + 1023) >> lp), n_pt - 1);
    lds_pg[j] = contig ? make_int2(it.pt_off + (int)q0, it.pt_off + (int)q1) : make_int2(ptg[q0], ptg[q1]);
  }
}

// expand, matrix-core item of at most kMfmaTokCols tokens, by a workgroup of 4 wavefronts: stage the
// page pairs, then every wavefront takes its 128 columns (column-split form above).
template <int DT, bool COH = false>
__device__ __forceinline__ void expand_mfma_cols_item(const LaunchArgs& a, const ItemRec it, const SlotRec sl,
                                                      const float* __restrict__ v, uint8_t* __restrict__ y,
                                                      int2* lds_pg, int chunk) {
  constexpr int EB = 2;
  const int n0i = chunk * 512;
  if (n0i >= sl.d_out) return;  // uniform over the workgroup
  const uint64_t rowb = (uint64_t)sl.d_out * EB;
  const uint64_t base = (uint64_t)it.rank * EB * ((uint64_t)sl.cum + (uint64_t)sl.d_in) + (uint64_t)n0i * EB;
  expand_stage_pages(a, it, lds_pg, base, rowb, EB);
  __syncthreads();
  if (item_once(it)) expand_mfma_cols_body<DT, 1, true, COH>(a, it, sl, v, y, lds_pg, chunk, base, rowb);
  else expand_mfma_cols_body<DT, 1, false, COH>(a, it, sl, v, y, lds_pg, chunk, base, rowb);
}

// expand, matrix-core item of 17 .. 64 tokens (batches with many large groups: prefill):
// D[token, col] += V[token, j] * B[j, col] for up to 64 tokens x 512 columns, by a workgroup of 4
// wavefronts with B held stationary in LDS.  The 512 columns are done as two halves of 256; rows of
// B in panels of 64.  For a panel the 4 wavefronts each fetch one 32-row x 128-column tile of B
// (8 loads of 16 bytes per lane: lane (g, c) gets the 8x8 block rows 8 g .. 8 g + 7 x columns
// 8 c .. 8 c + 7), transpose it in registers into eight 8-value K-vectors (one per column offset cc)
// and park them in LDS in MFMA operand order.  Then wavefront w multiplies token tile w (16 tokens)
// against all four tiles: MFMA cc of a tile yields the real columns 8 c + cc, so a lane ends with 8
// consecutive columns of y for each of its 4 token rows and updates y with 16-byte
// read-modify-writes.  B is read once per 64 tokens; v goes in as hi + lo 16-bit halves (two MFMAs)
// so that fp32 v loses nothing that matters.  Order of the requests in a panel: the tile of B; once it
// has arrived and is on its way into LDS, the rows of v (they overlap the transposition and the
// barrier; asked for together with B they would cost 16 registers at the point where most are live);
// and in a half's last panel, right after the barrier, the half's rows of y, which then travel while
// the products are formed.  (Requesting the rows of y before B is staged costs more in registers,
// hence resident workgroups, than the overlap returns; strips of 128 columns per workgroup instead of
// 512 are slower too: v is then re-read four times as often.)
// HALF: the workgroup does one of the two halves only (half_sel), the other one belongs to another
// workgroup: twice the workgroups, each with half the accumulators (4 instead of 3 fit a CU) and
// half as long a chain, at the price of reading v twice as often - for launches that are too short
// to hide a workgroup's chain behind others.
static_assert(kMfmaTokE == 64, "host work items must match the kernel's tiles");

template <int DT, bool HALF>
__device__ __forceinline__ void expand_panel_item(const LaunchArgs& a, const ItemRec it, const SlotRec sl,
                                                  const float* __restrict__ v, uint8_t* __restrict__ y,
                                                  uint4 (*op)[8][kWave], int2* lds_pg, int chunk, int half_sel) {
  constexpr int EB = 2;
  const int tid = threadIdx.x, wave = wave_id(), lane = tid & 63;
  const int g = lane >> 4, c = lane & 15;
  const int r = it.rank, d_out = sl.d_out, vs = a.v_stride, lp = a.log2_page;
  const int n0i = chunk * 512;
  if (n0i >= d_out) return;  // uniform over the workgroup
  const uint32_t pmask = (1u << lp) - 1;
  const uint64_t rowb = (uint64_t)d_out * EB;
  const uint64_t base = (uint64_t)r * EB * ((uint64_t)sl.cum + (uint64_t)sl.d_in) + (uint64_t)n0i * EB;
  expand_stage_pages(a, it, lds_pg, base, rowb, EB);
  const int32_t* perm = a.perm + it.tok[0];
  const bool has_tok = wave * 16 < it.ntok;            // this wavefront owns token tile `wave`
  const int tc = perm[imin(wave * 16 + c, it.ntok - 1)];  // token of operand row c
  const float* vrow = v + (int64_t)tc * vs;
  int64_t trow[4];                                       // tokens of the result rows this lane holds
#pragma unroll
  for (int i = 0; i < 4; ++i) trow[i] = __shfl(tc, g * 4 + i, 64);
  float rs = 1.f, inv[4] = {1.f, 1.f, 1.f, 1.f};         // fp16: scale of operand row c, inverses of the result rows
  if constexpr (DT == 0) {
    const uint32_t ex = row_exponent<false>(vrow, r, g);
    rs = exp_scale(ex);
#pragma unroll
    for (int i = 0; i < 4; ++i) inv[i] = exp_inverse((uint32_t)__shfl((int)ex, g * 4 + i, 64));
  }
  __syncthreads();

  const int ks_w = wave >> 1, ct_w = wave & 1;  // the tile this wavefront stages: K-step in panel, column tile
  for (int half = HALF ? half_sel : 0; half < (HALF ? half_sel + 1 : 2); ++half) {
    const int nh0 = n0i + half * 256;
    if (nh0 >= d_out) break;
    uint4 yq[2][4];
    f32x4 acc[2][8];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int cc = 0; cc < 8; ++cc) acc[ct][cc] = f32x4{0.f, 0.f, 0.f, 0.f};

    // one panel of 64 rows of B; kLast: the half's last one, which also requests the rows of y
    auto do_panel = [&](const int j0, auto last_tag) {
      constexpr bool kLast = decltype(last_tag)::value;
      float vf[2][8];  // this wavefront's rows of v for the panel
      {  // stage tile (ks_w, ct_w) of this panel
        const int ncol = nh0 + ct_w * 128 + 8 * c;
        const bool okc = ncol < d_out;
        const uint32_t lane_b = okc ? (uint32_t)((half * 256 + ct_w * 128) * EB + c * 16) : 0;
        const int j8 = j0 + ks_w * 32 + 8 * g;
        uint4 wr[8];
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
          const int je = imin(j8 + jj, r - 1);
          const uint64_t vo = base + (uint64_t)je * rowb;
          const uint32_t inpage = ((uint32_t)vo & pmask) + lane_b;
          const int2 pp = lds_pg[je];
          const uint64_t pg = (uint64_t)(uint32_t)((inpage >> lp) ? pp.y : pp.x);
          wr[jj] = ldw16<false>(a.slab + (pg << lp) + (inpage & pmask));
        }
#pragma unroll
        for (int jj = 0; jj < 8; ++jj)
          if (j8 + jj >= r || !okc) wr[jj] = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const uint32_t r0 = (&wr[0].x)[d], r1 = (&wr[1].x)[d], r2 = (&wr[2].x)[d], r3 = (&wr[3].x)[d];
          const uint32_t r4 = (&wr[4].x)[d], r5 = (&wr[5].x)[d], r6 = (&wr[6].x)[d], r7 = (&wr[7].x)[d];
          op[wave][2 * d][lane] =
              make_uint4(__builtin_amdgcn_perm(r1, r0, 0x05040100u), __builtin_amdgcn_perm(r3, r2, 0x05040100u),
                         __builtin_amdgcn_perm(r5, r4, 0x05040100u), __builtin_amdgcn_perm(r7, r6, 0x05040100u));
          op[wave][2 * d + 1][lane] =
              make_uint4(__builtin_amdgcn_perm(r1, r0, 0x07060302u), __builtin_amdgcn_perm(r3, r2, 0x07060302u),
                         __builtin_amdgcn_perm(r5, r4, 0x07060302u), __builtin_amdgcn_perm(r7, r6, 0x07060302u));
        }
        __builtin_amdgcn_sched_barrier(0);  // the rows of v only now: the registers of the tile are free again
        if (has_tok) {
#pragma unroll
          for (int ks = 0; ks < 2; ++ks) {
            const int jv = j0 + ks * 32 + 8 * g;
            if (jv + 8 <= r && (vs & 3) == 0) {
              const float4 va = *reinterpret_cast<const float4*>(vrow + jv);
              const float4 vb = *reinterpret_cast<const float4*>(vrow + jv + 4);
              vf[ks][0] = va.x; vf[ks][1] = va.y; vf[ks][2] = va.z; vf[ks][3] = va.w;
              vf[ks][4] = vb.x; vf[ks][5] = vb.y; vf[ks][6] = vb.z; vf[ks][7] = vb.w;
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e) vf[ks][e] = (jv + e < r) ? vrow[jv + e] : 0.f;
            }
          }
        }
      }
      __syncthreads();
      if (kLast && has_tok) {
        // both column tiles' rows of y in one trip, under way while the products are formed
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
          const int n = imin(nh0 + ct * 128 + 8 * c, d_out - 8);
#pragma unroll
          for (int i = 0; i < 4; ++i) yq[ct][i] = ldy16(y + ((uint64_t)trow[i] * d_out + n) * EB);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (has_tok) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          if (j0 + ks * 32 < r) {  // uniform
            uint4 vhi, vlo;
            if constexpr (DT == 0) {
#pragma unroll
              for (int e = 0; e < 8; ++e) vf[ks][e] *= rs;
            }
            split_hi_lo<DT>(vf[ks], vhi, vlo);
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
              for (int cc = 0; cc < 8; ++cc) {
                const uint4 w = op[ks * 2 + ct][cc][lane];
                acc[ct][cc] = mfma16<DT>(vhi, w, acc[ct][cc]);
                acc[ct][cc] = mfma16<DT>(vlo, w, acc[ct][cc]);
              }
          }
        }
      }
      __syncthreads();
    };
    {
      int j0 = 0;
      for (; j0 + 64 < r; j0 += 64) do_panel(j0, std::false_type{});
      do_panel(j0, std::true_type{});
    }
    if (has_tok) {
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) {
        const int n = nh0 + ct * 128 + 8 * c;
        if (n < d_out) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if (wave * 16 + g * 4 + i < it.ntok) {
              float yf[8];
              unpack<DT>(yq[ct][i], yf);
#pragma unroll
              for (int cc = 0; cc < 8; ++cc) {
                if constexpr (DT == 0) yf[cc] = __builtin_fmaf(it.scale, inv[i] * acc[ct][cc][i], yf[cc]);
                else yf[cc] = __builtin_fmaf(it.scale, acc[ct][cc][i], yf[cc]);
              }
              sty16(y + ((uint64_t)trow[i] * d_out + n) * EB, pack<DT>(yf));
            }
          }
        }
      }
    }
  }
}

// Shrink: workgroups of 4 wavefronts.  The work list is a sequence of blocks of 4 records: either
// one matrix-core item (first record, the other three are padding) that the 4 wavefronts share,
// or up to 4 independent vector-ALU items, one per wavefront.  The matrix-core blocks come first in
// the list, so their long dependent chains start first and the short items fill the machine around
// and after them in the same launch.
// DEPTH: runs of 64 k-values that a matrix-core item keeps in flight (1 or 2).
template <int DT, int DEPTH>
__global__ __launch_bounds__(256, kWgPerCu) void k_shrink(const LaunchArgs a, const SlotPtrs p) {
  __shared__ __align__(16) uint8_t tile[4][2][kSmRows * kSmPitch];  // [wavefront][A | x]
  __shared__ int32_t lds_pt[kPtWindow];
  const int blk = a.slot_fastest ? blockIdx.z : blockIdx.x;
  const int q = a.slot_fastest ? blockIdx.x : blockIdx.z;
  const SlotRec sl = a.slots[p.slot[q]];
  const uint8_t* x = (const uint8_t*)p.a[q];
  float* v = (float*)p.b[q];
  const ItemRec first = load_item(a.items + (4 * blk));
  if constexpr (DT != 2) {
    if (item_kind(first) == 1) {
      if (item_once(first)) shrink_mfma4_body<DT, true, DEPTH>(a, first, sl, x, v, tile, lds_pt);
      else shrink_mfma4_body<DT, false, DEPTH>(a, first, sl, x, v, tile, lds_pt);
      return;
    }
  }
  const int wave = wave_id();
  const ItemRec it = load_item(a.items + (4 * blk + wave));
  if (it.kind < 0) return;  // this path has no workgroup barrier: a wavefront may leave alone
  shrink_valu_item<DT>(a, it, sl, x, v, lds_pt + wave * (kPtWindow / 4));
}

// Expand: same block structure as shrink (one matrix-core item per workgroup, or up to 4
// independent vector-ALU items, one per wavefront); the column chunk (512 columns) comes from the
// grid.
// Grid coordinates of an expand workgroup: list position, 512-column chunk, slot entry.
// (Plain selects: assigning through the three references in branches makes the compiler route the
// block indices through a stack array, and everything indexed by them stops being wavefront-uniform.)
__device__ __forceinline__ void expand_coords(const LaunchArgs& a, int& pos, int& chunk, int& q) {
  const int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z, sf = a.slot_fastest;
  q = sf == 1 ? bx : bz;
  pos = sf == 0 ? bx : by;
  chunk = sf == 1 ? bz : (sf == 2 ? bx : by);
}

template <int DT>
__global__ __launch_bounds__(256, kWgPerCu) void k_expand(const LaunchArgs a, const SlotPtrs p) {
  __shared__ int2 my_pg[4 * kMaxRank];  // page pairs: one part per wavefront (vector-ALU items) ...
  int2* lds_pg = my_pg;                 // ... or the first part for the workgroup's matrix-core item
  int blk, chunk, q;
  expand_coords(a, blk, chunk, q);
  const SlotRec sl = a.slots[p.slot[q]];
  const float* v = (const float*)p.a[q];
  uint8_t* y = (uint8_t*)p.b[q];
  const ItemRec first = load_item(a.items + (4 * blk));
  if constexpr (DT != 2) {
    if (item_kind(first) == 1) {  // at most kMfmaTokCols tokens: larger items go to k_expand_panel
      expand_mfma_cols_item<DT>(a, first, sl, v, y, lds_pg, chunk);
      return;
    }
  }
  const int wave = wave_id();
  const ItemRec it = load_item(a.items + (4 * blk + wave));
  if (it.kind < 0) return;  // this path has no workgroup barrier: a wavefront may leave alone
  expand_valu_item<DT>(a, it, sl, v, y, my_pg + wave * kMaxRank, chunk);
}

// The matrix-core blocks of a batch with many large adapter groups (prefill): one item of up to 64
// tokens per workgroup; the list holds matrix-core blocks only (first record of each block of 4).
// HALF: the grid's chunk coordinate counts halves of 256 columns (2 per 512-column chunk), one per
// workgroup; items in the column-split form are done whole by the workgroup of the first half.
template <int DT, bool HALF>
__global__ __launch_bounds__(256, kWgPerCu) void k_expand_panel(const LaunchArgs a, const SlotPtrs p) {
  __shared__ __align__(16) uint4 op[4][8][kWave];  // 4 staged tiles of B in MFMA operand order (32 KiB)
  __shared__ int2 lds_pg[kMaxRank];
  int blk, chunk, q;
  expand_coords(a, blk, chunk, q);
  const ItemRec it = load_item(a.items + (4 * blk));
  if (item_kind(it) != 1) return;  // uniform
  const int half_sel = HALF ? (chunk & 1) : 0;
  if (HALF) chunk >>= 1;
  const SlotRec sl = a.slots[p.slot[q]];
  const float* v = (const float*)p.a[q];
  uint8_t* y = (uint8_t*)p.b[q];
  if (it.ntok <= kMfmaTokCols) {
    if (half_sel == 0) expand_mfma_cols_item<DT>(a, it, sl, v, y, lds_pg, chunk);
  } else {
    expand_panel_item<DT, HALF>(a, it, sl, v, y, op, lds_pg, chunk, half_sel);
  }
}

// ------------------------------------------------------------------------------------------
// Cooperative forms for calls too small to fill the machine: one vector-ALU item per 256-thread
// workgroup, its dependent chain of loads cut in four.  A call over a few slots is bounded by the
// length of that chain (8 chunks of d_in, or r / 8 row blocks, each a round trip to memory), not by
// bandwidth; here the four wavefronts take every fourth chunk (shrink) or every fourth block of 8
// rows (expand) and add their partial sums through LDS in wavefront order, so the result does not
// depend on timing.
// ------------------------------------------------------------------------------------------
template <int DT, int NT, bool NTW, bool COH = false>
__device__ __forceinline__ void shrink_coop_body(const LaunchArgs& a, const ItemRec it, const SlotRec sl,
                                                 const uint8_t* __restrict__ x, float* __restrict__ v,
                                                 int32_t* lds_pt, float (*red)[kShrinkRows * kValuTok]) {
  constexpr int EB = Elt<DT>::B, VEC = Elt<DT>::VEC;
  const int wave = wave_id(), lane = lane_id();
  const int r = it.rank;
  const int d_in = sl.d_in;
  const int vs = a.v_stride;
  int64_t tok[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) tok[i] = it.tok[i];
  if (it.j0 == 0 && wave == 0) {
#pragma unroll
    for (int i = 0; i < NT; ++i)
      if (i < it.ntok)
        for (int j = r + lane; j < vs; j += kWave) st_v<COH>(v + tok[i] * vs + j, 0.f);
  }
  if (r == 0) return;  // uniform over the workgroup

  const int nrows = imin(kShrinkRows, r - it.j0);
  const uint64_t rowb = (uint64_t)d_in * EB;
  const uint64_t base = (uint64_t)r * EB * (uint64_t)sl.cum + (uint64_t)it.j0 * rowb;
  const int lp = a.log2_page;
  const uint32_t win0 = (uint32_t)(base >> lp);
  const uint32_t win_n = (uint32_t)((base + (uint64_t)nrows * rowb - 1) >> lp) - win0 + 1;
  const int32_t* ptg = a.pt + it.pt_off + win0;
  {
    const bool contig = item_contig(it);
    const int32_t page0 = it.pt_off + (int32_t)win0;
    for (uint32_t i = threadIdx.x; i < win_n; i += 256) lds_pt[i] = contig ? page0 + (int32_t)i : ptg[i];
  }
  __syncthreads();

  float acc[kShrinkRows][NT];
#pragma unroll
  for (int jj = 0; jj < kShrinkRows; ++jj)
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[jj][i] = 0.f;
  constexpr int CH = kWave * VEC;
  const int full = d_in / CH * CH;
  for (int k0 = wave * CH; k0 < full; k0 += 4 * CH)
    shrink_valu_chunk<DT, NT, kShrinkRows, false, NTW>(a, x, tok, lds_pt, win0, base, rowb, nrows, d_in, k0, acc);
  if (full < d_in && ((full / CH) & 3) == wave)
    shrink_valu_chunk<DT, NT, kShrinkRows, true, NTW>(a, x, tok, lds_pt, win0, base, rowb, nrows, d_in, full, acc);
  {
    constexpr int sh = wave_sums_shift<kShrinkRows * NT>();
    const float total = wave_sums<kShrinkRows * NT>(&acc[0][0], lane);
    if ((lane & ((1 << sh) - 1)) == 0) red[wave][lane >> sh] = total;
  }
  __syncthreads();
  if (wave == 0 && lane < kShrinkRows * NT) {
    const int jj = lane / NT, i = lane % NT;
    const float sum = ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
    const int ti = i == 1 ? it.tok[1] : i == 2 ? it.tok[2] : i == 3 ? it.tok[3] : it.tok[0];
    if (jj < nrows && i < it.ntok) st_v<COH>(v + (int64_t)ti * vs + it.j0 + jj, sum);
  }
}

template <int DT>
__global__ __launch_bounds__(256) void k_shrink_coop(const LaunchArgs a, const SlotPtrs p) {
  __shared__ int32_t lds_pt[kPtWindow / 4];
  __shared__ float red[4][kShrinkRows * kValuTok];
  const ItemRec it = load_item(a.items + (a.slot_fastest ? blockIdx.z : blockIdx.x));
  if (item_kind(it) != 0) return;  // uniform over the workgroup
  const int q = a.slot_fastest ? blockIdx.x : blockIdx.z;
  const SlotRec sl = a.slots[p.slot[q]];
  const uint8_t* x = (const uint8_t*)p.a[q];
  float* v = (float*)p.b[q];
  if (item_once(it)) {
    if (it.ntok <= 1) shrink_coop_body<DT, 1, true>(a, it, sl, x, v, lds_pt, red);
    else if (it.ntok == 2) shrink_coop_body<DT, 2, true>(a, it, sl, x, v, lds_pt, red);
    else shrink_coop_body<DT, kValuTok, true>(a, it, sl, x, v, lds_pt, red);
  } else {
    if (it.ntok <= 1) shrink_coop_body<DT, 1, false>(a, it, sl, x, v, lds_pt, red);
    else if (it.ntok == 2) shrink_coop_body<DT, 2, false>(a, it, sl, x, v, lds_pt, red);
    else shrink_coop_body<DT, kValuTok, false>(a, it, sl, x, v, lds_pt, red);
  }
}

template <int DT, int NT, bool COH = false>
__device__ __forceinline__ void expand_coop_body(const LaunchArgs& a, const ItemRec it, const SlotRec sl,
                                                 const float* __restrict__ v, uint8_t* __restrict__ y, int2* lds_pg,
                                                 float* red, int chunk, float* lds_v = nullptr) {
  constexpr int EB = Elt<DT>::B, VEC = Elt<DT>::VEC;
  const int wave = wave_id(), lane = lane_id();
  const int r = it.rank;
  const int d_out = sl.d_out;
  const int n0w = chunk * (kWave * VEC);
  if (n0w >= d_out || r == 0) return;  // uniform over the workgroup
  const int n = n0w + lane * VEC;
  const bool ok = n < d_out;
  const uint32_t lane_b = ok ? lane * 16 : 0;
  const int vs = a.v_stride;
  const int lp = a.log2_page;
  const uint32_t pmask = (1u << lp) - 1;
  const uint64_t rowb = (uint64_t)d_out * EB;
  const uint64_t base = (uint64_t)r * EB * ((uint64_t)sl.cum + (uint64_t)sl.d_in) + (uint64_t)n0w * EB;
  {
    const int n_pt = table_len(a, r, EB);
    const int32_t* ptg = a.pt + it.pt_off;
    const bool contig = item_contig(it);
    for (int j = threadIdx.x; j < r; j += 256) {
      const uint64_t vo = base + (uint64_t)j * rowb;
      const uint32_t q0 = (uint32_t)(vo >> lp);
      const uint32_t q1 = imin((int)((vo + kWave * 16 - 1) >> lp), n_pt - 1);
      lds_pg[j] = contig ? make_int2(it.pt_off + (int)q0, it.pt_off + (int)q1) : make_int2(ptg[q0], ptg[q1]);
    }
  }
  // wavefront w finishes token w: its row of y is requested now
  const bool fin = wave < it.ntok;
  const int tokw = wave == 1 ? it.tok[1] : wave == 2 ? it.tok[2] : wave == 3 ? it.tok[3] : it.tok[0];  // no indexed array
  uint8_t* yp = y + ((uint64_t)(fin ? tokw : it.tok[0]) * d_out + (ok ? n : n0w)) * EB;
  uint4 yq = make_uint4(0, 0, 0, 0);
  if (fin) yq = ldy16(yp);
  const float* vrow[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) vrow[i] = v + (int64_t)it.tok[i] * vs;
  if constexpr (COH) {  // the tokens' rows of v through device-scope loads, once, into LDS (row i at lds_v + i * r)
#pragma unroll
    for (int i = 0; i < NT; ++i)
      for (int j = threadIdx.x; j < r; j += 256) lds_v[i * r + j] = ld_v<true>(vrow[i] + j);
  }
  __syncthreads();

  float acc[NT][VEC];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[i][e] = 0.f;
  constexpr int U = kExpandU;
  const int nfull = r / U;  // whole blocks of U rows, dealt round robin; the ragged rest goes to the next wavefront
  for (int blk = wave; blk < nfull; blk += 4) {
    const int j = blk * U;
    uint4 wq[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t vo = base + (uint64_t)(j + u) * rowb;
      const uint32_t inpage = ((uint32_t)vo & pmask) + lane_b;
      const int2 pp = lds_pg[j + u];
      const uint64_t pg = (uint64_t)(uint32_t)((inpage >> lp) ? pp.y : pp.x);
      wq[u] = ldw16<false>(a.slab + (pg << lp) + (inpage & pmask));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float wf[VEC];
      unpack<DT>(wq[u], wf);
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        const float vj = COH ? lds_v[i * r + j + u] : vrow[i][j + u];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[i][e] = __builtin_fmaf(vj, wf[e], acc[i][e]);
      }
    }
  }
  if ((nfull & 3) == wave) {
    for (int j = nfull * U; j < r; ++j) {
      const uint64_t vo = base + (uint64_t)j * rowb;
      const uint32_t inpage = ((uint32_t)vo & pmask) + lane_b;
      const int2 pp = lds_pg[j];
      const uint64_t pg = (uint64_t)(uint32_t)((inpage >> lp) ? pp.y : pp.x);
      float wf[VEC];
      unpack<DT>(ldw16<false>(a.slab + (pg << lp) + (inpage & pmask)), wf);
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        const float vj = COH ? lds_v[i * r + j] : vrow[i][j];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[i][e] = __builtin_fmaf(vj, wf[e], acc[i][e]);
      }
    }
  }
  // red[wave][token][e][lane]
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int e = 0; e < VEC; ++e) red[((wave * kValuTok + i) * 8 + e) * kWave + lane] = acc[i][e];
  __syncthreads();
  if (fin && ok && wave < NT) {
    float yf[VEC];
    unpack<DT>(yq, yf);
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const float s0 = red[((0 * kValuTok + wave) * 8 + e) * kWave + lane], s1 = red[((1 * kValuTok + wave) * 8 + e) * kWave + lane];
      const float s2 = red[((2 * kValuTok + wave) * 8 + e) * kWave + lane], s3 = red[((3 * kValuTok + wave) * 8 + e) * kWave + lane];
      yf[e] = __builtin_fmaf(it.scale, ((s0 + s1) + s2) + s3, yf[e]);
    }
    sty16(yp, pack<DT>(yf));
  }
}

template <int DT>
__global__ __launch_bounds__(256) void k_expand_coop(const LaunchArgs a, const SlotPtrs p) {
  static_assert(kValuTok <= 4, "one finishing wavefront per token of the item");
  __shared__ int2 lds_pg[kMaxRank];
  __shared__ float red[4 * kValuTok * 8 * kWave];  // 32 KiB
  int pos, chunk, q;
  expand_coords(a, pos, chunk, q);
  const ItemRec it = load_item(a.items + (pos));
  if (item_kind(it) != 0) return;  // uniform over the workgroup
  const SlotRec sl = a.slots[p.slot[q]];
  const float* v = (const float*)p.a[q];
  uint8_t* y = (uint8_t*)p.b[q];
  if (it.ntok <= 1) expand_coop_body<DT, 1>(a, it, sl, v, y, lds_pg, red, chunk);
  else if (it.ntok == 2) expand_coop_body<DT, 2>(a, it, sl, v, y, lds_pg, red, chunk);
  else expand_coop_body<DT, kValuTok>(a, it, sl, v, y, lds_pg, red, chunk);
}

// ------------------------------------------------------------------------------------------
// Shrink and expand of a small call in one launch.  Workgroup w of a persistent grid of 256-thread
// workgroups runs tasks w, w + grid, ...: first the shrink tasks of all slots, slot after slot, then the
// expand tasks; each task is one workgroup's worth of an ordinary launch (a block of 4 records, or one
// cooperative record, times the 512-column chunk for expand).  An expand task needs every row of v of
// its slot: a shrink task adds one to its slot's counter once its stores of v have been performed, the
// task that completes the count publishes it in a few flag words, and an expand task polls one of
// them before it starts.  A workgroup's tasks ascend, so every shrink task comes behind shrink tasks
// only and runs without waiting for anything; the grid is no larger than what is resident together.
// The poll is bounded all the same (spin_limit polls, then the task is given up, counted for the host,
// and the workgroup goes on).  The sums are those of the separate kernels, in the same order.
// ------------------------------------------------------------------------------------------
constexpr int kFusedPg = 4 * kMaxRank * sizeof(int2);                  // expand block: page pairs of four vector-ALU items
constexpr int kFusedV = kValuTok * kMaxRank * sizeof(float);           // rows of v of one vector-ALU item
constexpr int kFusedLds = kFusedPg + 4 * kFusedV;                      // the expand block with its four items' rows of v: the largest user
static_assert(kFusedLds >= 4 * 2 * kSmRows * kSmPitch + kPtWindow * 4, "shrink block: tiles and page-table window");
static_assert(kFusedLds >= (int)(kMaxRank * sizeof(int2) + 4 * kValuTok * 8 * kWave * sizeof(float)) + kFusedV, "cooperative expand: page pairs, partial sums, rows of v");

template <int DT>
__global__ __launch_bounds__(256, kWgPerCu) void k_delta_queue(const FusedArgs f, const FusedPtrs p) {
  __shared__ __align__(16) uint8_t lds[kFusedLds];
  __shared__ int s_ready;
  LaunchArgs a;
  a.slab = f.slab; a.perm = f.perm; a.pt = f.pt; a.items = nullptr; a.slots = f.slots;
  a.elems_per_rank = f.elems_per_rank; a.n_items = 0; a.pad0 = 0; a.log2_page = f.log2_page; a.v_stride = f.v_stride;
  a.slot_fastest = 0; a.pad = 0;
  const int per_slot_e = f.n_e * f.chunks;
  const int total_s = f.n_s * f.n_slots;
  const int total = total_s + per_slot_e * f.n_slots;
  const int wave = wave_id();
  for (int t = blockIdx.x; t < total; t += gridDim.x) {
    __syncthreads();  // the previous task is done with the LDS space
    const bool is_shrink = t < total_s;
    const int q = is_shrink ? t / f.n_s : (t - total_s) / per_slot_e;
    const int w = is_shrink ? t - q * f.n_s : (t - total_s) - q * per_slot_e;
    const SlotRec sl = f.slots[p.slot[q]];
    if (is_shrink) {
      // ---- a shrink task of slot q
      const uint8_t* x = (const uint8_t*)p.x[q];
      float* v = p.v[q];
      if (f.coop_s) {
        int32_t* lds_pt = reinterpret_cast<int32_t*>(lds);
        auto red = reinterpret_cast<float(*)[kShrinkRows * kValuTok]>(lds + (kPtWindow / 4) * 4);
        const ItemRec it = load_item(f.items_s + w);
        if (item_kind(it) == 0) {
          if (item_once(it)) {
            if (it.ntok <= 1) shrink_coop_body<DT, 1, true, true>(a, it, sl, x, v, lds_pt, red);
            else if (it.ntok == 2) shrink_coop_body<DT, 2, true, true>(a, it, sl, x, v, lds_pt, red);
            else shrink_coop_body<DT, kValuTok, true, true>(a, it, sl, x, v, lds_pt, red);
          } else {
            if (it.ntok <= 1) shrink_coop_body<DT, 1, false, true>(a, it, sl, x, v, lds_pt, red);
            else if (it.ntok == 2) shrink_coop_body<DT, 2, false, true>(a, it, sl, x, v, lds_pt, red);
            else shrink_coop_body<DT, kValuTok, false, true>(a, it, sl, x, v, lds_pt, red);
          }
        }
      } else {
        auto tile = reinterpret_cast<uint8_t(*)[2][kSmRows * kSmPitch]>(lds);
        int32_t* lds_pt = reinterpret_cast<int32_t*>(lds + 4 * 2 * kSmRows * kSmPitch);
        const ItemRec first = load_item(f.items_s + 4 * w);
        bool matrix = false;
        if constexpr (DT != 2) {
          if (item_kind(first) == 1) {
            matrix = true;
            if (item_once(first)) shrink_mfma4_body<DT, true, 2, true>(a, first, sl, x, v, tile, lds_pt);
            else shrink_mfma4_body<DT, false, 2, true>(a, first, sl, x, v, tile, lds_pt);
          }
        }
        if (!matrix) {
          const ItemRec it = load_item(f.items_s + 4 * w + wave);
          if (it.kind >= 0) shrink_valu_item<DT, true>(a, it, sl, x, v, lds_pt + wave * (kPtWindow / 4));
        }
      }
      // the stores of v are device-scope stores; the barrier waits until every wavefront's have been performed,
      // then one thread counts the task, and the last one of the slot raises the slot's flags
      __syncthreads();
      if (threadIdx.x == 0) {
        const uint32_t done = atomicAdd(&f.queue[q], 1u) + 1u;
        if (done == p.target[q]) {
#pragma unroll
          for (int k = 0; k < kFlagCopies; ++k)
            __hip_atomic_store(&f.queue[kQueueFlag0 + (q * kFlagCopies + k) * kFlagStride], done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    } else {
      // ---- an expand task of slot q: wait for the slot's rows of v
      if (threadIdx.x == 0) {
        int ready = 0;
        const uint32_t* flag = &f.queue[kQueueFlag0 + (q * kFlagCopies + (int)(blockIdx.x % kFlagCopies)) * kFlagStride];
        const uint32_t target = p.target[q];
        for (uint32_t n = 0; n <= f.spin_limit; ++n) {
          // (the counters only grow; the difference is taken so that a wrap after 2^32 tasks does no harm)
          if ((int32_t)(__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) >= 0) { ready = 1; break; }
          __builtin_amdgcn_s_sleep(8);
        }
        if (!ready) __hip_atomic_fetch_add(f.timeouts, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        s_ready = ready;
      }
      __syncthreads();
      const int ready = __builtin_amdgcn_readfirstlane(s_ready);
      if (!ready) continue;  // given up: y of this task stays as it was, the host finds the count
      // (v is read with device-scope loads, issued after the barrier above: they see what the counter covers)
      const int blk = w / f.chunks, chunk = w - blk * f.chunks;
      const float* v = p.v[q];
      uint8_t* y = (uint8_t*)p.y[q];
      if (f.coop_e) {
        int2* lds_pg = reinterpret_cast<int2*>(lds);
        float* red = reinterpret_cast<float*>(lds + kMaxRank * sizeof(int2));
        float* lds_v = reinterpret_cast<float*>(lds + kMaxRank * sizeof(int2) + 4 * kValuTok * 8 * kWave * sizeof(float));
        const ItemRec it = load_item(f.items_e + blk);
        if (item_kind(it) == 0) {
          if (it.ntok <= 1) expand_coop_body<DT, 1, true>(a, it, sl, v, y, lds_pg, red, chunk, lds_v);
          else if (it.ntok == 2) expand_coop_body<DT, 2, true>(a, it, sl, v, y, lds_pg, red, chunk, lds_v);
          else expand_coop_body<DT, kValuTok, true>(a, it, sl, v, y, lds_pg, red, chunk, lds_v);
        }
      } else {
        int2* my_pg = reinterpret_cast<int2*>(lds);
        const ItemRec first = load_item(f.items_e + 4 * blk);
        bool matrix = false;
        if constexpr (DT != 2) {
          if (item_kind(first) == 1) {
            matrix = true;
            expand_mfma_cols_item<DT, true>(a, first, sl, v, y, my_pg, chunk);
          }
        }
        if (!matrix) {
          const ItemRec it = load_item(f.items_e + 4 * blk + wave);
          if (it.kind >= 0)
            expand_valu_item<DT, true>(a, it, sl, v, y, my_pg + wave * kMaxRank, chunk, reinterpret_cast<float*>(lds + kFusedPg + wave * kFusedV));
        }
      }
    }
  }
}

// Staged load (Sec. III-B: adapters arrive in a staging area and are then moved into their pages):
// the blob lies contiguous in `staging`; workgroup (piece, page) copies one 16 KiB piece of one
// virtual page to the physical page that the run table names.  Streaming loads and stores: neither
// side is read again before the next batch.
__global__ __launch_bounds__(256) void k_scatter_pages(const uint8_t* __restrict__ staging, uint8_t* __restrict__ slab,
                                                       const ScatterRuns runs, const int log2_page,
                                                       const uint64_t bytes, const int vpage0) {
  const int vpage = vpage0 + (int)blockIdx.y;
  int lo = 0, hi = runs.n_runs - 1;  // last run that starts at or before vpage
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (runs.first_vpage[mid] <= vpage) lo = mid; else hi = mid - 1;
  }
  const uint64_t page = (uint64_t)(runs.phys_page[lo] + (vpage - runs.first_vpage[lo]));
  const uint64_t in_page = (uint64_t)blockIdx.x * kScatterPiece;
  const uint64_t src0 = ((uint64_t)vpage << log2_page) + in_page;
  if (src0 >= bytes) return;
  uint64_t left = bytes - src0;  // to the end of the blob, of the page and of the piece
  const uint64_t page_left = ((uint64_t)1 << log2_page) - in_page;
  if (page_left < left) left = page_left;
  const uint32_t n = (uint32_t)(left < (uint64_t)kScatterPiece ? left : (uint64_t)kScatterPiece);
  const uint8_t* src = staging + src0;
  uint8_t* dst = slab + (page << log2_page) + in_page;
#pragma unroll
  for (uint32_t o = threadIdx.x * 16u; o < (uint32_t)kScatterPiece; o += 256u * 16u) {
    if (o < n) {
      const u32x4_t q = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src + o));
      __builtin_nontemporal_store(q, reinterpret_cast<u32x4_t*>(dst + o));
    }
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Static device array for callers that cannot allocate (plora_delta_static): 16 MiB per GPU the
// library runs on, held until the process ends.  On the host the array's name only stands for the
// symbol; its device address is looked up once per device and every use goes through that pointer.
// ------------------------------------------------------------------------------------------
constexpr uint64_t kStaticScratchBytes = 16ull << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

uint64_t static_scratch_bytes() { return kStaticScratchBytes; }

hipError_t static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* q = nullptr;
    e = hipGetSymbolAddress(&q, HIP_SYMBOL(scratch));  // with device `dev` current: each GPU has its own copy
    if (e != hipSuccess) return e;
    if (!q) return hipErrorInvalidSymbol;
    ptr[dev] = q;
  }
  *out = ptr[dev];
  return hipSuccess;
}

// Launch with optional timing events attached to the dispatch itself (start / stop timestamps of
// this kernel; no extra packets in the queue).
typedef void (*KernelFn)(const LaunchArgs, const SlotPtrs);
static void launch(KernelFn k, dim3 grid, dim3 block, hipStream_t st, hipEvent_t e0, hipEvent_t e1, const LaunchArgs& a,
                   const SlotPtrs& p) {
  if (e0 || e1) hipExtLaunchKernelGGL(k, grid, block, 0, st, e0, e1, 0, a, p);
  else hipLaunchKernelGGL(k, grid, block, 0, st, a, p);
}

hipError_t launch_shrink(int dtype, const LaunchArgs& a0, const SlotPtrs& p, int n_slots, int mode, hipStream_t st,
                         hipEvent_t e0, hipEvent_t e1) {
  const bool single = mode == kModeCoop;  // one record per workgroup
  if (a0.n_items <= 0 || n_slots <= 0) return hipSuccess;
  if (!single && a0.n_items % 4) return hipErrorInvalidValue;  // blocks of 4 records
  // kModeDeep: as kModeBlocks with two runs in flight per matrix-core item (fp32 has no such items)
  static const KernelFn table[3][3] = {{k_shrink<0, 1>, k_shrink<1, 1>, k_shrink<2, 1>},
                                       {k_shrink_coop<0>, k_shrink_coop<1>, k_shrink_coop<2>},
                                       {k_shrink<0, 2>, k_shrink<1, 2>, k_shrink<2, 1>}};
  if (mode < 0 || mode > 2 || dtype < 0 || dtype > 2) return hipErrorInvalidValue;
  LaunchArgs a = a0;
  const int per = single ? 1 : 4;  // records per workgroup
  const int n_blocks = a0.n_items / per;
  const int step = a0.slot_fastest ? 65535 : n_blocks;  // grid.z is limited to 65535
  for (int first = 0; first < n_blocks; first += step) {
    const int nb = n_blocks - first < step ? n_blocks - first : step;
    a.items = a0.items + per * first;
    a.n_items = per * nb;
    const dim3 grid = a.slot_fastest ? dim3(n_slots, 1, nb) : dim3(nb, 1, n_slots);
    launch(table[mode][dtype], grid, dim3(256), st, first == 0 ? e0 : nullptr, first + step >= n_blocks ? e1 : nullptr, a, p);
  }
  return hipGetLastError();
}

hipError_t launch_expand(int dtype, const LaunchArgs& a0, const SlotPtrs& p, int n_slots, int max_chunks, int mode,
                         hipStream_t st, hipEvent_t e0, hipEvent_t e1) {
  const bool single = mode == kModeCoop;  // one record per workgroup
  if (a0.n_items <= 0 || n_slots <= 0 || max_chunks <= 0) return hipSuccess;
  if ((!single && a0.n_items % 4) || max_chunks > 65535) return hipErrorInvalidValue;
  static const KernelFn table[4][3] = {{k_expand<0>, k_expand<1>, k_expand<2>},
                                       {k_expand_coop<0>, k_expand_coop<1>, k_expand_coop<2>},
                                       {k_expand_panel<0, false>, k_expand_panel<1, false>, nullptr},
                                       {k_expand_panel<0, true>, k_expand_panel<1, true>, nullptr}};
  if (mode < 0 || mode > 3 || dtype < 0 || dtype > 2 || !table[mode][dtype]) return hipErrorInvalidValue;
  const int grid_chunks = mode == kModePanelHalf ? 2 * max_chunks : max_chunks;  // halves of 256 columns
  if (grid_chunks > 65535) return hipErrorInvalidValue;
  LaunchArgs a = a0;
  const int per = single ? 1 : 4;  // records per workgroup
  const int n_blocks = a0.n_items / per;
  const int step = a0.slot_fastest ? 65535 : n_blocks;  // grid.y is limited to 65535
  for (int first = 0; first < n_blocks; first += step) {
    const int nb = n_blocks - first < step ? n_blocks - first : step;
    a.items = a0.items + per * first;
    a.n_items = per * nb;
    const dim3 grid = a.slot_fastest == 1 ? dim3(n_slots, nb, grid_chunks)
                    : a.slot_fastest == 2 ? dim3(grid_chunks, nb, n_slots) : dim3(nb, grid_chunks, n_slots);
    launch(table[mode][dtype], grid, dim3(256), st, first == 0 ? e0 : nullptr, first + step >= n_blocks ? e1 : nullptr, a, p);
  }
  return hipGetLastError();
}

hipError_t launch_delta_queue(int dtype, const FusedArgs& f, const FusedPtrs& p, hipStream_t st, hipEvent_t e0, hipEvent_t e1) {
  typedef void (*Fn)(const FusedArgs, const FusedPtrs);
  static const Fn table[3] = {k_delta_queue<0>, k_delta_queue<1>, k_delta_queue<2>};
  if (dtype < 0 || dtype > 2 || f.n_slots < 1 || f.n_slots > kMaxSlotsFused || f.n_s < 0 || f.n_e < 0 || f.chunks < 1 || !f.queue || !f.timeouts)
    return hipErrorInvalidValue;
  const int64_t total = ((int64_t)f.n_s + (int64_t)f.n_e * f.chunks) * f.n_slots;
  if (total <= 0) return hipSuccess;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  // a persistent grid: as many workgroups as stay resident together on this device, or fewer if the tasks are fewer
  static int resident_of[64] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (resident_of[dev] == 0) {
    int cus = 0, per_cu = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, table[dtype], 256, 0);
    if (e != hipSuccess) return e;
    if (cus < 1 || per_cu < 1) return hipErrorInvalidValue;
    resident_of[dev] = cus * (per_cu < kWgPerCu ? per_cu : kWgPerCu);
  }
  const int64_t resident = resident_of[dev];
  const dim3 grid((unsigned)(total < resident ? total : resident));
  if (e0 || e1) hipExtLaunchKernelGGL(table[dtype], grid, dim3(256), 0, st, e0, e1, 0, f, p);
  else hipLaunchKernelGGL(table[dtype], grid, dim3(256), 0, st, f, p);
  return hipGetLastError();
}

hipError_t launch_scatter(const uint8_t* staging, uint8_t* slab, int log2_page, uint64_t bytes, const int32_t* pt,
                          uint32_t n_pages, hipStream_t st) {
  if (bytes == 0 || n_pages == 0) return hipSuccess;
  if (!staging || !slab || !pt || log2_page < 12 || (bytes & 15) || bytes > ((uint64_t)n_pages << log2_page) ||
      bytes <= ((uint64_t)(n_pages - 1) << log2_page))
    return hipErrorInvalidValue;
  const uint64_t P = (uint64_t)1 << log2_page;
  const unsigned pieces = (unsigned)((P + kScatterPiece - 1) / kScatterPiece);
  uint32_t l = 0;
  while (l < n_pages) {  // one launch per kScatterRuns runs of consecutive physical pages
    ScatterRuns runs;
    runs.n_runs = 0;
    const uint32_t vpage0 = l;
    while (l < n_pages && runs.n_runs < kScatterRuns) {
      uint32_t h = l + 1;
      while (h < n_pages && pt[h] == pt[h - 1] + 1) ++h;
      runs.first_vpage[runs.n_runs] = (int32_t)l;
      runs.phys_page[runs.n_runs] = pt[l];
      ++runs.n_runs;
      l = h;
    }
    for (uint32_t v0 = vpage0; v0 < l; v0 += 65535u) {  // grid.y is limited to 65535
      const uint32_t nv = l - v0 < 65535u ? l - v0 : 65535u;
      hipLaunchKernelGGL(k_scatter_pages, dim3(pieces, nv), dim3(256), 0, st, staging, slab, runs, log2_page, bytes, (int)v0);
    }
  }
  return hipGetLastError();
}

}  // namespace plora
