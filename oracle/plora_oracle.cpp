// CPU oracle for the paged multi-LoRA delta.  TEST INFRASTRUCTURE ONLY: nothing on the
// product path may include, link or call this file.  It shares no code with the HIP
// library; it is written straight from the paper's statement of the method.
//
// What it computes, with the passage that defines each part:
//   * LoRA delta (Sec. II-A, Eq. 1): W = W0 + B A, B in R^{d x r}, A in R^{r x k}.  For a
//     token with input x the adapter adds  B (A x).  Stored orientation used here: the
//     paper's A row-major (r rows of d_in) and the paper's B transposed, row-major (r rows
//     of d_out), so in row-vector form  delta = scale * (x A^T) B^T_stored.
//   * Page structure (Sec. III-C "Page Structure"): an adapter of S bytes occupies
//     ceil(S / P) fixed-size pages, scattered physically, contiguous virtually.
//   * Page table (Sec. III-C "Page Table"): logical page l of an adapter -> physical page;
//     virtual byte o lives at  pool + pt[o / P] * P + o % P.  Translation of a batch
//     (token -> adapter grouping) happens once per batch.
//   * Evict (Sec. III-B "Eviction Policy", mechanism only): the adapter's pages return to
//     the free set.
// Readings where the paper is silent (placement policy = the lowest-numbered free pages in
// ascending order; tight packing of the blob slot after slot as [A_s | B_s]; per-adapter
// fp32 scale applied once at the end; v kept in the accumulator type between the two
// steps; one round-to-nearest-even of y_old + scale*acc to the element type).
//
// Arithmetic: naive per-token loops.  acc_mode 0 = fp32 accumulators (compile with
// -ffp-contract=off so every multiply and add rounds on its own); acc_mode 1 = fp64
// accumulators (the reference used for tolerance checks).
//
// Pins (tests/test_oracle_*.py): page-count closed form and the paper's printed adapter
// sizes, allocator invariants and a brute-force rescan allocator, byte-exact virtual view,
// numpy stable argsort for the batch translation, fp64 dense x (A^T B) for the delta, and
// the invariances listed in the tests; hand-worked examples and invariants for the compaction
// (tests/test_oracle_compact.py).  The eviction *policy* is not part of this file.

#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <cmath>
#include <vector>
#include <algorithm>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

enum { O_OK = 0, O_INVAL = -1, O_NOMEM = -2, O_EXISTS = -3, O_NOTFOUND = -4 };
enum { DT_F16 = 0, DT_BF16 = 1, DT_F32 = 2 };

struct OAdapter {
  bool present = false;
  int rank = 0;
  float scale = 0.f;
  std::vector<int32_t> pt;
};

struct OPool {
  size_t P = 0;
  uint32_t n_pages = 0;
  int n_slots = 0;
  std::vector<int64_t> d_in, d_out, cum;  // cum[s] = sum_{s'<s} (d_in + d_out)
  int dtype = 0;
  size_t elt = 2;
  int max_adapters = 0, max_rank = 0;
  int64_t C = 0;  // sum over slots of (d_in + d_out)
  uint8_t* mem = nullptr;
  std::vector<uint8_t> is_free;
  uint32_t n_free = 0;
  std::vector<OAdapter> ad;
  uint64_t loads = 0, evictions = 0, nomem = 0, resident_bytes = 0;
};

// ---- element decoding / encoding, written out bit by bit --------------------------------

inline float bits_to_float(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }
inline uint32_t float_to_bits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }

inline float bf16_to_float(uint16_t h) { return bits_to_float(uint32_t(h) << 16); }

inline float f16_to_float(uint16_t h) {
  uint32_t sign = uint32_t(h & 0x8000u) << 16;
  int e = (h >> 10) & 0x1f;
  uint32_t m = h & 0x3ffu;
  if (e == 0) {
    if (m == 0) return bits_to_float(sign);
    float v = std::ldexp(float(m), -24);  // subnormal: m * 2^-24, exact in fp32
    return (sign ? -v : v);
  }
  if (e == 31) return bits_to_float(sign | 0x7f800000u | (m << 13));
  return bits_to_float(sign | uint32_t(e - 15 + 127) << 23 | (m << 13));
}

inline uint16_t float_to_bf16_rne(float f) {
  uint32_t u = float_to_bits(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);  // quiet NaN
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  return uint16_t(u >> 16);
}

inline uint16_t float_to_f16_rne(float f) {
  uint32_t u = float_to_bits(f);
  uint16_t sign = uint16_t((u >> 16) & 0x8000u);
  uint32_t a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return uint16_t(sign | 0x7e00u);
  if (a >= 0x477ff000u) {  // >= 65520 rounds to inf (65504 is the largest finite half)
    return uint16_t(sign | 0x7c00u);
  }
  if (a < 0x33000001u) return sign;  // <= 2^-25 rounds to zero (ties to even -> 0)
  int e = int(a >> 23) - 127;
  uint32_t m = (a & 0x7fffffu) | 0x800000u;  // 24-bit significand
  int shift;                                 // bits to drop from the 24-bit significand
  uint32_t base;
  if (e < -14) { shift = 13 + (-14 - e); base = 0; }           // subnormal half
  else { shift = 13; base = uint32_t(e + 15) << 10; m &= 0x7fffffu; }
  uint32_t q = m >> shift;
  uint32_t rem = m & ((1u << shift) - 1u);
  uint32_t half = 1u << (shift - 1);
  if (rem > half || (rem == half && (q & 1u))) q += 1;  // carry into the exponent is correct
  return uint16_t(sign | (base + q));
}

inline float load_elt(const OPool* p, const uint8_t* at) {
  if (p->dtype == DT_F32) { float f; std::memcpy(&f, at, 4); return f; }
  uint16_t h; std::memcpy(&h, at, 2);
  return p->dtype == DT_BF16 ? bf16_to_float(h) : f16_to_float(h);
}

inline void store_elt(const OPool* p, uint8_t* at, float f) {
  if (p->dtype == DT_F32) { std::memcpy(at, &f, 4); return; }
  uint16_t h = p->dtype == DT_BF16 ? float_to_bf16_rne(f) : float_to_f16_rne(f);
  std::memcpy(at, &h, 2);
}

// ---- virtual -> physical (Sec. III-C "Page Table") ---------------------------------------

inline const uint8_t* vaddr(const OPool* p, const OAdapter& a, uint64_t o) {
  return p->mem + uint64_t(a.pt[o / p->P]) * p->P + (o % p->P);
}
inline uint64_t off_A(const OPool* p, int s, int r) { return uint64_t(r) * p->elt * uint64_t(p->cum[s]); }
inline uint64_t off_B(const OPool* p, int s, int r) {
  return off_A(p, s, r) + uint64_t(r) * uint64_t(p->d_in[s]) * p->elt;
}

template <typename ACC>
void shrink_token(const OPool* p, int s, const uint8_t* x, int64_t t, const OAdapter& a, ACC* vrow) {
  const int64_t din = p->d_in[s];
  const uint64_t base = off_A(p, s, a.rank);
  for (int j = 0; j < a.rank; ++j) {
    ACC acc = 0;
    for (int64_t k = 0; k < din; ++k) {
      ACC xv = (ACC)load_elt(p, x + (uint64_t(t) * din + k) * p->elt);
      ACC av = (ACC)load_elt(p, vaddr(p, a, base + (uint64_t(j) * din + k) * p->elt));
      ACC prod = xv * av;
      acc = acc + prod;
    }
    vrow[j] = acc;
  }
}

template <typename ACC>
void expand_token(const OPool* p, int s, const ACC* vrow, uint8_t* y, int64_t t, const OAdapter& a) {
  const int64_t dout = p->d_out[s];
  const uint64_t base = off_B(p, s, a.rank);
  for (int64_t n = 0; n < dout; ++n) {
    ACC acc = 0;
    for (int j = 0; j < a.rank; ++j) {
      ACC bv = (ACC)load_elt(p, vaddr(p, a, base + (uint64_t(j) * dout + n) * p->elt));
      ACC prod = vrow[j] * bv;
      acc = acc + prod;
    }
    uint8_t* at = y + (uint64_t(t) * dout + n) * p->elt;
    ACC yo = (ACC)load_elt(p, at);
    ACC sc = (ACC)a.scale * acc;
    ACC yn = yo + sc;
    store_elt(p, at, (float)yn);  // fp64 mode: one extra rounding to fp32 first (<= 2^-24 rel.)
  }
}

}  // namespace

extern "C" {

int oracle_pool_create(uint64_t page_bytes, uint32_t n_pages, int32_t n_slots, const int32_t* d_in,
                       const int32_t* d_out, int32_t dtype, int32_t max_adapters, int32_t max_rank,
                       void** out) {
  if (!out || !d_in || !d_out || n_slots <= 0 || n_pages == 0 || max_adapters <= 0 || max_rank <= 0) return O_INVAL;
  if (page_bytes < 4096 || (page_bytes & (page_bytes - 1))) return O_INVAL;
  if (dtype < 0 || dtype > 2) return O_INVAL;
  OPool* p = new OPool;
  p->P = page_bytes; p->n_pages = n_pages; p->n_slots = n_slots; p->dtype = dtype;
  p->elt = dtype == DT_F32 ? 4 : 2;
  p->max_adapters = max_adapters; p->max_rank = max_rank;
  int64_t c = 0;
  for (int s = 0; s < n_slots; ++s) {
    if (d_in[s] <= 0 || d_out[s] <= 0 || d_in[s] % 8 || d_out[s] % 8) { delete p; return O_INVAL; }
    p->d_in.push_back(d_in[s]); p->d_out.push_back(d_out[s]); p->cum.push_back(c);
    c += int64_t(d_in[s]) + d_out[s];
  }
  p->C = c;
  p->mem = (uint8_t*)std::calloc(size_t(n_pages), page_bytes);  // lazily zero pages
  if (!p->mem) { delete p; return O_NOMEM; }
  p->is_free.assign(n_pages, 1); p->n_free = n_pages;
  p->ad.resize(max_adapters);
  *out = p;
  return O_OK;
}

int oracle_pool_destroy(void* h) {
  OPool* p = (OPool*)h;
  if (!p) return O_INVAL;
  std::free(p->mem);
  delete p;
  return O_OK;
}

uint64_t oracle_adapter_bytes(void* h, int32_t rank) {
  OPool* p = (OPool*)h;
  return uint64_t(rank) * p->elt * uint64_t(p->C);
}

// Place adapter `id`: m = ceil(S / P) pages, the m lowest-numbered free ones, ascending.
// On success copies the blob page by page in logical order; the tail of the last page is
// left as it was.  page_table_out (may be null) receives m entries.
int oracle_load(void* h, int32_t id, int32_t rank, float scale, const void* blob,
                int32_t* page_table_out, uint32_t* n_pages_out) {
  OPool* p = (OPool*)h;
  if (!p || !blob || id < 0 || id >= p->max_adapters || rank < 1 || rank > p->max_rank) return O_INVAL;
  OAdapter& a = p->ad[id];
  if (a.present) return O_EXISTS;
  uint64_t S = uint64_t(rank) * p->elt * uint64_t(p->C);
  uint64_t m = (S + p->P - 1) / p->P;
  if (m > p->n_free) { p->nomem++; return O_NOMEM; }
  a.pt.clear();
  for (uint32_t q = 0; q < p->n_pages && a.pt.size() < m; ++q)
    if (p->is_free[q]) { a.pt.push_back(int32_t(q)); }
  for (int32_t q : a.pt) p->is_free[q] = 0;
  p->n_free -= uint32_t(m);
  for (uint64_t l = 0; l < m; ++l) {
    uint64_t lo = l * p->P, hi = std::min<uint64_t>(lo + p->P, S);
    std::memcpy(p->mem + uint64_t(a.pt[l]) * p->P, (const uint8_t*)blob + lo, hi - lo);
  }
  a.present = true; a.rank = rank; a.scale = scale;
  p->loads++; p->resident_bytes += S;
  if (page_table_out) std::memcpy(page_table_out, a.pt.data(), m * 4);
  if (n_pages_out) *n_pages_out = uint32_t(m);
  return O_OK;
}

int oracle_evict(void* h, int32_t id) {
  OPool* p = (OPool*)h;
  if (!p || id < 0 || id >= p->max_adapters) return O_INVAL;
  OAdapter& a = p->ad[id];
  if (!a.present) return O_NOTFOUND;
  for (int32_t q : a.pt) p->is_free[q] = 1;
  p->n_free += uint32_t(a.pt.size());
  p->resident_bytes -= uint64_t(a.rank) * p->elt * uint64_t(p->C);
  a.pt.clear(); a.present = false; a.rank = 0; a.scale = 0.f;
  p->evictions++;
  return O_OK;
}

// Compaction (Sec. III-C "Defragmentation": background compaction coalesces free pages).  The paper
// gives no procedure.  Reading: the resident adapters are taken in ascending order of their first
// page; each is placed anew as a load would place it if its own pages were free as well - on the m
// lowest-numbered pages among the free ones and its own, ascending - and its bytes move with it.
// Adapters named in skip[] stay where they are (the library leaves out adapters that an open batch
// uses or whose load has not completed).  max_pages > 0 bounds the pages whose content moves in one
// call: an adapter moves whole or not at all, and the first one that does not fit ends the call.
// moved_out[0] = pages moved, moved_out[1] = adapters moved.
int oracle_compact(void* h, uint32_t max_pages, const int32_t* skip, int32_t n_skip, uint32_t* moved_out) {
  OPool* p = (OPool*)h;
  if (!p || n_skip < 0 || (n_skip > 0 && !skip)) return O_INVAL;
  std::vector<int32_t> order;
  for (int32_t id = 0; id < p->max_adapters; ++id)
    if (p->ad[id].present && std::find(skip, skip + n_skip, id) == skip + n_skip) order.push_back(id);
  std::sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return p->ad[x].pt[0] < p->ad[y].pt[0]; });
  uint32_t pages = 0, adapters = 0;
  for (int32_t id : order) {
    OAdapter& a = p->ad[id];
    const size_t m = a.pt.size();
    for (int32_t q : a.pt) p->is_free[q] = 1;
    std::vector<int32_t> to;
    for (uint32_t q = 0; q < p->n_pages && to.size() < m; ++q)
      if (p->is_free[q]) to.push_back(int32_t(q));
    uint32_t changed = 0;
    for (size_t l = 0; l < m; ++l) changed += to[l] != a.pt[l];
    if (max_pages > 0 && pages + changed > max_pages) {  // does not fit: it stays, and the call ends
      for (int32_t q : a.pt) p->is_free[q] = 0;
      break;
    }
    if (changed) {
      std::vector<uint8_t> bytes(m * p->P);  // the adapter's pages in logical order, then into their new places
      for (size_t l = 0; l < m; ++l) std::memcpy(bytes.data() + l * p->P, p->mem + uint64_t(a.pt[l]) * p->P, p->P);
      for (size_t l = 0; l < m; ++l) std::memcpy(p->mem + uint64_t(to[l]) * p->P, bytes.data() + l * p->P, p->P);
      a.pt = to;
      pages += changed;
      adapters++;
    }
    for (int32_t q : a.pt) p->is_free[q] = 0;
  }
  if (moved_out) { moved_out[0] = pages; moved_out[1] = adapters; }
  return O_OK;
}

int oracle_page_table(void* h, int32_t id, int32_t* out, uint32_t cap, uint32_t* n_out) {
  OPool* p = (OPool*)h;
  if (!p || id < 0 || id >= p->max_adapters) return O_INVAL;
  OAdapter& a = p->ad[id];
  if (!a.present) return O_NOTFOUND;
  if (n_out) *n_out = uint32_t(a.pt.size());
  if (out) std::memcpy(out, a.pt.data(), std::min<size_t>(cap, a.pt.size()) * 4);
  return O_OK;
}

// out[0..7]: n_pages, free pages, used pages, resident adapter bytes, loads, evictions,
// nomem failures, page_bytes.
int oracle_stats(void* h, uint64_t* out) {
  OPool* p = (OPool*)h;
  if (!p || !out) return O_INVAL;
  out[0] = p->n_pages; out[1] = p->n_free; out[2] = p->n_pages - p->n_free;
  out[3] = p->resident_bytes; out[4] = p->loads; out[5] = p->evictions; out[6] = p->nomem; out[7] = p->P;
  return O_OK;
}

int oracle_free_map(void* h, uint8_t* out) {
  OPool* p = (OPool*)h;
  if (!p || !out) return O_INVAL;
  std::memcpy(out, p->is_free.data(), p->n_pages);
  return O_OK;
}

// The "contiguous virtual view": nbytes of adapter id starting at virtual byte `off`.
int oracle_read_virtual(void* h, int32_t id, uint64_t off, uint64_t nbytes, void* out) {
  OPool* p = (OPool*)h;
  if (!p || id < 0 || id >= p->max_adapters || !out) return O_INVAL;
  OAdapter& a = p->ad[id];
  if (!a.present) return O_NOTFOUND;
  uint64_t S = uint64_t(a.rank) * p->elt * uint64_t(p->C);
  if (off + nbytes > S) return O_INVAL;
  for (uint64_t i = 0; i < nbytes; ++i) ((uint8_t*)out)[i] = *vaddr(p, a, off + i);
  return O_OK;
}

// Once-per-batch translation: stable counting sort of token indices by adapter id
// (ascending); tokens with id -1 carry no adapter and are dropped.  perm gets the token
// indices, seg_adapter the distinct ids, seg_start the n_seg+1 boundaries into perm.
// A token naming an adapter that is not resident -> NOTFOUND, nothing written.
int oracle_translate(void* h, const int32_t* tok2adapter, int32_t T, int32_t* perm, int32_t* seg_adapter,
                     int32_t* seg_start, int32_t* n_seg_out, int32_t* n_perm_out) {
  OPool* p = (OPool*)h;
  if (!p || T < 0 || (T > 0 && !tok2adapter)) return O_INVAL;
  std::vector<int32_t> count(p->max_adapters, 0);
  for (int32_t t = 0; t < T; ++t) {
    int32_t i = tok2adapter[t];
    if (i == -1) continue;
    if (i < 0 || i >= p->max_adapters) return O_INVAL;
    if (!p->ad[i].present) return O_NOTFOUND;
    count[i]++;
  }
  std::vector<int32_t> start(p->max_adapters, 0);
  int32_t n_seg = 0, run = 0;
  for (int32_t i = 0; i < p->max_adapters; ++i) {
    start[i] = run;
    if (count[i]) { seg_adapter[n_seg] = i; seg_start[n_seg] = run; n_seg++; run += count[i]; }
  }
  seg_start[n_seg] = run;
  for (int32_t t = 0; t < T; ++t) {
    int32_t i = tok2adapter[t];
    if (i == -1) continue;
    perm[start[i]++] = t;
  }
  *n_seg_out = n_seg; *n_perm_out = run;
  return O_OK;
}

// Shrink, slot s: v[t, j] = sum_k x[t,k] * A_i[j,k] for j < r_i (i = tok2adapter[t]), and 0
// for j >= r_i or i == -1.  x: T x d_in elements; v: T x max_rank, float (acc_mode 0) or
// double (acc_mode 1).  tok_sel (may be null) restricts the work to those token indices.
int oracle_shrink(void* h, int32_t s, const void* x, const int32_t* tok2adapter, int32_t T,
                  const int32_t* tok_sel, int32_t n_sel, int32_t acc_mode, int32_t threads, void* v) {
  OPool* p = (OPool*)h;
  if (!p || s < 0 || s >= p->n_slots || !x || !v || !tok2adapter) return O_INVAL;
  int32_t n = tok_sel ? n_sel : T;
  int bad = 0;
  (void)threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads) if (threads > 1) reduction(| : bad)
  for (int32_t q = 0; q < n; ++q) {
    int32_t t = tok_sel ? tok_sel[q] : q;
    int32_t i = tok2adapter[t];
    if (acc_mode == 0) {
      float* row = (float*)v + uint64_t(t) * p->max_rank;
      for (int j = 0; j < p->max_rank; ++j) row[j] = 0.f;
      if (i == -1) continue;
      if (i < 0 || i >= p->max_adapters || !p->ad[i].present) { bad = 1; continue; }
      shrink_token<float>(p, s, (const uint8_t*)x, t, p->ad[i], row);
    } else {
      double* row = (double*)v + uint64_t(t) * p->max_rank;
      for (int j = 0; j < p->max_rank; ++j) row[j] = 0.0;
      if (i == -1) continue;
      if (i < 0 || i >= p->max_adapters || !p->ad[i].present) { bad = 1; continue; }
      shrink_token<double>(p, s, (const uint8_t*)x, t, p->ad[i], row);
    }
  }
  return bad ? O_NOTFOUND : O_OK;
}

// Expand, slot s: y[t,n] = round_elt( y[t,n] + scale_i * sum_j v[t,j] * B_i[j,n] ), in place.
int oracle_expand(void* h, int32_t s, const void* v, const int32_t* tok2adapter, int32_t T,
                  const int32_t* tok_sel, int32_t n_sel, int32_t acc_mode, int32_t threads, void* y) {
  OPool* p = (OPool*)h;
  if (!p || s < 0 || s >= p->n_slots || !y || !v || !tok2adapter) return O_INVAL;
  int32_t n = tok_sel ? n_sel : T;
  int bad = 0;
  (void)threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads) if (threads > 1) reduction(| : bad)
  for (int32_t q = 0; q < n; ++q) {
    int32_t t = tok_sel ? tok_sel[q] : q;
    int32_t i = tok2adapter[t];
    if (i == -1) continue;
    if (i < 0 || i >= p->max_adapters || !p->ad[i].present) { bad = 1; continue; }
    if (acc_mode == 0) expand_token<float>(p, s, (const float*)v + uint64_t(t) * p->max_rank, (uint8_t*)y, t, p->ad[i]);
    else expand_token<double>(p, s, (const double*)v + uint64_t(t) * p->max_rank, (uint8_t*)y, t, p->ad[i]);
  }
  return bad ? O_NOTFOUND : O_OK;
}

// Element codecs exposed so that tests can pin them against numpy's float16 and a bit-level
// bfloat16 definition.
float oracle_decode_elt(int32_t dtype, uint32_t bits) {
  if (dtype == DT_F32) return bits_to_float(bits);
  return dtype == DT_BF16 ? bf16_to_float(uint16_t(bits)) : f16_to_float(uint16_t(bits));
}
uint32_t oracle_encode_elt(int32_t dtype, float f) {
  if (dtype == DT_F32) return float_to_bits(f);
  return dtype == DT_BF16 ? float_to_bf16_rne(f) : float_to_f16_rne(f);
}

int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

}  // extern "C"
