// Host side of the paged multi-LoRA library: page pool, first-fit allocator, page tables, the
// pinned-host -> GPU copy path and the once-per-batch translation.  See include/plora.h for the
// contract of every entry point (and the passages of the paper each one follows).
#include "../../include/plora.h"
#include "plora_internal.h"

#include <algorithm>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <vector>

using namespace plora;

static thread_local int g_last_hip = 0;

#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) {                             \
      g_last_hip = (int)e_;                             \
      (void)hipGetLastError();                          \
      return PLORA_ERR_HIP;                             \
    }                                                   \
  } while (0)

namespace {

// Completion marker of one or more batches that ended on the same stream.  It is recorded lazily:
// an event recorded later on the stream still implies that the batches' kernels have finished, and
// one record per few batches keeps the extra packet out of most steps' queues.
struct Event {
  hipEvent_t ev = nullptr;
  hipStream_t stream = nullptr;
  bool recorded = false;
  int users = 0;  // batches that ended under this marker so far
  ~Event() { if (ev) (void)hipEventDestroy(ev); }
};

struct Adapter {
  bool present = false;
  int32_t rank = 0;
  float scale = 0.f;
  uint64_t bytes = 0;
  std::vector<int32_t> pt;
  bool contig = false;  // the pages are physically consecutive: kernels derive the table from pt[0]
  hipEvent_t ev_start = nullptr, ev_ready = nullptr;  // created on first use, reused
  bool copy_pending = false;                          // ready event not yet observed complete
  bool moved = false;                                 // the pending copies are a compaction's page moves, not a load
  int pins = 0;
  std::vector<std::shared_ptr<Event>> last_use;  // completion markers of the last batches that read it: one per stream
};

// Work items of one operation in flat storage: the records of group g (one adapter's items that
// share x rows, v rows or a piece of B and should meet in one XCD's L2) are items[first[g] ..
// first[g + 1]).  The vectors live in the pool and keep their capacity from batch to batch.
struct ItemGroups {
  std::vector<ItemRec> items;
  std::vector<uint32_t> first;  // size groups + 1 once closed
  std::vector<double> cost;
  void clear() { items.clear(); first.assign(1, 0); cost.clear(); }
  void close_group(double c) {
    if (items.size() == first.back()) return;  // empty group
    first.push_back((uint32_t)items.size());
    cost.push_back(c);
  }
  size_t groups() const { return cost.size(); }
};

}  // namespace

struct plora_batch {
  plora_pool* pool = nullptr;
  bool open = false;
  bool panel = false;  // expand: the matrix-core blocks go to the panel kernel
  bool full_shrink_tiles = false;  // shrink: the matrix-core items average at least half a token tile
  hipStream_t stream = nullptr;
  int32_t n_tokens = 0, n_seg = 0, n_perm = 0;
  // host copies for plora_batch_info
  std::vector<int32_t> perm, seg_adapter, seg_start;
  // staging (pinned) and device image
  uint8_t* h_img = nullptr;
  uint8_t* d_img = nullptr;
  size_t cap = 0;
  // offsets inside the image
  size_t off_perm = 0, off_pt = 0;
  // state of the one-launch form of plora_delta: counters and flags on the device (zero when allocated,
  // never reset), and the value each slot position's counter will have reached after the launches so far
  uint32_t* d_queue = nullptr;
  mutable uint32_t q_target[kMaxSlotsFused] = {};
  // work lists (blocks of 4 records): [op][layout], op 0 = shrink, 1 = expand; layout 0 = longest
  // first (for launches whose fastest grid dimension is the slot), 1 = dealt into 8 interleaved XCD
  // queues
  // 2 = every group as vector-ALU records, one record per workgroup (cooperative kernels of small calls)
  size_t off_items[2][3] = {{0, 0, 0}, {0, 0, 0}};
  int32_t n_items[2][3] = {{0, 0, 0}, {0, 0, 0}};
  int32_t n_heavy[2] = {0, 0};  // layout 0 only: records of the leading matrix-core blocks
  std::vector<int32_t> adapters;      // pinned adapters
  std::shared_ptr<Event> done;        // recorded by plora_batch_end; the images are reusable once it has passed
  hipEvent_t ev_img = nullptr;        // the image has arrived on the device (recorded on the pool's aux stream)
  // Streams other than `stream` that kernels of this batch were launched on (the caller orders them after
  // `stream`); plora_batch_end makes `stream` wait for each of them, so that the batch's completion marker on
  // `stream` covers their kernels too.  ev_other: one event per entry, kept for reuse.
  mutable std::vector<hipStream_t> other_streams;
  std::vector<hipEvent_t> ev_other;
};

struct plora_pool {
  size_t P = 0;
  int log2P = 0;
  uint32_t n_pages = 0;
  bool placement_only = false;
  int dtype = 0, elt = 2, max_adapters = 0, max_rank = 0, n_slots = 0;
  std::vector<SlotRec> slots;
  int64_t C = 0;
  int max_d_out = 0;
  int min_chunks = 1;  // 512-column chunks (64 lanes x 16 bytes) of the narrowest slot: the fewest workgroups per expand block
  uint8_t* slab = nullptr;
  bool own_slab = false;
  SlotRec* d_slots = nullptr;
  std::vector<uint64_t> free_bits;  // bit set = page free
  uint32_t n_free = 0;
  uint32_t hint_word = 0;  // no free bit below this word
  std::vector<Adapter> ad;
  // Markers of batches that last read pages since freed, each with the copy streams that already wait
  // for it: any stream that copies into free pages has to be ordered after them, until they have passed.
  struct ReuseWait { std::shared_ptr<Event> m; std::vector<hipStream_t> waited; };
  std::vector<ReuseWait> reuse_wait;
  std::shared_ptr<Event> cur_done;                 // marker of the batches ended since the last record
  int cols_max_group = kMfmaColsMaxGroup;          // expand, panel batches: (remainders of) groups of at most this many tokens go as column-split items
  int panel_min_blocks = 8;  // expand: a batch with at least this many 64-token blocks of large groups (prefill) sends its
                             // matrix-core blocks to the panel kernel; other batches cut every large group into
                             // column-split items (0 = never)
  int64_t panel_half_max_workgroups = 8192;  // expand: a panel launch of at most this many workgroups (of 512 columns) is
                                             // issued with one workgroup per 256 columns instead (0 = never)
  int batches_per_marker = 4;                      // record the marker once this many batches share it
  std::vector<plora_batch*> batches;               // all batch objects ever made (recycled)
  int open_batches = 0;
  std::vector<int32_t> count, cursor;              // per-adapter scratch of the counting sort
  // scratch of the work-list construction (capacity kept from batch to batch)
  ItemGroups wl[2][2];                             // [op][0 vector-ALU | 1 matrix-core]
  std::vector<ItemRec> wl_lists[2][3], wl_tg;
  std::vector<uint32_t> wl_bucket;
  std::vector<int32_t> wl_touched;
  // tunables
  // A group of n tokens on a rank-r adapter takes matrix-core items when n >= min_tokens or its work
  // reaches min_work (min_tokens 0 = never).  Shrink: work = n * r.  Expand: work = n * r * (r / r
  // rounded up to 32), the second factor being the used part of the 32-row contraction tile.
  int mfma_min_tokens = 16, mfma_min_tokens_expand = 64;
  int64_t mfma_min_work = 64, mfma_min_work_expand = 128;
  // launch geometry, [shrink, expand]
  int xcd_remap[2] = {1, 0};  // item-fastest launches take the lists dealt into XCD queues
  hipStream_t aux = nullptr;  // pool-owned side stream that carries the batch images
  std::vector<std::pair<int, int>> run_order;  // scratch of a shrink / expand call, n_slots entries (never grows)
  std::vector<float*> static_v;                // scratch of plora_delta_static, n_slots entries (never grows)
  // plora_delta on small calls: one launch whose workgroups take shrink and then expand tasks from a queue
  int64_t fused_max_tasks = 0;        // calls of at most this many workgroup tasks (shrink + expand) take it (0 = never, the
                                      // default: on this GPU two launches are faster at every call size measured)
  int64_t fused_spin_limit = 1 << 20; // polls before an expand task gives up waiting for its slot's shrink tasks
  uint32_t* h_timeouts = nullptr;     // page-locked word the kernel counts given-up tasks in
  uint32_t* d_timeouts = nullptr;     // the same word as the device sees it
  uint64_t fused_launches = 0;
  int contig_fast_path = 1;   // adapters on consecutive pages: their items carry the first page instead of a table offset
  int mfma_shrink_depth = 0;  // runs in flight per matrix-core shrink item: 1, 2, or 0 = by batch and slot shape
  int64_t deep_max_workgroups = 2500;  // shrink launches of at most this many workgroups take the two-runs-in-flight kernel
  int64_t coop_max_workgroups[2] = {192, 2500};  // [shrink, expand]: calls whose ordinary launch would have at
                                                 // most this many workgroups use the cooperative kernels (0 = never)
  int slot_major[2] = {-1, 2}; // -1: slots are the fastest grid dimension when their count is a multiple of 8; 0 never; 1 always;
                               // 2 (expand): the 512-column chunks are the fastest dimension
  // staged loads: two device buffers that take a blob in one copy before a kernel moves it into its pages
  uint64_t staging_cap = 0;       // largest blob that goes staged (0 = loads copy straight into the pages)
  uint64_t stage_bytes = 0;       // bytes allocated per buffer
  int staging_min_runs = 3;       // a placement of at least this many runs of consecutive pages goes staged
  uint8_t* stage[2] = {nullptr, nullptr};
  hipEvent_t stage_free[2] = {nullptr, nullptr};  // recorded after the scatter that last read the buffer
  bool stage_used[2] = {false, false};
  int stage_next = 0;
  uint64_t staged_loads = 0;
  // kernel timing (plora_profile)
  bool profiling = false;
  struct ProfRec { int cls; hipEvent_t e0, e1; };
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> prof_free;
  // statistics
  uint64_t resident_adapters = 0, resident_bytes = 0, loads = 0, evictions = 0, nomem = 0;
  uint64_t h2d_bytes = 0, h2d_copies = 0;
  double h2d_ms = 0.0;
  uint64_t compactions = 0, compacted_pages = 0;  // adapters / pages moved by plora_compact
  double compact_ms = 0.0;
  std::vector<int32_t> compact_order, compact_to;  // scratch of plora_compact
};

namespace {

// Harvest the copy time of a finished load.  Returns 1 ready, 0 pending, <0 error.
int poll_ready(plora_pool* p, Adapter& a) {
  if (!a.copy_pending) return 1;
  hipError_t e = hipEventQuery(a.ev_ready);
  if (e == hipErrorNotReady) { (void)hipGetLastError(); return 0; }
  if (e != hipSuccess) { g_last_hip = (int)e; (void)hipGetLastError(); return PLORA_ERR_HIP; }
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, a.ev_start, a.ev_ready) == hipSuccess) (a.moved ? p->compact_ms : p->h2d_ms) += ms;
  else (void)hipGetLastError();
  a.copy_pending = false;
  a.moved = false;
  return 1;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Records the marker on its stream if that has not happened yet.
int record_now(Event& e) {
  if (e.recorded) return PLORA_OK;
  if (!e.ev) HIP_TRY(hipEventCreateWithFlags(&e.ev, hipEventDisableTiming));
  HIP_TRY(hipEventRecord(e.ev, e.stream));
  e.recorded = true;
  return PLORA_OK;
}

// 1 = the marker has passed, 0 = not yet (it is recorded first if need be), < 0 = error.
int marker_passed(Event& e) {
  const int rc = record_now(e);
  if (rc != PLORA_OK) return rc;
  const hipError_t q = hipEventQuery(e.ev);
  if (q == hipSuccess) return 1;
  (void)hipGetLastError();
  if (q == hipErrorNotReady) return 0;
  g_last_hip = (int)q;
  return PLORA_ERR_HIP;
}

// Appends the records idx[0 .. n) of `src`, longest first: a stable counting sort by rank,
// descending (equal ranks keep their order, so the token groups of one adapter stay neighbours).
void append_by_rank(const std::vector<ItemRec>& src, const uint32_t* idx, size_t n, std::vector<ItemRec>& out,
                    std::vector<uint32_t>& bucket) {
  bucket.assign(kMaxRank + 2, 0);
  for (size_t i = 0; i < n; ++i) bucket[kMaxRank - src[idx ? idx[i] : i].rank + 1]++;
  for (int r = 0; r <= kMaxRank; ++r) bucket[r + 1] += bucket[r];
  const size_t base = out.size();
  out.resize(base + n);
  for (size_t i = 0; i < n; ++i) {
    const ItemRec& it = src[idx ? idx[i] : i];
    out[base + bucket[kMaxRank - it.rank]++] = it;
  }
}

// Work list of a kernel: blocks of 4 records, one 256-thread workgroup each.  Workgroup i of a launch
// runs on XCD i % 8.  A matrix-core item fills a block alone (3 padding records); vector-ALU items go
// four to a block, one per wavefront: the 4 wavefronts of a block hold their workgroup's resources
// until the last one ends, so items of similar length (rank) are put together, longest first.
// Matrix-core blocks first (their dependent chains are the long ones).  With xcd_aware the groups
// are dealt into 8 queues (longest first, each to the least loaded queue) and the queues are
// interleaved block by block; queues that run out are padded with empty blocks.
void arrange_blocks(const ItemGroups& heavy, const ItemGroups& light, bool xcd_aware, std::vector<ItemRec>& out,
                    std::vector<uint32_t>& bucket, int32_t* n_heavy_records = nullptr) {
  out.clear();
  ItemRec pad{};
  pad.kind = -1;
  if (!xcd_aware) {
    out.reserve(4 * heavy.items.size() + light.items.size() + 4);
    for (const ItemRec& it : heavy.items) { out.push_back(it); out.insert(out.end(), 3, pad); }
    append_by_rank(light.items, nullptr, light.items.size(), out, bucket);
    while (out.size() % 4) out.push_back(pad);
    if (n_heavy_records) *n_heavy_records = (int32_t)(4 * heavy.items.size());
    return;
  }
  if (n_heavy_records) *n_heavy_records = 0;
  constexpr int nq = kXcds;
  std::vector<uint32_t> qh[nq], ql[nq];  // record indices per queue
  double load[nq] = {0, 0, 0, 0, 0, 0, 0, 0};
  std::vector<uint32_t> order;
  auto deal = [&](const ItemGroups& g, std::vector<uint32_t>* dst) {
    order.resize(g.groups());
    for (size_t i = 0; i < order.size(); ++i) order[i] = (uint32_t)i;
    std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) { return g.cost[x] > g.cost[y]; });
    for (uint32_t gi : order) {
      int best = 0;
      for (int k = 1; k < nq; ++k) if (load[k] < load[best]) best = k;
      for (uint32_t i = g.first[gi]; i < g.first[gi + 1]; ++i) dst[best].push_back(i);
      load[best] += g.cost[gi];
    }
  };
  deal(heavy, qh);
  deal(light, ql);
  std::vector<ItemRec> blocks[nq];  // per queue, 4 records per block
  size_t longest = 0;
  for (int k = 0; k < nq; ++k) {
    blocks[k].reserve(4 * qh[k].size() + ql[k].size() + 4);
    for (uint32_t i : qh[k]) { blocks[k].push_back(heavy.items[i]); blocks[k].insert(blocks[k].end(), 3, pad); }
    append_by_rank(light.items, ql[k].data(), ql[k].size(), blocks[k], bucket);
    while (blocks[k].size() % 4) blocks[k].push_back(pad);
    longest = std::max(longest, blocks[k].size() / 4);
  }
  out.reserve(longest * 4 * nq);
  for (size_t i = 0; i < longest; ++i)
    for (int k = 0; k < nq; ++k)
      for (int w = 0; w < 4; ++w) out.push_back(4 * i + w < blocks[k].size() ? blocks[k][4 * i + w] : pad);
}

}  // namespace

// Copies into reused pages must not overtake kernels of batches that read them: `st` is made to wait
// for every listed marker that has not passed yet (once per stream and marker).
static int wait_for_earlier_readers(plora_pool* p, hipStream_t st) {
  for (size_t k = 0; k < p->reuse_wait.size();) {
    auto& w = p->reuse_wait[k];
    const int passed = marker_passed(*w.m);
    if (passed < 0) return passed;
    if (passed) { p->reuse_wait.erase(p->reuse_wait.begin() + k); continue; }
    if (std::find(w.waited.begin(), w.waited.end(), st) == w.waited.end()) {
      HIP_TRY(hipStreamWaitEvent(st, w.m->ev, 0));
      w.waited.push_back(st);
    }
    ++k;
  }
  return PLORA_OK;
}

extern "C" {

int plora_version(void) { return 100; }
int plora_last_hip(void) { return g_last_hip; }

int plora_pool_create(size_t page_bytes, uint32_t n_pages, const plora_layout* lay, void* slab_or_null, uint32_t flags,
                      plora_pool** out) {
  if (!out || !lay || !lay->d_in || !lay->d_out) return PLORA_ERR_INVAL;
  if (page_bytes < 4096 || page_bytes > ((size_t)1 << 30) || (page_bytes & (page_bytes - 1))) return PLORA_ERR_INVAL;
  if (n_pages == 0 || n_pages > 0x7fffffffu) return PLORA_ERR_INVAL;
  if (lay->n_slots < 1 || lay->n_slots > 32767 || lay->dtype < 0 || lay->dtype > 2 || lay->max_adapters < 1) return PLORA_ERR_INVAL;
  if (lay->max_rank < 1 || lay->max_rank > kMaxRank) return PLORA_ERR_INVAL;
  if (flags & ~PLORA_POOL_PLACEMENT_ONLY) return PLORA_ERR_INVAL;
  if (slab_or_null && ((uintptr_t)slab_or_null & 255)) return PLORA_ERR_INVAL;
  const int elt = lay->dtype == PLORA_F32 ? 4 : 2;
  int64_t c = 0;
  int max_in = 0, max_out = 0, min_out = 1 << 30;
  std::vector<SlotRec> slots;
  for (int s = 0; s < lay->n_slots; ++s) {
    const int32_t di = lay->d_in[s], dn = lay->d_out[s];
    if (di <= 0 || dn <= 0 || di % 8 || dn % 8) return PLORA_ERR_INVAL;
    slots.push_back(SlotRec{di, dn, c});
    c += (int64_t)di + dn;
    max_in = std::max(max_in, di);
    max_out = std::max(max_out, dn);
    min_out = std::min(min_out, dn);
  }
  // page-table windows staged in LDS: 32 rows per matrix-core item (kPtWindow entries), 8 rows per
  // vector-ALU item (a quarter of that)
  static_assert(kMfmaRows == 4 * kShrinkRows, "window budget assumes 32 and 8 rows");
  if ((uint64_t)kMfmaRows * (uint64_t)max_in * elt / page_bytes + 8 > (uint64_t)kPtWindow) return PLORA_ERR_INVAL;

  plora_pool* p = new (std::nothrow) plora_pool;
  if (!p) return PLORA_ERR_NOMEM;
  p->P = page_bytes;
  while (((size_t)1 << p->log2P) < page_bytes) p->log2P++;
  p->n_pages = n_pages;
  p->placement_only = (flags & PLORA_POOL_PLACEMENT_ONLY) != 0;
  p->dtype = lay->dtype; p->elt = elt; p->max_adapters = lay->max_adapters; p->max_rank = lay->max_rank;
  p->n_slots = lay->n_slots; p->slots = slots; p->C = c; p->max_d_out = max_out;
  p->min_chunks = (min_out + kWave * (16 / elt) - 1) / (kWave * (16 / elt));
  p->free_bits.assign(((size_t)n_pages + 63) / 64, ~(uint64_t)0);
  if (n_pages & 63) p->free_bits.back() = (((uint64_t)1 << (n_pages & 63)) - 1);
  p->n_free = n_pages;
  p->ad.resize(lay->max_adapters);
  p->run_order.resize(lay->n_slots);
  p->static_v.resize(lay->n_slots);
  p->count.assign(lay->max_adapters, 0);
  p->cursor.assign(lay->max_adapters, 0);
  if (!p->placement_only) {
    hipError_t e = hipSuccess;
    if (slab_or_null) p->slab = (uint8_t*)slab_or_null;
    else { e = hipMalloc((void**)&p->slab, (size_t)n_pages * page_bytes); p->own_slab = (e == hipSuccess); }
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_slots, sizeof(SlotRec) * slots.size());
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&p->aux, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipMemcpy(p->d_slots, slots.data(), sizeof(SlotRec) * slots.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipHostMalloc((void**)&p->h_timeouts, 256, hipHostMallocDefault);
    if (e == hipSuccess) {
      *p->h_timeouts = 0;
      e = hipHostGetDevicePointer((void**)&p->d_timeouts, p->h_timeouts, 0);
    }
    if (e != hipSuccess) {
      g_last_hip = (int)e; (void)hipGetLastError();
      if (p->own_slab) (void)hipFree(p->slab);
      if (p->d_slots) (void)hipFree(p->d_slots);
      if (p->h_timeouts) (void)hipHostFree(p->h_timeouts);
      if (p->aux) (void)hipStreamDestroy(p->aux);
      delete p;
      return PLORA_ERR_HIP;
    }
  }
  *out = p;
  return PLORA_OK;
}

int plora_pool_destroy(plora_pool* p) {
  if (!p) return PLORA_ERR_INVAL;
  if (p->open_batches) return PLORA_ERR_BUSY;
  if (!p->placement_only) {
    (void)hipDeviceSynchronize();
    for (auto& a : p->ad) {
      if (a.ev_start) (void)hipEventDestroy(a.ev_start);
      if (a.ev_ready) (void)hipEventDestroy(a.ev_ready);
    }
    if (p->own_slab) (void)hipFree(p->slab);
    if (p->d_slots) (void)hipFree(p->d_slots);
    if (p->h_timeouts) (void)hipHostFree(p->h_timeouts);
    if (p->aux) (void)hipStreamDestroy(p->aux);
    for (auto& r : p->prof) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
    for (hipEvent_t e : p->prof_free) (void)hipEventDestroy(e);
  }
  for (int i = 0; i < 2; ++i) {
    if (p->stage[i]) (void)hipFree(p->stage[i]);
    if (p->stage_free[i]) (void)hipEventDestroy(p->stage_free[i]);
  }
  for (plora_batch* b : p->batches) {
    if (b->h_img) { if (p->placement_only) ::operator delete(b->h_img); else (void)hipHostFree(b->h_img); }
    if (b->d_img) (void)hipFree(b->d_img);
    if (b->d_queue) (void)hipFree(b->d_queue);
    if (b->ev_img) (void)hipEventDestroy(b->ev_img);
    for (hipEvent_t e : b->ev_other) (void)hipEventDestroy(e);
    delete b;
  }
  delete p;
  return PLORA_OK;
}

uint64_t plora_adapter_bytes(const plora_pool* p, int32_t rank) {
  if (!p || rank < 1 || rank > p->max_rank) return 0;
  return (uint64_t)rank * p->elt * (uint64_t)p->C;
}

int plora_load_adapter(plora_pool* p, int32_t id, int32_t rank, float scale, const void* host, plora_stream cs,
                       const int32_t** pt_out, uint32_t* n_out) {
  if (!p || id < 0 || id >= p->max_adapters || rank < 1 || rank > p->max_rank) return PLORA_ERR_INVAL;
  if (!p->placement_only && !host) return PLORA_ERR_INVAL;
  Adapter& a = p->ad[id];
  if (a.present) return PLORA_ERR_EXISTS;
  const uint64_t S = (uint64_t)rank * p->elt * (uint64_t)p->C;
  const uint64_t m = (S + p->P - 1) / p->P;
  if (m > p->n_free) { p->nomem++; return PLORA_ERR_NOMEM; }
  hipStream_t st = (hipStream_t)cs;
  if (!p->placement_only) {
    hipPointerAttribute_t at;
    hipError_t e = hipPointerGetAttributes(&at, host);
    if (e != hipSuccess || at.type != hipMemoryTypeHost) { (void)hipGetLastError(); return PLORA_ERR_INVAL; }
    if (!a.ev_start) {
      HIP_TRY(hipEventCreate(&a.ev_start));
      HIP_TRY(hipEventCreate(&a.ev_ready));
    }
  }
  // first fit: the m lowest-numbered free pages, ascending
  a.pt.clear();
  a.pt.reserve(m);
  uint32_t w = p->hint_word;
  while (a.pt.size() < m) {
    uint64_t bits = p->free_bits[w];
    while (bits && a.pt.size() < m) {
      const int b = __builtin_ctzll(bits);
      bits &= bits - 1;
      a.pt.push_back((int32_t)(w * 64 + b));
    }
    p->free_bits[w] = bits;  // taken bits cleared; if we stopped early, the rest stay set
    if (a.pt.size() < m) ++w;
  }
  // restore bits of word w that were cleared in `bits` but not taken: none (we clear only taken ones)
  while (p->hint_word < p->free_bits.size() && p->free_bits[p->hint_word] == 0) p->hint_word++;
  p->n_free -= (uint32_t)m;

  if (!p->placement_only) {
    uint64_t runs = 1;
    for (uint64_t l = 1; l < m; ++l) runs += a.pt[l] != a.pt[l - 1] + 1;
    const bool staged = p->staging_cap >= S && runs >= (uint64_t)p->staging_min_runs;
    hipError_t e = hipSuccess;
    int rc = PLORA_OK;
    if (staged) {
      // one copy into a staging buffer (it may run while earlier readers of the freed pages still do),
      // then a kernel that moves the pages into place
      const int k = p->stage_next;
      p->stage_next ^= 1;
      if (p->stage_used[k]) e = hipStreamWaitEvent(st, p->stage_free[k], 0);
      if (e == hipSuccess) e = hipEventRecord(a.ev_start, st);
      if (e == hipSuccess) e = hipMemcpyAsync(p->stage[k], host, S, hipMemcpyHostToDevice, st);
      p->h2d_copies++;
      if (e == hipSuccess) rc = wait_for_earlier_readers(p, st);
      if (e == hipSuccess && rc == PLORA_OK) e = launch_scatter(p->stage[k], p->slab, p->log2P, S, a.pt.data(), (uint32_t)m, st);
      if (e == hipSuccess && rc == PLORA_OK) {
        e = hipEventRecord(p->stage_free[k], st);
        p->stage_used[k] = true;
      }
    } else {
      rc = wait_for_earlier_readers(p, st);
      if (rc == PLORA_OK) e = hipEventRecord(a.ev_start, st);
      uint64_t l = 0;
      while (rc == PLORA_OK && e == hipSuccess && l < m) {  // one copy per run of consecutive physical pages
        uint64_t h = l + 1;
        while (h < m && a.pt[h] == a.pt[h - 1] + 1) ++h;
        const uint64_t lo = l * p->P, hi = std::min<uint64_t>(h * p->P, S);
        e = hipMemcpyAsync(p->slab + (uint64_t)a.pt[l] * p->P, (const uint8_t*)host + lo, hi - lo, hipMemcpyHostToDevice, st);
        p->h2d_copies++;
        l = h;
      }
    }
    if (e == hipSuccess && rc == PLORA_OK) e = hipEventRecord(a.ev_ready, st);
    if (e != hipSuccess || rc != PLORA_OK) {  // undo the placement
      if (e != hipSuccess) { g_last_hip = (int)e; (void)hipGetLastError(); rc = PLORA_ERR_HIP; }
      // Copies (or the scatter kernel) already queued on the stream still write into these pages or read
      // the staging buffer: let them finish before the pages are handed out again.  A rare path, so the
      // host simply waits.
      (void)hipStreamSynchronize(st);
      (void)hipGetLastError();
      if (staged) p->stage_next ^= 1;  // the buffer was not used after all (and is idle now)
      for (int32_t q : a.pt) p->free_bits[q >> 6] |= (uint64_t)1 << (q & 63);
      p->n_free += (uint32_t)m;
      p->hint_word = std::min<uint32_t>(p->hint_word, a.pt.empty() ? p->hint_word : (uint32_t)a.pt[0] >> 6);
      a.pt.clear();
      return rc;
    }
    if (staged) p->staged_loads++;
    a.copy_pending = true;
    p->h2d_bytes += S;
  }
  a.present = true; a.rank = rank; a.scale = scale; a.bytes = S; a.pins = 0; a.last_use.clear();
  a.contig = p->contig_fast_path && a.pt.back() - a.pt.front() + 1 == (int32_t)a.pt.size();
  p->loads++; p->resident_adapters++; p->resident_bytes += S;
  if (pt_out) *pt_out = a.pt.data();
  if (n_out) *n_out = (uint32_t)m;
  return PLORA_OK;
}

int plora_adapter_ready(plora_pool* p, int32_t id) {
  if (!p || id < 0 || id >= p->max_adapters) return PLORA_ERR_INVAL;
  Adapter& a = p->ad[id];
  if (!a.present) return PLORA_ERR_NOTFOUND;
  if (p->placement_only) return 1;
  return poll_ready(p, a);
}

int plora_wait_adapter(plora_pool* p, int32_t id, plora_stream s) {
  if (!p || id < 0 || id >= p->max_adapters) return PLORA_ERR_INVAL;
  Adapter& a = p->ad[id];
  if (!a.present) return PLORA_ERR_NOTFOUND;
  if (p->placement_only || !a.copy_pending) return PLORA_OK;
  HIP_TRY(hipStreamWaitEvent((hipStream_t)s, a.ev_ready, 0));
  return PLORA_OK;
}

int plora_sync_adapter(plora_pool* p, int32_t id) {
  if (!p || id < 0 || id >= p->max_adapters) return PLORA_ERR_INVAL;
  Adapter& a = p->ad[id];
  if (!a.present) return PLORA_ERR_NOTFOUND;
  if (p->placement_only || !a.copy_pending) return PLORA_OK;
  HIP_TRY(hipEventSynchronize(a.ev_ready));
  const int rdy = poll_ready(p, a);
  return rdy < 0 ? rdy : PLORA_OK;
}

int plora_evict(plora_pool* p, int32_t id) {
  if (!p || id < 0 || id >= p->max_adapters) return PLORA_ERR_INVAL;
  Adapter& a = p->ad[id];
  if (!a.present) return PLORA_ERR_NOTFOUND;
  if (a.pins > 0) return PLORA_ERR_BUSY;
  if (!p->placement_only) {
    const int rdy = poll_ready(p, a);
    if (rdy < 0) return rdy;
    if (rdy == 0) return PLORA_ERR_BUSY;
    for (auto& m : a.last_use) {
      const int passed = marker_passed(*m);
      if (passed < 0) return passed;
      if (passed == 0 && std::none_of(p->reuse_wait.begin(), p->reuse_wait.end(),
                                      [&](const plora_pool::ReuseWait& w) { return w.m == m; }))
        p->reuse_wait.push_back({m, {}});
    }
  }
  for (int32_t q : a.pt) p->free_bits[q >> 6] |= (uint64_t)1 << (q & 63);
  p->n_free += (uint32_t)a.pt.size();
  if (!a.pt.empty()) p->hint_word = std::min<uint32_t>(p->hint_word, (uint32_t)a.pt[0] >> 6);
  p->resident_adapters--; p->resident_bytes -= a.bytes; p->evictions++;
  a.pt.clear(); a.pt.shrink_to_fit();
  a.present = false; a.rank = 0; a.scale = 0.f; a.bytes = 0; a.last_use.clear();
  return PLORA_OK;
}

int plora_adapter_pages(plora_pool* p, int32_t id, const int32_t** pt_out, uint32_t* n_out) {
  if (!p || id < 0 || id >= p->max_adapters) return PLORA_ERR_INVAL;
  Adapter& a = p->ad[id];
  if (!a.present) return PLORA_ERR_NOTFOUND;
  if (pt_out) *pt_out = a.pt.data();
  if (n_out) *n_out = (uint32_t)a.pt.size();
  return PLORA_OK;
}

int plora_compact(plora_pool* p, plora_stream cs, uint32_t max_pages, uint32_t* pages_out, uint32_t* adapters_out) {
  if (!p) return PLORA_ERR_INVAL;
  if (pages_out) *pages_out = 0;
  if (adapters_out) *adapters_out = 0;
  hipStream_t st = (hipStream_t)cs;
  // candidates in ascending order of their first page; adapters that an open batch names (its image
  // carries their tables) or whose pages are still being written stay where they are
  std::vector<int32_t>& order = p->compact_order;
  order.clear();
  for (int32_t id = 0; id < p->max_adapters; ++id) {
    Adapter& a = p->ad[id];
    if (!a.present || a.pins > 0) continue;
    if (!p->placement_only) {
      const int rdy = poll_ready(p, a);
      if (rdy < 0) return rdy;
      if (rdy == 0) continue;
    }
    order.push_back(id);
  }
  std::sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return p->ad[x].pt[0] < p->ad[y].pt[0]; });
  uint32_t pages = 0, adapters = 0;
  std::vector<int32_t>& to = p->compact_to;
  for (int32_t id : order) {
    Adapter& a = p->ad[id];
    const size_t m = a.pt.size();
    // where a load would put it if its own pages were free as well: the m lowest of both
    for (int32_t q : a.pt) p->free_bits[q >> 6] |= (uint64_t)1 << (q & 63);
    to.clear();
    for (uint32_t w = std::min<uint32_t>(p->hint_word, (uint32_t)a.pt[0] >> 6); to.size() < m; ++w) {
      uint64_t bits = p->free_bits[w];
      while (bits && to.size() < m) {
        to.push_back((int32_t)(w * 64 + __builtin_ctzll(bits)));
        bits &= bits - 1;
      }
    }
    uint32_t changed = 0;
    for (size_t l = 0; l < m; ++l) changed += to[l] != a.pt[l];
    if (changed == 0 || (max_pages > 0 && pages + changed > max_pages)) {
      for (int32_t q : a.pt) p->free_bits[q >> 6] &= ~((uint64_t)1 << (q & 63));
      if (changed) break;  // does not fit the bound: it stays, and the call ends
      continue;
    }
    if (!p->placement_only) {
      // The moves write free pages (which batches still in flight may be reading through evicted
      // adapters' tables) and pages of this adapter itself (which batches in flight read through its
      // old table): the stream waits for all of those readers first.
      int rc = wait_for_earlier_readers(p, st);
      hipError_t e = hipSuccess;
      for (auto& mk : a.last_use) {
        if (rc != PLORA_OK || e != hipSuccess) break;
        const int passed = marker_passed(*mk);
        if (passed < 0) rc = passed;
        else if (passed == 0) e = hipStreamWaitEvent(st, mk->ev, 0);
      }
      if (rc == PLORA_OK && e == hipSuccess && !a.ev_start) {
        e = hipEventCreate(&a.ev_start);
        if (e == hipSuccess) e = hipEventCreate(&a.ev_ready);
      }
      if (rc == PLORA_OK && e == hipSuccess) e = hipEventRecord(a.ev_start, st);
      // Page l goes from pt[l] down to to[l] <= pt[l], in ascending l: a page is overwritten only after it
      // has been copied (to[l] <= pt[l] < pt[l + 1]).  Runs of consecutive pages go in one copy, cut so
      // that a copy's source and destination do not overlap.
      size_t l = 0;
      while (rc == PLORA_OK && e == hipSuccess && l < m) {
        if (to[l] == a.pt[l]) { ++l; continue; }
        const size_t gap = (size_t)(a.pt[l] - to[l]);
        size_t h = l + 1;
        while (h < m && h - l < gap && to[h] == to[h - 1] + 1 && a.pt[h] == a.pt[h - 1] + 1) ++h;
        e = hipMemcpyAsync(p->slab + (uint64_t)to[l] * p->P, p->slab + (uint64_t)a.pt[l] * p->P, (h - l) * p->P,
                           hipMemcpyDeviceToDevice, st);
        l = h;
      }
      if (rc == PLORA_OK && e == hipSuccess) e = hipEventRecord(a.ev_ready, st);
      // The pages it leaves are free from now on, but whoever writes them next has to wait for these
      // copies (they read them) and for the batches in flight that read them through the old table.
      std::shared_ptr<Event> done;
      if (rc == PLORA_OK && e == hipSuccess) {
        done = std::make_shared<Event>();
        done->stream = st;
        rc = record_now(*done);
      }
      if (rc != PLORA_OK || e != hipSuccess) {
        // Some pages may already have been overwritten on the way: the adapter is in neither place as a
        // whole.  It leaves the pool (the caller loads it again); both sets of pages become free once the
        // stream has drained.  A failing copy call is not expected outside a broken runtime.
        if (e != hipSuccess) { g_last_hip = (int)e; (void)hipGetLastError(); rc = PLORA_ERR_HIP; }
        (void)hipStreamSynchronize(st);
        (void)hipGetLastError();
        for (int32_t q : to) p->free_bits[q >> 6] |= (uint64_t)1 << (q & 63);
        p->n_free += (uint32_t)m;
        p->hint_word = std::min<uint32_t>(p->hint_word, (uint32_t)to[0] >> 6);
        p->resident_adapters--; p->resident_bytes -= a.bytes; p->evictions++;
        a.pt.clear();
        a.present = false; a.rank = 0; a.scale = 0.f; a.bytes = 0; a.last_use.clear();
        if (pages_out) *pages_out = pages;
        if (adapters_out) *adapters_out = adapters;
        return rc;
      }
      for (auto& mk : a.last_use)
        if (!mk->recorded || hipEventQuery(mk->ev) != hipSuccess) {
          (void)hipGetLastError();
          if (std::none_of(p->reuse_wait.begin(), p->reuse_wait.end(), [&](const plora_pool::ReuseWait& w) { return w.m == mk; }))
            p->reuse_wait.push_back({mk, {st}});
        }
      p->reuse_wait.push_back({done, {st}});
      a.last_use.clear();  // readers of the old pages; whatever reads the new ones comes after ev_ready
      a.copy_pending = true;
      a.moved = true;
    }
    for (int32_t q : to) p->free_bits[q >> 6] &= ~((uint64_t)1 << (q & 63));
    a.pt.assign(to.begin(), to.end());
    a.contig = p->contig_fast_path && a.pt.back() - a.pt.front() + 1 == (int32_t)a.pt.size();
    p->hint_word = 0;
    while (p->hint_word < p->free_bits.size() && p->free_bits[p->hint_word] == 0) p->hint_word++;
    pages += changed;
    adapters++;
  }
  p->compactions += adapters;
  p->compacted_pages += pages;
  if (pages_out) *pages_out = pages;
  if (adapters_out) *adapters_out = adapters;
  return PLORA_OK;
}

int plora_pool_stats(plora_pool* p, plora_stats* o) {
  if (!p || !o) return PLORA_ERR_INVAL;
  if (!p->placement_only)
    for (auto& a : p->ad)
      if (a.present && a.copy_pending) (void)poll_ready(p, a);
  o->page_bytes = p->P; o->n_pages = p->n_pages; o->free_pages = p->n_free; o->used_pages = p->n_pages - p->n_free;
  o->resident_adapters = p->resident_adapters; o->resident_bytes = p->resident_bytes;
  o->internal_frag_bytes = o->used_pages * p->P - p->resident_bytes;
  o->loads = p->loads; o->evictions = p->evictions; o->nomem_failures = p->nomem;
  o->h2d_bytes = p->h2d_bytes; o->h2d_copies = p->h2d_copies; o->h2d_ms = p->h2d_ms; o->staged_loads = p->staged_loads;
  o->fused_launches = p->fused_launches;
  o->compacted_adapters = p->compactions; o->compacted_pages = p->compacted_pages; o->compact_ms = p->compact_ms;
  o->fused_timeouts = p->h_timeouts ? *(volatile uint32_t*)p->h_timeouts : 0;
  return PLORA_OK;
}

int plora_pool_set_option(plora_pool* p, const char* key, int64_t value) {
  if (!p || !key) return PLORA_ERR_INVAL;
  const std::string k(key);
  if (k == "mfma_min_tokens" || k == "mfma_min_tokens_expand") {
    if (value < 0 || value > (1 << 30)) return PLORA_ERR_INVAL;
    (k == "mfma_min_tokens" ? p->mfma_min_tokens : p->mfma_min_tokens_expand) = (int)value;
    return PLORA_OK;
  }
  if (k == "mfma_min_work" || k == "mfma_min_work_expand") {
    if (value < 1 || value > (1 << 30)) return PLORA_ERR_INVAL;
    (k == "mfma_min_work" ? p->mfma_min_work : p->mfma_min_work_expand) = value;
    return PLORA_OK;
  }
  if (k == "staging_min_runs") {
    if (value < 1 || value > (1 << 30)) return PLORA_ERR_INVAL;
    p->staging_min_runs = (int)value;
    return PLORA_OK;
  }
  if (k == "staging_bytes") {
    if (value < 0 || value > ((int64_t)1 << 36) || p->placement_only) return PLORA_ERR_INVAL;
    if (value == 0) { p->staging_cap = 0; return PLORA_OK; }  // the buffers stay: copies may be in flight
    const uint64_t want = align_up((uint64_t)value, 256);
    uint64_t have = 0;
    if (p->stage[0] && p->stage[1]) have = p->stage_bytes;
    if (want > have) {
      HIP_TRY(hipDeviceSynchronize());
      for (int i = 0; i < 2; ++i) {
        if (p->stage[i]) { HIP_TRY(hipFree(p->stage[i])); p->stage[i] = nullptr; }
        p->stage_used[i] = false;
      }
      p->staging_cap = 0;
      p->stage_bytes = 0;
      for (int i = 0; i < 2; ++i) {
        HIP_TRY(hipMalloc((void**)&p->stage[i], want));
        if (!p->stage_free[i]) HIP_TRY(hipEventCreateWithFlags(&p->stage_free[i], hipEventDisableTiming));
      }
      p->stage_bytes = want;
    }
    p->staging_cap = (uint64_t)value;
    return PLORA_OK;
  }
  if (k == "panel_min_blocks") {
    if (value < 0 || value > (1 << 30)) return PLORA_ERR_INVAL;
    p->panel_min_blocks = (int)value;
    return PLORA_OK;
  }
  if (k == "panel_half_max_workgroups") {
    if (value < 0 || value > ((int64_t)1 << 40)) return PLORA_ERR_INVAL;
    p->panel_half_max_workgroups = value;
    return PLORA_OK;
  }
  if (k == "mfma_cols_max_group") {
    if (value < 0 || value > (1 << 30)) return PLORA_ERR_INVAL;
    p->cols_max_group = (int)value;
    return PLORA_OK;
  }
  if (k == "fused_max_tasks") {
    if (value < 0 || value > (1 << 30)) return PLORA_ERR_INVAL;
    p->fused_max_tasks = value;
    return PLORA_OK;
  }
  if (k == "fused_spin_limit") {
    if (value < 0 || value > ((int64_t)1 << 31)) return PLORA_ERR_INVAL;
    p->fused_spin_limit = value;
    return PLORA_OK;
  }
  if (k == "contig_fast_path") {
    if (value != 0 && value != 1) return PLORA_ERR_INVAL;
    p->contig_fast_path = (int)value;
    return PLORA_OK;
  }
  if (k == "mfma_shrink_depth") {
    if (value < 0 || value > 2) return PLORA_ERR_INVAL;
    p->mfma_shrink_depth = (int)value;
    return PLORA_OK;
  }
  if (k == "batches_per_marker") {
    if (value < 1 || value > 64) return PLORA_ERR_INVAL;
    p->batches_per_marker = (int)value;
    return PLORA_OK;
  }
  if (k == "coop_max_workgroups_shrink" || k == "coop_max_workgroups_expand") {
    if (value < 0 || value > (1 << 30)) return PLORA_ERR_INVAL;
    p->coop_max_workgroups[k == "coop_max_workgroups_expand"] = value;
    return PLORA_OK;
  }
  if (k == "xcd_remap" || k == "xcd_remap_shrink" || k == "xcd_remap_expand") {
    if (value != 0 && value != 1) return PLORA_ERR_INVAL;
    if (k != "xcd_remap_expand") p->xcd_remap[0] = (int)value;
    if (k != "xcd_remap_shrink") p->xcd_remap[1] = (int)value;
    return PLORA_OK;
  }
  if (k == "slot_major" || k == "slot_major_shrink" || k == "slot_major_expand") {
    if (value < -1 || value > (k == "slot_major_expand" ? 2 : 1)) return PLORA_ERR_INVAL;  // 2: chunks fastest
    if (k != "slot_major_expand") p->slot_major[0] = (int)value;
    if (k != "slot_major_shrink") p->slot_major[1] = (int)value;
    return PLORA_OK;
  }
  return PLORA_ERR_INVAL;
}

// ---------------------------------------------------------------------------------------------
// batch translation
// ---------------------------------------------------------------------------------------------
int plora_batch_begin(plora_pool* p, const int32_t* t2a, int32_t T, plora_stream s, plora_batch** out) {
  if (!p || !out || T < 0 || (T > 0 && !t2a)) return PLORA_ERR_INVAL;
  // pass 1: validate and count (nothing is modified on failure except the scratch counters)
  int rc = PLORA_OK;
  int32_t n_none = 0;
  std::vector<int32_t> touched;
  for (int32_t t = 0; t < T; ++t) {
    const int32_t i = t2a[t];
    if (i == -1) { n_none++; continue; }
    if (i < 0 || i >= p->max_adapters) { rc = PLORA_ERR_INVAL; break; }
    if (!p->ad[i].present) { rc = PLORA_ERR_NOTFOUND; break; }
    if (p->count[i]++ == 0) touched.push_back(i);
  }
  if (rc != PLORA_OK) {
    for (int32_t i : touched) p->count[i] = 0;
    return rc;
  }
  std::sort(touched.begin(), touched.end());
  const int32_t n_seg = (int32_t)touched.size();
  const int32_t n_perm = T - n_none;

  plora_batch* b = nullptr;
  bool unrecorded = false;
  for (plora_batch* c : p->batches) {
    if (c->open) continue;
    if (c->done) {  // its last copy and kernels may still be in flight
      if (!c->done->recorded) { unrecorded = true; continue; }
      if (marker_passed(*c->done) != 1) continue;
      c->done.reset();
    }
    b = c;
    break;
  }
  if (!b) {
    // nothing to recycle: make sure the closed batches' marker is on its way, and take a new object
    if (unrecorded && p->cur_done) (void)record_now(*p->cur_done);
    b = new (std::nothrow) plora_batch;
    if (!b) { for (int32_t i : touched) p->count[i] = 0; return PLORA_ERR_NOMEM; }
    b->pool = p;
    b->other_streams.reserve(8);
    p->batches.push_back(b);
  }
  b->stream = (hipStream_t)s;
  b->n_tokens = T; b->n_seg = n_seg; b->n_perm = n_perm;
  b->perm.assign(T, 0);
  b->seg_adapter.assign(touched.begin(), touched.end());
  b->seg_start.assign(n_seg + 1, 0);
  int32_t run = 0;
  for (int32_t u = 0; u < n_seg; ++u) {
    const int32_t i = touched[u];
    b->seg_start[u] = run; p->cursor[i] = run; run += p->count[i];
  }
  b->seg_start[n_seg] = run;
  int32_t none_cur = n_perm;  // tokens without adapter go behind the sorted ones (device side only)
  for (int32_t t = 0; t < T; ++t) {
    const int32_t i = t2a[t];
    if (i == -1) b->perm[none_cur++] = t; else b->perm[p->cursor[i]++] = t;
  }

  // work items, grouped per adapter (tokens without adapter form one rank-0 group: shrink clears their v rows)
  const bool mfma_ok = p->dtype != PLORA_F32;  // matrix-core items exist for the 16-bit element types
  ItemGroups(&wl)[2][2] = p->wl;               // [op][0 vector-ALU | 1 matrix-core]
  for (int op = 0; op < 2; ++op)
    for (int k = 0; k < 2; ++k) wl[op][k].clear();
  std::vector<ItemRec>& tg = p->wl_tg;  // one vector-ALU record per token group of the current adapter
  // the vector-ALU records of one adapter group: token groups of kValuTok tokens
  auto token_groups = [&](int16_t rank, float scale, int32_t pt_off, int16_t contig, int32_t start, int32_t n) {
    tg.clear();
    for (int32_t t0 = 0; t0 < n; t0 += kValuTok) {
      const int16_t nt = (int16_t)std::min(kValuTok, n - t0);
      // one token group: nobody else reads the group's weights
      ItemRec it{(int16_t)((n <= kValuTok ? kItemOnce : 0) | contig), nt, rank, 0, scale, pt_off, {0, 0, 0, 0}};
      for (int i = 0; i < 4; ++i) it.tok[i] = b->perm[start + t0 + std::min<int>(i, nt - 1)];
      tg.push_back(it);
    }
  };
  constexpr int kTokBlock = 128;
  auto expand_on_matrix_cores = [&](const Adapter& a, int32_t n) {
    const int64_t r32 = ((int64_t)a.rank + 31) / 32 * 32;
    return mfma_ok && p->mfma_min_tokens_expand > 0 &&
           (n >= p->mfma_min_tokens_expand || (int64_t)n * a.rank * a.rank >= p->mfma_min_work_expand * r32);
  };
  // How the large groups' expand work is cut: a batch with many 64-token blocks (prefill) keeps them
  // (B is then staged once per 64 tokens) and runs them in the panel kernel; a batch with few
  // (decode: at most a hot adapter or two) cuts them into column-split items of one token tile.
  int64_t panel_blocks = 0;
  for (int32_t u = 0; u < n_seg && p->panel_min_blocks > 0; ++u) {
    const int32_t n = p->count[touched[u]];
    if (!expand_on_matrix_cores(p->ad[touched[u]], n)) continue;
    for (int32_t b0 = 0; b0 < n; b0 += kTokBlock)
      for (int32_t left = std::min(n - b0, kTokBlock); left > p->cols_max_group; left -= kMfmaTokE) ++panel_blocks;
  }
  b->panel = p->panel_min_blocks > 0 && panel_blocks >= p->panel_min_blocks;
  const int32_t cols_max_group = b->panel ? p->cols_max_group : kTokBlock;
  size_t n_pt_total = 0;
  int64_t mfma_shrink_items = 0, mfma_shrink_tokens = 0;
  for (int32_t u = 0; u < n_seg; ++u) {
    const Adapter& a = p->ad[touched[u]];
    const int32_t n = p->count[touched[u]];
    const int32_t start = b->seg_start[u];
    // an adapter on consecutive pages needs no table in the image: its records carry its first page
    const int16_t contig = (int16_t)(a.contig ? kItemContig : 0);
    const int32_t pt_off = a.contig ? a.pt[0] : (int32_t)n_pt_total;
    if (!a.contig) n_pt_total += a.pt.size();
    const int16_t rank = (int16_t)a.rank;
    const bool mf_s = mfma_ok && p->mfma_min_tokens > 0 &&
                      (n >= p->mfma_min_tokens || (int64_t)n * a.rank >= p->mfma_min_work);
    const bool mf_e = expand_on_matrix_cores(a, n);
    // Matrix-core items.  Large groups (prefill) are cut into blocks of kTokBlock tokens: a block is
    // the unit that is dealt to an XCD, and inside a block the shrink items go row group by row
    // group with the token groups innermost, so a tile of A is re-read back to back and the block's
    // x tiles (at most kTokBlock rows) stay in L2 for the next row group.
    for (int32_t b0 = 0; b0 < n && (mf_s || mf_e); b0 += kTokBlock) {
      const int32_t b1 = std::min(n, b0 + kTokBlock);
      if (mf_s) {
        double cost = 0.0;
        // the rows of A are read by one item only when the group is a single token tile
        const int16_t kind = (int16_t)((n <= kMfmaTokS ? 1 | kItemOnce : 1) | contig);
        for (int32_t j0 = 0; j0 < a.rank; j0 += kMfmaRows)
          for (int32_t t0 = b0; t0 < b1; t0 += kMfmaTokS) {
            const int16_t nt = (int16_t)std::min(kMfmaTokS, b1 - t0);
            ++mfma_shrink_items;
            mfma_shrink_tokens += nt;
            wl[0][1].items.push_back(ItemRec{kind, nt, rank, (int16_t)j0, a.scale, pt_off, {start + t0, 0, 0, 0}});
            cost += std::min(kMfmaRows, a.rank - j0) + nt;
          }
        wl[0][1].close_group(cost);
      }
      if (mf_e) {
        double cost = 0.0;
        const int16_t kind = (int16_t)((n <= kMfmaTokCols ? 1 | kItemOnce : 1) | contig);
        // a remainder of at most cols_max_group tokens goes as column-split items of one token tile
        for (int32_t t0 = b0; t0 < b1;) {
          const int32_t left = b1 - t0;
          const int16_t nt = (int16_t)std::min(left <= cols_max_group ? kMfmaTokCols : kMfmaTokE, left);
          wl[1][1].items.push_back(ItemRec{kind, nt, rank, 0, a.scale, pt_off, {start + t0, 0, 0, 0}});
          cost += a.rank + 2 * nt;
          t0 += nt;
        }
        wl[1][1].close_group(cost);
      }
    }
    // Vector-ALU items.
    if (!mf_s || !mf_e) {
      token_groups(rank, a.scale, pt_off, contig, start, n);
      if (!mf_e) {
        double cost = 0.0;
        for (const ItemRec& it : tg) { wl[1][0].items.push_back(it); cost += a.rank + 2 * it.ntok; }
        wl[1][0].close_group(cost);
      }
      // shrink: token groups innermost, so that the re-read of a row block by the next token
      // group follows closely and finds the rows in L2
      if (!mf_s) {
        double cost = 0.0;
        for (int32_t j0 = 0; j0 < a.rank; j0 += kShrinkRows)
          for (ItemRec it : tg) {
            it.j0 = (int16_t)j0;
            wl[0][0].items.push_back(it);
            cost += std::min(kShrinkRows, a.rank - j0) + it.ntok;
          }
        wl[0][0].close_group(cost);
      }
    }
  }
  b->full_shrink_tiles = mfma_shrink_items > 0 && 2 * mfma_shrink_tokens >= (int64_t)kMfmaTokS * mfma_shrink_items;
  // tokens without adapter: one rank-0 group of shrink items
  auto none_groups = [&](std::vector<ItemRec>& dst) {
    for (int32_t t0 = 0; t0 < n_none; t0 += kValuTok) {
      const int16_t nt = (int16_t)std::min(kValuTok, n_none - t0);
      ItemRec it{0, nt, 0, 0, 0.f, 0, {0, 0, 0, 0}};
      for (int i = 0; i < 4; ++i) it.tok[i] = b->perm[n_perm + t0 + std::min<int>(i, nt - 1)];
      dst.push_back(it);
    }
  };
  if (n_none > 0) {
    none_groups(wl[0][0].items);
    wl[0][0].close_group(0.1 * ((n_none + kValuTok - 1) / kValuTok));
  }
  std::vector<ItemRec>(&lists)[2][3] = p->wl_lists;  // [op][layout]
  for (int op = 0; op < 2; ++op) {
    arrange_blocks(wl[op][1], wl[op][0], false, lists[op][0], p->wl_bucket, &b->n_heavy[op]);
    // the XCD-dealt form only if launches may ask for it
    if (p->xcd_remap[op]) arrange_blocks(wl[op][1], wl[op][0], true, lists[op][1], p->wl_bucket);
    else lists[op][1].clear();
    // Cooperative form (calls too small to fill the machine): every group as vector-ALU records, one per
    // workgroup, longest chains first.  Not needed when even one slot's ordinary launch is past its limit.
    lists[op][2].clear();
    const int64_t min_grid = op == 1 ? p->min_chunks : 1;  // workgroups per block of the list in the smallest launch
    if (p->coop_max_workgroups[op] > 0 && (int64_t)(lists[op][0].size() / 4) * min_grid <= p->coop_max_workgroups[op]) {
      std::vector<ItemRec>& all = wl[op][1].items;  // reused as scratch: the matrix-core records are arranged already
      all.clear();
      size_t pt_run = 0;
      for (int32_t u = 0; u < n_seg; ++u) {
        const Adapter& a = p->ad[touched[u]];
        token_groups((int16_t)a.rank, a.scale, a.contig ? a.pt[0] : (int32_t)pt_run, (int16_t)(a.contig ? kItemContig : 0),
                     b->seg_start[u], p->count[touched[u]]);
        if (!a.contig) pt_run += a.pt.size();
        if (op == 1) all.insert(all.end(), tg.begin(), tg.end());
        else
          for (int32_t j0 = 0; j0 < a.rank; j0 += kShrinkRows)
            for (ItemRec it : tg) { it.j0 = (int16_t)j0; all.push_back(it); }
      }
      if (op == 0 && n_none > 0) none_groups(all);
      append_by_rank(all, nullptr, all.size(), lists[op][2], p->wl_bucket);
    }
  }
  for (int32_t i : touched) p->count[i] = 0;

  // image layout
  size_t off = 0;
  b->off_perm = off; off = align_up(off + (size_t)T * 4, 256);
  b->off_pt = off; off = align_up(off + (n_pt_total + 1) * 4, 256);
  for (int op = 0; op < 2; ++op)
    for (int k = 0; k < 3; ++k) {
      b->off_items[op][k] = off; b->n_items[op][k] = (int32_t)lists[op][k].size();
      off = align_up(off + lists[op][k].size() * sizeof(ItemRec), 256);
    }
  const size_t need = std::max<size_t>(off, 256);
  if (need > b->cap) {
    const size_t cap = align_up(need + need / 2, 4096);
    if (p->placement_only) {
      if (b->h_img) ::operator delete(b->h_img);
      b->h_img = (uint8_t*)::operator new(cap, std::nothrow);
      if (!b->h_img) { b->cap = 0; return PLORA_ERR_NOMEM; }
    } else {
      if (b->h_img) { (void)hipHostFree(b->h_img); b->h_img = nullptr; }
      if (b->d_img) { (void)hipFree(b->d_img); b->d_img = nullptr; }
      b->cap = 0;
      HIP_TRY(hipHostMalloc((void**)&b->h_img, cap, hipHostMallocDefault));
      HIP_TRY(hipMalloc((void**)&b->d_img, cap));
      if (!b->d_queue) {
        HIP_TRY(hipMalloc((void**)&b->d_queue, kQueueWords * sizeof(uint32_t)));
        HIP_TRY(hipMemsetAsync(b->d_queue, 0, kQueueWords * sizeof(uint32_t), p->aux));  // ahead of the image copy below
      }
    }
    b->cap = cap;
  }
  if (T) std::memcpy(b->h_img + b->off_perm, b->perm.data(), (size_t)T * 4);
  {
    int32_t* dst = (int32_t*)(b->h_img + b->off_pt);
    for (int32_t u = 0; u < n_seg; ++u) {
      const Adapter& a = p->ad[touched[u]];
      if (a.contig) continue;  // its records carry the first page
      std::memcpy(dst, a.pt.data(), a.pt.size() * 4);
      dst += a.pt.size();
    }
    *dst = 0;
  }
  for (int op = 0; op < 2; ++op)
    for (int k = 0; k < 3; ++k)
      if (!lists[op][k].empty())
        std::memcpy(b->h_img + b->off_items[op][k], lists[op][k].data(), lists[op][k].size() * sizeof(ItemRec));
  b->perm.resize(n_perm);

  if (!p->placement_only) {
    // the image travels on the pool's side stream, so it overlaps kernels already queued on `stream`
    if (!b->ev_img) HIP_TRY(hipEventCreateWithFlags(&b->ev_img, hipEventDisableTiming));
    HIP_TRY(hipMemcpyAsync(b->d_img, b->h_img, need, hipMemcpyHostToDevice, p->aux));
    HIP_TRY(hipEventRecord(b->ev_img, p->aux));
    HIP_TRY(hipStreamWaitEvent(b->stream, b->ev_img, 0));
    for (int32_t i : touched) {
      Adapter& a = p->ad[i];
      if (a.copy_pending && poll_ready(p, a) == 0) HIP_TRY(hipStreamWaitEvent(b->stream, a.ev_ready, 0));
    }
  }
  b->adapters.assign(touched.begin(), touched.end());
  for (int32_t i : touched) p->ad[i].pins++;
  b->open = true;
  p->open_batches++;
  *out = b;
  return PLORA_OK;
}

int plora_batch_info(const plora_batch* b, int32_t* n_seg, int32_t* n_perm, const int32_t** perm,
                     const int32_t** seg_adapter, const int32_t** seg_start) {
  if (!b || !b->open) return PLORA_ERR_INVAL;
  if (n_seg) *n_seg = b->n_seg;
  if (n_perm) *n_perm = b->n_perm;
  if (perm) *perm = b->perm.data();
  if (seg_adapter) *seg_adapter = b->seg_adapter.data();
  if (seg_start) *seg_start = b->seg_start.data();
  return PLORA_OK;
}

static int run_slots(plora_pool* p, const plora_batch* b, int32_t slot0, int32_t n_slots, const void* const* in,
                     void* const* outp, plora_stream s, bool is_shrink) {
  if (!p || !b || !b->open || b->pool != p || p->placement_only) return PLORA_ERR_INVAL;
  if (slot0 < 0 || n_slots < 0 || slot0 + n_slots > p->n_slots) return PLORA_ERR_INVAL;
  if (n_slots == 0 || b->n_tokens == 0) return PLORA_OK;
  if (!in || !outp) return PLORA_ERR_INVAL;
  for (int q = 0; q < n_slots; ++q)
    if (!in[q] || !outp[q] || ((uintptr_t)in[q] & 15) || ((uintptr_t)outp[q] & 15)) return PLORA_ERR_INVAL;
  // kernels on a stream other than the batch's own: plora_batch_end has to cover that stream too
  if ((hipStream_t)s != b->stream &&
      std::find(b->other_streams.begin(), b->other_streams.end(), (hipStream_t)s) == b->other_streams.end())
    b->other_streams.push_back((hipStream_t)s);
  LaunchArgs a;
  a.slab = p->slab;
  a.perm = (const int32_t*)(b->d_img + b->off_perm);
  a.pt = (const int32_t*)(b->d_img + b->off_pt);
  a.slots = p->d_slots;
  a.log2_page = p->log2P;
  a.v_stride = p->max_rank;
  a.elems_per_rank = p->C;
  const int vec = 16 / p->elt;
  const int op = is_shrink ? 0 : 1;
  a.pad0 = 0;
  a.pad = 0;
  // Launch classes: an expand launch has one grid dimension for the 512-column chunks, so slots with
  // different chunk counts go in launches of their own (no empty workgroups) ...; shrink has one class.
  std::pair<int, int>* order = p->run_order.data();  // (chunks, index within the call), stable by chunks
  for (int q = 0; q < n_slots; ++q) {
    const int d_out = (int)p->slots[slot0 + q].d_out;
    order[q] = {is_shrink ? 1 : (d_out + kWave * vec - 1) / (kWave * vec), q};
  }
  bool sorted = true;
  for (int q = 1; q < n_slots; ++q) sorted = sorted && order[q - 1].first <= order[q].first;
  if (!sorted)  // (std::stable_sort may allocate; an insertion sort of a few width classes does not)
    for (int q = 1; q < n_slots; ++q) {
      const std::pair<int, int> cur = order[q];
      int k = q;
      while (k > 0 && order[k - 1].first > cur.first) { order[k] = order[k - 1]; --k; }
      order[k] = cur;
    }
  // ... but only when every class keeps a multiple of 8 slots (one slot per XCD, all XCDs alike):
  // a short odd-sized launch costs more in ramp and tail than the empty workgroups it saves.
  bool classes = true;
  for (int q0 = 0; q0 < n_slots;) {
    int nq = 1;
    while (q0 + nq < n_slots && order[q0 + nq].first == order[q0].first) ++nq;
    if (nq % kXcds) classes = false;
    q0 += nq;
  }
  if (!classes) {  // one class in call order, with the largest chunk count
    const int max_chunks = order[n_slots - 1].first;
    for (int q = 0; q < n_slots; ++q) order[q] = {max_chunks, q};
  }
  for (int q0 = 0; q0 < n_slots;) {
    int nq = 1;
    while (q0 + nq < n_slots && nq < kMaxSlotsPerLaunch && order[q0 + nq].first == order[q0].first) ++nq;
    SlotPtrs ptrs;
    for (int q = 0; q < nq; ++q) {
      const int qi = order[q0 + q].second;
      ptrs.a[q] = in[qi];
      ptrs.b[q] = outp[qi];
      ptrs.slot[q] = slot0 + qi;
    }
    const int chunks = order[q0].first;
    q0 += nq;
    // slots fastest when that keeps every slot on one XCD and all XCDs equally loaded; else the
    // items are the fastest dimension and (optionally) come dealt into XCD queues
    a.slot_fastest = p->slot_major[op] == 2 ? 2 : (p->slot_major[op] == 1 || (p->slot_major[op] < 0 && nq % kXcds == 0)) ? 1 : 0;
    // a batch whose matrix-core expand blocks go to the panel kernel uses the longest-first list: the
    // matrix-core blocks are its first part
    const bool panel = op == 1 && b->panel && b->n_heavy[1] > 0;
    int layout = (!panel && a.slot_fastest != 1 && p->xcd_remap[op] && b->n_items[op][1] > 0) ? 1 : 0;
    // a call that cannot fill the machine is bound by its longest dependent chain: cooperative kernels
    const bool coop = !panel && p->coop_max_workgroups[op] > 0 && b->n_items[op][2] > 0 &&
                      (int64_t)nq * (b->n_items[op][layout] / 4) * chunks <= p->coop_max_workgroups[op];
    if (coop) layout = 2;
    const ItemRec* list = (const ItemRec*)(b->d_img + b->off_items[op][layout]);
    const int n_all = b->n_items[op][layout];
    if (n_all == 0) continue;
    // matrix-core shrink items keep two runs of k-values in flight where that pays: token tiles that
    // are mostly full (prefill), or a long contraction
    bool deep = false;
    if (is_shrink && !coop && p->dtype != PLORA_F32 && b->n_heavy[0] > 0) {
      int32_t max_in = 0;
      for (int q = 0; q < nq; ++q) max_in = std::max(max_in, p->slots[ptrs.slot[q]].d_in);
      // ... or a launch too small to hide the chain of an item's runs behind other workgroups
      const bool small_launch = (int64_t)nq * (n_all / 4) <= p->deep_max_workgroups;
      deep = p->mfma_shrink_depth == 2 || (p->mfma_shrink_depth == 0 && (b->full_shrink_tiles || max_in > 4096 || small_launch));
    }
    // one launch over the whole block list, or (panel batches) the matrix-core blocks in the panel kernel
    // followed by the vector-ALU quads in the ordinary one
    struct Part { const ItemRec* items; int n; int mode; };
    // a short panel launch goes with one workgroup per 256 columns: twice the workgroups, half the chain each
    const int panel_mode = panel && 2 * chunks <= 65535 &&
                                   (int64_t)nq * (b->n_heavy[op] / 4) * chunks <= p->panel_half_max_workgroups
                               ? kModePanelHalf : kModePanel;
    const Part parts[2] = {{list, panel ? b->n_heavy[op] : n_all, panel ? panel_mode : coop ? kModeCoop : deep ? kModeDeep : kModeBlocks},
                           {list + b->n_heavy[op], panel ? n_all - b->n_heavy[op] : 0, kModeBlocks}};
    plora_pool::ProfRec rec{op, nullptr, nullptr};
    if (p->profiling) {
      for (hipEvent_t* ev : {&rec.e0, &rec.e1}) {
        if (!p->prof_free.empty()) { *ev = p->prof_free.back(); p->prof_free.pop_back(); }
        else HIP_TRY(hipEventCreate(ev));
      }
    }
    const int last_part = parts[1].n > 0 ? 1 : 0;
    for (int k = 0; k < 2; ++k) {
      const Part& part = parts[k];
      if (part.n == 0) continue;
      a.items = part.items;
      a.n_items = part.n;
      // the events ride on the dispatches: start of the first kernel, end of the last
      const hipEvent_t e0 = (k == 0 || parts[0].n == 0) ? rec.e0 : nullptr;
      const hipEvent_t e1 = k == last_part ? rec.e1 : nullptr;
      hipError_t e;
      if (is_shrink) e = launch_shrink(p->dtype, a, ptrs, nq, part.mode, (hipStream_t)s, e0, e1);
      else e = launch_expand(p->dtype, a, ptrs, nq, chunks, part.mode, (hipStream_t)s, e0, e1);
      HIP_TRY(e);
    }
    if (p->profiling) p->prof.push_back(rec);
  }
  return PLORA_OK;
}

int plora_shrink(plora_pool* p, const plora_batch* b, int32_t slot0, int32_t n_slots, const void* const* x, float* const* v,
                 plora_stream s) {
  return run_slots(p, b, slot0, n_slots, x, (void* const*)v, s, true);
}

int plora_expand(plora_pool* p, const plora_batch* b, int32_t slot0, int32_t n_slots, const float* const* v, void* const* y,
                 plora_stream s) {
  return run_slots(p, b, slot0, n_slots, (const void* const*)v, y, s, false);
}

// plora_delta on a small call: shrink and expand as tasks of one persistent launch (k_delta_queue).  Taken
// when the call is on the batch's own stream (launches on one stream cannot overlap, and they share the
// batch's queue state), covers at most kMaxSlotsFused slots and at most fused_max_tasks tasks, and the
// batch has no panel blocks.  Returns 0 = launched, 1 = not applicable (use the two launches), < 0 = error.
static int delta_in_one_launch(plora_pool* p, const plora_batch* b, int32_t slot0, int32_t n_slots, const void* const* x,
                               float* const* v, void* const* y, plora_stream s) {
  if (p->fused_max_tasks <= 0 || n_slots > kMaxSlotsFused || (hipStream_t)s != b->stream || !b->d_queue) return 1;
  if (b->panel && b->n_heavy[1] > 0) return 1;
  {
    // a captured launch would be replayed with this call's counter targets: graphs take the two launches
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing((hipStream_t)s, &cap) != hipSuccess) { (void)hipGetLastError(); return 1; }
    if (cap != hipStreamCaptureStatusNone) return 1;
  }
  for (int q = 0; q < n_slots; ++q)
    if (!x[q] || !v[q] || ((uintptr_t)x[q] & 15) || ((uintptr_t)v[q] & 15)) return PLORA_ERR_INVAL;
  const int vec = 16 / p->elt;
  int chunks = 1;
  for (int q = 0; q < n_slots; ++q) chunks = std::max(chunks, (int)((p->slots[slot0 + q].d_out + kWave * vec - 1) / (kWave * vec)));
  FusedArgs f;
  // the same choice of lists as the separate launches make: cooperative records for the smallest calls
  const bool coop_s = p->coop_max_workgroups[0] > 0 && b->n_items[0][2] > 0 &&
                      (int64_t)n_slots * (b->n_items[0][0] / 4) <= p->coop_max_workgroups[0];
  const bool coop_e = p->coop_max_workgroups[1] > 0 && b->n_items[1][2] > 0 &&
                      (int64_t)n_slots * (b->n_items[1][0] / 4) * chunks <= p->coop_max_workgroups[1];
  f.coop_s = coop_s; f.coop_e = coop_e;
  f.n_s = coop_s ? b->n_items[0][2] : b->n_items[0][0] / 4;
  f.n_e = coop_e ? b->n_items[1][2] : b->n_items[1][0] / 4;
  const int64_t tasks = ((int64_t)f.n_s + (int64_t)f.n_e * chunks) * n_slots;
  if (tasks > p->fused_max_tasks) return 1;
  if (tasks == 0) return 0;
  f.items_s = (const ItemRec*)(b->d_img + b->off_items[0][coop_s ? 2 : 0]);
  f.items_e = (const ItemRec*)(b->d_img + b->off_items[1][coop_e ? 2 : 0]);
  f.slab = p->slab;
  f.perm = (const int32_t*)(b->d_img + b->off_perm);
  f.pt = (const int32_t*)(b->d_img + b->off_pt);
  f.slots = p->d_slots;
  f.queue = b->d_queue;
  f.timeouts = p->d_timeouts;
  f.elems_per_rank = p->C;
  f.chunks = chunks; f.n_slots = n_slots;
  f.log2_page = p->log2P; f.v_stride = p->max_rank;
  f.spin_limit = (uint32_t)std::min<int64_t>(p->fused_spin_limit, 0xffffffffll);
  f.pad = 0;
  FusedPtrs ptrs;
  for (int q = 0; q < n_slots; ++q) {
    ptrs.x[q] = x[q]; ptrs.v[q] = v[q]; ptrs.y[q] = y[q]; ptrs.slot[q] = slot0 + q;
    ptrs.target[q] = b->q_target[q] + (uint32_t)f.n_s;
  }
  for (int q = n_slots; q < kMaxSlotsFused; ++q) { ptrs.x[q] = nullptr; ptrs.v[q] = nullptr; ptrs.y[q] = nullptr; ptrs.slot[q] = 0; ptrs.target[q] = 0; }
  plora_pool::ProfRec rec{2, nullptr, nullptr};
  if (p->profiling) {
    for (hipEvent_t* ev : {&rec.e0, &rec.e1}) {
      if (!p->prof_free.empty()) { *ev = p->prof_free.back(); p->prof_free.pop_back(); }
      else HIP_TRY(hipEventCreate(ev));
    }
  }
  HIP_TRY(launch_delta_queue(p->dtype, f, ptrs, (hipStream_t)s, rec.e0, rec.e1));
  for (int q = 0; q < n_slots; ++q) b->q_target[q] = ptrs.target[q];  // the launch is queued: its shrink tasks will count
  if (p->profiling) p->prof.push_back(rec);
  p->fused_launches++;
  return 0;
}

int plora_delta(plora_pool* p, const plora_batch* b, int32_t slot0, int32_t n_slots, const void* const* x, float* const* v,
                void* const* y, plora_stream s) {
  if (!p || !b || !b->open || b->pool != p || p->placement_only) return PLORA_ERR_INVAL;
  if (slot0 < 0 || n_slots < 0 || slot0 + n_slots > p->n_slots) return PLORA_ERR_INVAL;
  if (n_slots == 0 || b->n_tokens == 0) return PLORA_OK;
  if (!x || !v || !y) return PLORA_ERR_INVAL;
  for (int q = 0; q < n_slots; ++q)  // the second half's arguments, before anything is queued
    if (!y[q] || ((uintptr_t)y[q] & 15)) return PLORA_ERR_INVAL;
  const int fused = delta_in_one_launch(p, b, slot0, n_slots, x, v, y, s);
  if (fused != 1) return fused < 0 ? fused : PLORA_OK;  // done in one launch, or an error
  const int rc = run_slots(p, b, slot0, n_slots, x, (void* const*)v, s, true);
  if (rc != PLORA_OK) return rc;
  return run_slots(p, b, slot0, n_slots, (const void* const*)v, y, s, false);
}

int plora_delta_static(plora_pool* p, const plora_batch* b, int32_t slot0, int32_t n_slots, const void* const* x,
                       void* const* y, plora_stream s) {
  if (!p || !b || !b->open || b->pool != p || p->placement_only || p->profiling) return PLORA_ERR_INVAL;
  if (slot0 < 0 || n_slots < 0 || slot0 + n_slots > p->n_slots) return PLORA_ERR_INVAL;
  if (n_slots == 0 || b->n_tokens == 0) return PLORA_OK;
  // one v region per slot of the call, each rounded up to 256 bytes, in the library's static device array
  const uint64_t per_slot = align_up((uint64_t)b->n_tokens * (uint64_t)p->max_rank * sizeof(float), 256);
  if (per_slot * (uint64_t)n_slots > static_scratch_bytes()) return PLORA_ERR_LIMIT;
  void* base = nullptr;
  HIP_TRY(static_scratch(&base));
  for (int q = 0; q < n_slots; ++q) p->static_v[q] = (float*)((uint8_t*)base + (uint64_t)q * per_slot);
  return plora_delta(p, b, slot0, n_slots, x, p->static_v.data(), y, s);
}

int plora_profile(plora_pool* p, int enable) {
  if (!p || p->placement_only) return PLORA_ERR_INVAL;
  p->profiling = enable != 0;
  return PLORA_OK;
}

int plora_profile_read(plora_pool* p, double* ms, uint64_t* launches) {
  if (!p || !ms || !launches || p->placement_only) return PLORA_ERR_INVAL;
  for (int k = 0; k < 3; ++k) { ms[k] = 0.0; launches[k] = 0; }
  for (auto& r : p->prof) {
    HIP_TRY(hipEventSynchronize(r.e1));
    float t = 0.f;
    HIP_TRY(hipEventElapsedTime(&t, r.e0, r.e1));
    ms[r.cls] += t;
    launches[r.cls]++;
    p->prof_free.push_back(r.e0);
    p->prof_free.push_back(r.e1);
  }
  p->prof.clear();
  return PLORA_OK;
}

int plora_batch_end(plora_pool* p, plora_batch* b) {
  if (!p || !b || !b->open || b->pool != p) return PLORA_ERR_INVAL;
  std::shared_ptr<Event> done;
  if (!p->placement_only) {
    // kernels that ran on other streams: the batch's own stream waits for them, so that its marker
    // (recorded below or later, but after these waits) stands for all of the batch's kernels
    for (size_t k = 0; k < b->other_streams.size(); ++k) {
      if (b->ev_other.size() <= k) {
        hipEvent_t ev = nullptr;
        HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        b->ev_other.push_back(ev);
      }
      HIP_TRY(hipEventRecord(b->ev_other[k], b->other_streams[k]));
      HIP_TRY(hipStreamWaitEvent(b->stream, b->ev_other[k], 0));
    }
    b->other_streams.clear();
    if (!p->cur_done || p->cur_done->recorded || p->cur_done->stream != b->stream) {
      if (p->cur_done && !p->cur_done->recorded) {  // another stream takes over: close the old marker
        const int rc = record_now(*p->cur_done);
        if (rc != PLORA_OK) return rc;
      }
      p->cur_done = std::make_shared<Event>();
      p->cur_done->stream = b->stream;
    }
    done = p->cur_done;
    if (++done->users >= p->batches_per_marker) {
      const int rc = record_now(*done);
      if (rc != PLORA_OK) return rc;
    }
  }
  for (int32_t i : b->adapters) {
    Adapter& a = p->ad[i];
    a.pins--;
    if (done && (a.last_use.empty() || a.last_use.back() != done)) {
      // a later marker of the same stream covers the earlier one; readers on other streams stay listed
      auto& lu = a.last_use;
      lu.erase(std::remove_if(lu.begin(), lu.end(), [&](const std::shared_ptr<Event>& m) { return m->stream == done->stream; }),
               lu.end());
      lu.push_back(done);
    }
  }
  b->adapters.clear();
  b->done = done;
  b->open = false;
  p->open_batches--;
  return PLORA_OK;
}

}  // extern "C"
