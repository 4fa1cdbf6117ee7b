// Ordering of the library's copies and kernels, checked on the CPU against a stand-in HIP runtime
// (fake_hip.*) whose streams run only when pumped, in random orders that stream and event semantics
// allow.  Random histories of loads, evictions, compactions and batches on two compute and two copy
// streams (a batch's kernels sometimes on the compute stream it was not begun on; a compaction on any
// of the four, now and then with one of its copies failing); the
// stubbed kernels, when they finally run, look at what they would read:
//   * the batch image must have landed (sane work records),
//   * every page that a record's page table names must hold the blob of an adapter (and of the very
//     load) that the batch was begun with, at the right virtual page: a copy onto freed pages that
//     overtook a queued kernel, a kernel that overtook its adapter's copy, or a batch object reused
//     under a queued kernel all show up as a foreign or missing tag.
// With the runtime's waits switched off the same histories must produce violations (the check has teeth).
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <set>
#include <vector>

#include "fake_hip.h"
#include "plora.h"
#include "plora_internal.h"

namespace {
long g_violations = 0, g_kernels_run = 0, g_pages_checked = 0, g_staged_loads = 0, g_failed_loads = 0, g_moved_adapters = 0, g_failed_moves = 0;
bool g_verbose = true;
std::shared_ptr<std::set<uint64_t>> g_expect;  // (adapter + 1) << 24 | load generation, of the batch being queued
int g_elt = 2;

void violation(const char* what, long a = 0, long b = 0) {
  if (g_verbose && g_violations < 5) std::printf("  violation: %s (%ld, %ld)\n", what, a, b);
  ++g_violations;
}

uint64_t word_of(int adapter, int gen, uint64_t vpage) { return ((uint64_t)(adapter + 1) << 48) | ((uint64_t)gen << 24) | vpage; }

void kernel_body(const plora::LaunchArgs a, std::shared_ptr<std::set<uint64_t>> expect) {
  ++g_kernels_run;
  const uint64_t P = (uint64_t)1 << a.log2_page;
  for (int i = 0; i < a.n_items; ++i) {
    const plora::ItemRec it = a.items[i];
    if (it.kind < 0) {
      if (it.kind != -1) { violation("work record is not one the host wrote (image not there?)", i, it.kind); return; }
      continue;
    }
    if ((it.kind & 0xff) > 1 || (it.kind & ~0x3ff) || it.rank < 0 || it.rank > 512 || it.ntok < 1 || it.pt_off < 0) {
      violation("work record is not one the host wrote (image not there?)", i, it.kind);
      return;
    }
    if (it.rank == 0) continue;
    const uint64_t pages = ((uint64_t)it.rank * g_elt * a.elems_per_rank + P - 1) / P;
    for (uint64_t k = 0; k < pages; ++k) {
      const int32_t page = (it.kind & plora::kItemContig) ? it.pt_off + (int32_t)k : a.pt[it.pt_off + k];
      uint64_t w;
      std::memcpy(&w, a.slab + (uint64_t)page * P, 8);
      ++g_pages_checked;
      if ((w & 0xffffff) != k) {
        if (g_verbose && g_violations < 2) {
          std::printf("  item %d kind %d rank %d pt_off %d k %llu page %d: holds adapter %ld gen %ld vpage %ld; expected one of:", i, it.kind, it.rank, it.pt_off,
                      (unsigned long long)k, page, (long)(w >> 48) - 1, (long)((w >> 24) & 0xffffff), (long)(w & 0xffffff));
          for (uint64_t e : *expect) std::printf(" (%ld gen %ld)", (long)(e >> 24) - 1, (long)(e & 0xffffff));
          std::printf("\n");
        }
        violation("page does not hold the expected virtual page", page, (long)(w & 0xffffff));
        return;
      }
      if (!expect->count(w >> 24)) { violation("page holds another adapter (or another load of it)", page, (long)(w >> 48) - 1); return; }
    }
  }
}
}  // namespace

namespace plora {
hipError_t launch_shrink(int, const LaunchArgs& a, const SlotPtrs&, int, int, hipStream_t st, hipEvent_t, hipEvent_t) {
  auto expect = g_expect;
  fakehip::enqueue_kernel(st, [a, expect] { kernel_body(a, expect); });
  return hipSuccess;
}
hipError_t launch_expand(int, const LaunchArgs& a, const SlotPtrs&, int, int, int, hipStream_t st, hipEvent_t, hipEvent_t) {
  auto expect = g_expect;
  fakehip::enqueue_kernel(st, [a, expect] { kernel_body(a, expect); });
  return hipSuccess;
}
// The one-launch form reads both lists (and the same pages) on its stream.
hipError_t launch_delta_queue(int, const FusedArgs& f, const FusedPtrs&, hipStream_t st, hipEvent_t, hipEvent_t) {
  auto expect = g_expect;
  for (int op = 0; op < 2; ++op) {
    LaunchArgs a{};
    a.slab = f.slab; a.perm = f.perm; a.pt = f.pt; a.slots = f.slots; a.elems_per_rank = f.elems_per_rank; a.log2_page = f.log2_page;
    a.items = op ? f.items_e : f.items_s;
    a.n_items = (op ? f.n_e : f.n_s) * ((op ? f.coop_e : f.coop_s) ? 1 : 4);
    fakehip::enqueue_kernel(st, [a, expect] { kernel_body(a, expect); });
  }
  return hipSuccess;
}
// The scatter of a staged load, done for real when the stream reaches it (device memory is host memory here).
hipError_t launch_scatter(const uint8_t* staging, uint8_t* slab, int log2_page, uint64_t bytes, const int32_t* pt,
                          uint32_t n_pages, hipStream_t st) {
  std::vector<int32_t> table(pt, pt + n_pages);
  fakehip::enqueue_kernel(st, [=] {
    const uint64_t P = (uint64_t)1 << log2_page;
    for (uint32_t l = 0; l < table.size(); ++l) {
      const uint64_t lo = l * P, hi = std::min<uint64_t>(lo + P, bytes);
      std::memcpy(slab + (uint64_t)table[l] * P, staging + lo, hi - lo);
    }
  });
  return hipSuccess;
}
// the static device array of plora_delta_static: plain host memory here
static unsigned char g_static_scratch[1 << 20];
uint64_t static_scratch_bytes() { return sizeof(g_static_scratch); }
hipError_t static_scratch(void** out) { *out = g_static_scratch; return hipSuccess; }
}  // namespace plora

#define CHECK(c) do { if (!(c)) { std::printf("CHECK failed at line %d: %s\n", __LINE__, #c); std::exit(1); } } while (0)

static uint64_t rnd(uint64_t& s) { s ^= s >> 12; s ^= s << 25; s ^= s >> 27; return s * 0x2545F4914F6CDD1DULL; }

// One random history; returns the number of violations the kernels saw.
static long history(uint64_t seed, int per_marker, bool ignore_waits, int staging) {
  g_violations = 0;
  fakehip::set_ignore_waits(ignore_waits);
  uint64_t rng = seed * 0x9E3779B97F4A7C15ULL + 1;
  const int32_t d_in[2] = {64, 32}, d_out[2] = {32, 64};
  const int max_ad = 12, max_rank = 64;
  plora_layout lay{2, d_in, d_out, PLORA_BF16, max_ad, max_rank};
  const size_t P = 4096;
  plora_pool* p = nullptr;
  CHECK(plora_pool_create(P, 24, &lay, nullptr, 0, &p) == PLORA_OK);
  CHECK(plora_pool_set_option(p, "batches_per_marker", per_marker) == PLORA_OK);
  if (staging) {  // every load of at most 4 pages' worth goes through the staging buffers, larger ones directly
    CHECK(plora_pool_set_option(p, "staging_bytes", 4 * 4096) == PLORA_OK);
    CHECK(plora_pool_set_option(p, "staging_min_runs", staging) == PLORA_OK);
  }
  hipStream_t compute[2], copy[2];
  for (auto* s : {&compute[0], &compute[1], &copy[0], &copy[1]}) CHECK(hipStreamCreateWithFlags(s, hipStreamNonBlocking) == hipSuccess);
  const std::vector<hipStream_t> prefer{copy[0], copy[1]};
  std::vector<int> rank_of(max_ad, 0), gen(max_ad, 0);
  std::vector<void*> blobs;
  void *x = nullptr, *v = nullptr, *y = nullptr;
  CHECK(hipMalloc(&x, 1 << 16) == hipSuccess && hipMalloc(&v, 1 << 16) == hipSuccess && hipMalloc(&y, 1 << 16) == hipSuccess);
  const void* xs[2] = {x, x};
  float* vs[2] = {(float*)v, (float*)v};
  const float* vsc[2] = {(float*)v, (float*)v};
  void* ys[2] = {y, y};
  int batches = 0, evictions = 0, busy = 0, cross_stream_batches = 0;
  long failed_loads = 0;
  hipEvent_t cross = nullptr;
  CHECK(hipEventCreateWithFlags(&cross, hipEventDisableTiming) == hipSuccess);
  for (int step = 0; step < 600; ++step) {
    const int what = rnd(rng) % 22;
    const int id = rnd(rng) % max_ad;
    if (what < 5) {
      if (!rank_of[id]) {
        const int r = 8 << (rnd(rng) % 4);
        const uint64_t S = plora_adapter_bytes(p, r);
        void* blob = nullptr;
        CHECK(hipHostMalloc(&blob, S, 0) == hipSuccess);
        blobs.push_back(blob);
        ++gen[id];
        for (uint64_t o = 0; o < S; o += 8) { const uint64_t w = word_of(id, gen[id], o / P); std::memcpy((char*)blob + o, &w, 8); }
        // now and then one of the load's copies fails after others were queued: the load must be undone
        // without leaving those copies in flight over pages that the next load may be given
        const bool fault = rnd(rng) % 8 == 0;
        if (fault) fakehip::fail_copy_in(1 + (int)(rnd(rng) % 3));
        const int rc = plora_load_adapter(p, id, r, 1.0f, blob, copy[rnd(rng) % 2], nullptr, nullptr);
        fakehip::fail_copy_in(0);
        CHECK(rc == PLORA_OK || rc == PLORA_ERR_NOMEM || (fault && rc == PLORA_ERR_HIP));
        if (rc == PLORA_ERR_HIP) { ++failed_loads; CHECK(plora_adapter_ready(p, id) == PLORA_ERR_NOTFOUND); }
        if (rc == PLORA_OK) rank_of[id] = r;
      }
    } else if (what < 10) {
      if (rank_of[id]) {
        const int rc = plora_evict(p, id);
        CHECK(rc == PLORA_OK || rc == PLORA_ERR_BUSY);  // busy: its copy has not finished yet
        if (rc == PLORA_OK) { rank_of[id] = 0; ++evictions; } else ++busy;
      }
    } else if (what < 19) {
      std::vector<int32_t> res;
      for (int a = 0; a < max_ad; ++a) if (rank_of[a]) res.push_back(a);
      if (res.empty()) continue;
      const int T = 1 + rnd(rng) % 40, n_used = 1 + rnd(rng) % 3;
      std::vector<int32_t> t2a(T);
      auto expect = std::make_shared<std::set<uint64_t>>();
      const size_t first = rnd(rng) % res.size();
      for (int t = 0; t < T; ++t) {
        t2a[t] = rnd(rng) % 9 == 0 ? -1 : res[(first + rnd(rng) % n_used) % res.size()];
        if (t2a[t] >= 0) expect->insert(((uint64_t)(t2a[t] + 1) << 24) | (uint64_t)gen[t2a[t]]);
      }
      const int which = (int)(rnd(rng) % 2);
      hipStream_t st = compute[which];
      plora_batch* b = nullptr;
      CHECK(plora_batch_begin(p, t2a.data(), T, st, &b) == PLORA_OK);
      g_expect = expect;
      // now and then the kernels run on the other compute stream, ordered after the batch's own by an
      // event as the contract asks of the caller: plora_batch_end has to cover that stream as well
      hipStream_t run_on = st;
      if (rnd(rng) % 3 == 0) {
        run_on = compute[1 - which];
        CHECK(hipEventRecord(cross, st) == hipSuccess);
        CHECK(hipStreamWaitEvent(run_on, cross, 0) == hipSuccess);
        ++cross_stream_batches;
      }
      const int form = (int)(rnd(rng) % 3);
      if (form == 0) {
        CHECK(plora_shrink(p, b, 0, 2, xs, vs, run_on) == PLORA_OK);
        if (rnd(rng) % 4 == 0) fakehip::pump_random(rng, 2, prefer);
        CHECK(plora_expand(p, b, 0, 2, vsc, ys, st) == PLORA_OK);  // (the expand on the batch's own stream)
      } else if (form == 1) {
        CHECK(plora_delta(p, b, 0, 2, xs, vs, ys, run_on) == PLORA_OK);
      } else {
        CHECK(plora_delta_static(p, b, 0, 2, xs, ys, run_on) == PLORA_OK);
      }
      CHECK(plora_batch_end(p, b) == PLORA_OK);
      ++batches;
    } else if (what < 21) {
      // compaction on any stream: its page moves must wait for the kernels in flight that read the pages
      // they overwrite (through old tables), and later loads into the vacated pages for the moves
      hipStream_t st = (rnd(rng) % 2 ? compute : copy)[rnd(rng) % 2];
      const uint32_t bound[4] = {0, 1, 3, 8};
      const bool fault = rnd(rng) % 10 == 0;
      if (fault) fakehip::fail_copy_in(1 + (int)(rnd(rng) % 2));
      uint32_t pages = 0, moved = 0;
      const int rc = plora_compact(p, st, bound[rnd(rng) % 4], &pages, &moved);
      fakehip::fail_copy_in(0);
      CHECK(rc == PLORA_OK || (fault && rc == PLORA_ERR_HIP));
      CHECK((pages == 0) == (moved == 0));
      g_moved_adapters += moved;
      if (rc == PLORA_ERR_HIP) {  // the adapter whose move failed has left the pool
        int gone = 0;
        for (int a = 0; a < max_ad; ++a)
          if (rank_of[a] && plora_adapter_ready(p, a) == PLORA_ERR_NOTFOUND) { rank_of[a] = 0; ++gone; }
        CHECK(gone == 1);
        ++g_failed_moves;
      }
    } else if (rnd(rng) % 4 == 0) {
      fakehip::drain();
    }
    fakehip::pump_random(rng, (int)(rnd(rng) % 7), prefer);
  }
  fakehip::drain();
  plora_stats stats;
  CHECK(plora_pool_stats(p, &stats) == PLORA_OK);
  CHECK(staging == 0 ? stats.staged_loads == 0 : staging == 1 ? stats.staged_loads > 10 : true);
  g_staged_loads += (long)stats.staged_loads;
  g_failed_loads += failed_loads;
  CHECK(hipEventDestroy(cross) == hipSuccess);
  CHECK(plora_pool_destroy(p) == PLORA_OK);
  for (void* bl : blobs) CHECK(hipHostFree(bl) == hipSuccess);
  CHECK(hipFree(x) == hipSuccess && hipFree(v) == hipSuccess && hipFree(y) == hipSuccess);
  for (hipStream_t s : {compute[0], compute[1], copy[0], copy[1]}) CHECK(hipStreamDestroy(s) == hipSuccess);
  CHECK(batches > 100 && evictions > 20 && cross_stream_batches > 20);
  return g_violations;
}

int main() {
  long total_kernels = 0;
  for (int per_marker : {1, 4, 64})
    for (uint64_t seed = 1; seed <= 40; ++seed) {
      for (int staging : {0, 1, 2}) {  // off; every small blob staged; only those in at least two runs
        const long bad = history(seed, per_marker, false, staging);
        if (bad) {
          std::printf("seed %llu, a completion event per %d batches, staging %d: %ld violations\n", (unsigned long long)seed,
                      per_marker, staging, bad);
          return 1;
        }
      }
    }
  total_kernels = g_kernels_run;
  CHECK(total_kernels > 10000 && g_pages_checked > 10000 && g_staged_loads > 1000 && g_failed_loads > 100);
  CHECK(g_moved_adapters > 1000 && g_failed_moves > 20);
  // the same histories without the runtime honouring waits: the kernels must notice
  g_verbose = false;
  int caught = 0;
  for (uint64_t seed = 1; seed <= 10; ++seed) caught += history(seed, 4, true, (int)(seed % 3)) > 0;
  CHECK(caught == 10);
  std::printf("host order run OK (%ld kernels, %ld pages checked, %ld staged loads, %ld adapters moved by compaction)\n", total_kernels, g_pages_checked, g_staged_loads, g_moved_adapters);
  return 0;
}
