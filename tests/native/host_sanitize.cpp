// Host-side stress of the library's allocator and batch translation on a placement-only pool (no
// GPU call is made), meant to be built with -fsanitize=address,undefined: random load / evict /
// batch histories with the invariants of Sec. III-C checked after every step.  The kernel launchers
// are stubbed: a placement-only pool never launches.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <set>
#include <vector>

#include "plora.h"
#include "plora_internal.h"

namespace plora {
hipError_t launch_shrink(int, const LaunchArgs&, const SlotPtrs&, int, int, hipStream_t, hipEvent_t, hipEvent_t) { return hipSuccess; }
hipError_t launch_expand(int, const LaunchArgs&, const SlotPtrs&, int, int, int, hipStream_t, hipEvent_t, hipEvent_t) { return hipSuccess; }
hipError_t launch_scatter(const uint8_t*, uint8_t*, int, uint64_t, const int32_t*, uint32_t, hipStream_t) { return hipSuccess; }
hipError_t launch_delta_queue(int, const FusedArgs&, const FusedPtrs&, hipStream_t, hipEvent_t, hipEvent_t) { return hipSuccess; }
uint64_t static_scratch_bytes() { return 0; }
hipError_t static_scratch(void**) { return hipErrorNotSupported; }
}  // namespace plora

#define CHECK(c) do { if (!(c)) { std::printf("CHECK failed at line %d: %s\n", __LINE__, #c); std::exit(1); } } while (0)

int main() {
  std::mt19937 rng(12345);
  for (int round = 0; round < 6; ++round) {
    const int32_t d_in[3] = {64, 264, 8}, d_out[3] = {1304, 8, 72};
    const int max_ad = 48, max_rank = round % 2 ? 40 : 128;
    plora_layout lay{3, d_in, d_out, round % 3, max_ad, max_rank};
    const size_t P = 4096u << (round % 3);
    const uint32_t n_pages = 64 + 61 * round;
    plora_pool* p = nullptr;
    CHECK(plora_pool_create(P, n_pages, &lay, nullptr, PLORA_POOL_PLACEMENT_ONLY, &p) == PLORA_OK);
    CHECK(plora_pool_set_option(p, "mfma_min_tokens", round) == PLORA_OK);
    CHECK(plora_pool_set_option(p, "coop_max_workgroups_shrink", round % 2 ? 0 : 100000) == PLORA_OK);
    std::vector<int> rank_of(max_ad, 0);
    std::vector<std::vector<int32_t>> table(max_ad);
    std::vector<plora_batch*> open;
    std::vector<std::vector<int32_t>> open_ids;
    for (int step = 0; step < 4000; ++step) {
      const int what = rng() % 10;
      const int id = rng() % max_ad;
      if (what < 4) {
        const int r = 1 + rng() % max_rank;
        const int32_t* pt = nullptr;
        uint32_t n = 0;
        const int rc = plora_load_adapter(p, id, r, 0.5f, nullptr, nullptr, &pt, &n);
        if (rank_of[id]) CHECK(rc == PLORA_ERR_EXISTS);
        else if (rc == PLORA_OK) {
          CHECK(n == (plora_adapter_bytes(p, r) + P - 1) / P);
          table[id].assign(pt, pt + n);
          for (uint32_t k = 1; k < n; ++k) CHECK(pt[k] > pt[k - 1]);
          rank_of[id] = r;
        } else CHECK(rc == PLORA_ERR_NOMEM);
      } else if (what < 7) {
        bool pinned = false;
        for (auto& ids : open_ids) for (int32_t a : ids) pinned |= a == id;
        const int rc = plora_evict(p, id);
        if (!rank_of[id]) CHECK(rc == PLORA_ERR_NOTFOUND);
        else if (pinned) CHECK(rc == PLORA_ERR_BUSY);
        else { CHECK(rc == PLORA_OK); rank_of[id] = 0; table[id].clear(); }
      } else if (what < 9 && open.size() < 3) {
        std::vector<int32_t> res;
        for (int a = 0; a < max_ad; ++a) if (rank_of[a]) res.push_back(a);
        const int T = rng() % 400;
        std::vector<int32_t> t2a(T);
        std::vector<int32_t> used;
        for (int t = 0; t < T; ++t) {
          t2a[t] = (res.empty() || rng() % 8 == 0) ? -1 : res[(rng() % res.size()) * (rng() % 2) % res.size()];
          if (t2a[t] >= 0) used.push_back(t2a[t]);
        }
        plora_batch* b = nullptr;
        CHECK(plora_batch_begin(p, t2a.data(), T, nullptr, &b) == PLORA_OK);
        int32_t n_seg = 0, n_perm = 0;
        const int32_t *perm = nullptr, *sa = nullptr, *ss = nullptr;
        CHECK(plora_batch_info(b, &n_seg, &n_perm, &perm, &sa, &ss) == PLORA_OK);
        CHECK(n_perm == (int32_t)used.size() && ss[n_seg] == n_perm);
        for (int u = 0; u < n_seg; ++u) {
          CHECK(u == 0 || sa[u] > sa[u - 1]);
          for (int k = ss[u]; k < ss[u + 1]; ++k) {
            CHECK(t2a[perm[k]] == sa[u]);
            CHECK(k == ss[u] || perm[k] > perm[k - 1]);  // stable
          }
        }
        open.push_back(b);
        open_ids.push_back(std::vector<int32_t>(sa, sa + n_seg));
      } else if (!open.empty()) {
        const size_t k = rng() % open.size();
        CHECK(plora_batch_end(p, open[k]) == PLORA_OK);
        open.erase(open.begin() + k);
        open_ids.erase(open_ids.begin() + k);
      }
      // tables pairwise disjoint, inside the pool, and consistent with the counters
      if (step % 50 == 0) {
        std::set<int32_t> seen;
        size_t total = 0;
        for (int a = 0; a < max_ad; ++a)
          for (int32_t q : table[a]) { CHECK(q >= 0 && (uint32_t)q < n_pages); CHECK(seen.insert(q).second); ++total; }
        plora_stats st;
        CHECK(plora_pool_stats(p, &st) == PLORA_OK);
        CHECK(st.used_pages == total && st.used_pages + st.free_pages == n_pages);
      }
    }
    CHECK(plora_pool_destroy(p) == (open.empty() ? PLORA_OK : PLORA_ERR_BUSY));
    for (plora_batch* b : open) CHECK(plora_batch_end(p, b) == PLORA_OK);
    if (!open.empty()) CHECK(plora_pool_destroy(p) == PLORA_OK);
  }
  std::printf("host sanitize run OK\n");
  return 0;
}
