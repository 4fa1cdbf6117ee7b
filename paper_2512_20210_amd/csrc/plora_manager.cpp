// Residency policy on top of the page pool (Sec. III-B): load on demand, eviction by the combined
// score of Eq. 3, threshold prefetching ("Proactive Prefetching").  Host code; it talks to the pool
// through the public entry points only.  See include/plora.h (plora_manager_*) for the contract and
// for the reading of what the paper leaves open.
//
// All score arithmetic is in double, one rounding per operation in the order written (this file is
// compiled without floating-point contraction), because the scores decide an order.
#include "../../include/plora.h"

#include <algorithm>
#include <cstring>
#include <deque>
#include <new>
#include <vector>

namespace {

struct Entry {
  int32_t rank = 0;      // 0 = not registered
  float scale = 0.f;
  const void* host = nullptr;
  bool resident = false, prefetched = false;
  int64_t last_use = 0;
  int32_t hits_in_window = 0;
};

}  // namespace

struct plora_manager {
  plora_pool* pool = nullptr;
  plora_manager_config cfg{};
  std::vector<Entry> ad;
  std::vector<float> p_hat;
  bool have_p_hat = false;
  int64_t clock = 0;
  std::deque<int32_t> recent;
  std::vector<int32_t> residents;  // unordered
  std::vector<int32_t> log;        // (kind, id) pairs: kind 0 = load, 1 = evict
  plora_manager_stats st{};
  bool filled = false;             // the pool has run out of pages at least once
  // scratch
  std::vector<int32_t> order, victims;
  std::vector<double> score;
};

namespace {

void touch(plora_manager* m, int32_t id) {
  m->clock += 1;
  m->recent.push_back(id);
  m->ad[id].hits_in_window += 1;
  if ((int64_t)m->recent.size() > (int64_t)m->cfg.window) {
    const int32_t old = m->recent.front();
    m->recent.pop_front();
    m->ad[old].hits_in_window -= 1;
  }
}

// Retention score of every resident adapter: ids ascending in m->order, scores beside them in m->score.
void compute_scores(plora_manager* m) {
  std::vector<int32_t>& ids = m->order;
  ids.assign(m->residents.begin(), m->residents.end());
  std::sort(ids.begin(), ids.end());
  const size_t n = ids.size();
  // position by last use, oldest first; equal clocks (adapters prefetched in one go) by id
  std::vector<int32_t> by_use(ids);
  std::stable_sort(by_use.begin(), by_use.end(), [&](int32_t a, int32_t b) { return m->ad[a].last_use < m->ad[b].last_use; });
  std::vector<double> lru(m->ad.size(), 0.0);
  for (size_t k = 0; k < n; ++k) lru[by_use[k]] = n > 1 ? (double)k / (double)(n - 1) : 1.0;
  int32_t cmax = 1;
  for (int32_t i : ids) cmax = std::max(cmax, m->ad[i].hits_in_window);
  m->score.resize(n);
  for (size_t k = 0; k < n; ++k) {
    const int32_t i = ids[k];
    const double ph = m->have_p_hat ? (double)m->p_hat[i] : 0.0;
    const double a = m->cfg.alpha * lru[i];
    const double b = m->cfg.beta * ((double)m->ad[i].hits_in_window / (double)cmax);
    const double c = m->cfg.gamma * ph;
    m->score[k] = (a + b) + c;
  }
}

bool predicted(const plora_manager* m, int32_t i) { return m->have_p_hat && (double)m->p_hat[i] > m->cfg.theta; }

void sample_utilisation(plora_manager* m) {
  plora_stats s;
  if (plora_pool_stats(m->pool, &s) != PLORA_OK) return;
  const double pu = (double)s.used_pages / (double)s.n_pages;
  const double bu = (double)s.resident_bytes / ((double)s.n_pages * (double)s.page_bytes);
  if (m->st.util_samples == 0) { m->st.page_util_min = pu; m->st.byte_util_min = bu; }
  m->st.util_samples += 1;
  m->st.page_util_sum += pu;
  m->st.byte_util_sum += bu;
  m->st.page_util_min = std::min(m->st.page_util_min, pu);
  m->st.byte_util_min = std::min(m->st.byte_util_min, bu);
}

// Loads `id` on `stream`, evicting residents in ascending order of score (ties: lowest id) while the pool is
// out of pages; with spare_predicted only residents whose prediction is at most theta may go.  The scores
// are taken once, when the pool first refuses.  1 = loaded, 0 = no room could be made, < 0 = error.
int load_with_eviction(plora_manager* m, int32_t id, plora_stream stream, bool spare_predicted) {
  Entry& e = m->ad[id];
  bool have_victims = false;
  size_t next_victim = 0;
  const bool may_wait = !spare_predicted;  // loads on demand wait for a busy victim's copy, prefetches do not
  auto evicted_now = [&](int32_t v) {
    Entry& ve = m->ad[v];
    ve.resident = false;
    m->residents.erase(std::find(m->residents.begin(), m->residents.end(), v));
    m->log.push_back(1);
    m->log.push_back(v);
    m->st.evictions += 1;
    if (ve.prefetched) { ve.prefetched = false; m->st.wasted_prefetches += 1; }
  };
  for (;;) {
    const int rc = plora_load_adapter(m->pool, id, e.rank, e.scale, e.host, stream, nullptr, nullptr);
    if (rc == PLORA_OK) {
      e.resident = true;
      e.last_use = m->clock;
      m->residents.push_back(id);
      m->log.push_back(0);
      m->log.push_back(id);
      m->st.loads += 1;
      if (m->filled) sample_utilisation(m);
      return 1;
    }
    if (rc != PLORA_ERR_NOMEM) return rc;
    m->filled = true;
    if (!have_victims) {
      compute_scores(m);
      std::vector<int32_t> idx(m->order.size());
      for (size_t k = 0; k < idx.size(); ++k) idx[k] = (int32_t)k;
      std::stable_sort(idx.begin(), idx.end(), [&](int32_t a, int32_t b) { return m->score[a] < m->score[b]; });
      m->victims.clear();
      for (int32_t k : idx)
        if (!spare_predicted || !predicted(m, m->order[k])) m->victims.push_back(m->order[k]);
      have_victims = true;
      next_victim = 0;
    }
    bool evicted = false;
    while (next_victim < m->victims.size()) {
      const int32_t v = m->victims[next_victim++];
      if (v < 0) continue;  // gone already
      const int ev = plora_evict(m->pool, v);
      if (ev == PLORA_ERR_BUSY) { m->st.skipped_busy += 1; continue; }  // still being copied, or in use by an open batch
      if (ev != PLORA_OK) return ev;
      m->victims[next_victim - 1] = -1;
      evicted_now(v);
      evicted = true;
      break;
    }
    if (!evicted && may_wait) {
      // only busy victims are left: wait for the copy of each in score order and take the first that lets go
      for (size_t k = 0; k < m->victims.size() && !evicted; ++k) {
        const int32_t v = m->victims[k];
        if (v < 0) continue;
        const int w = plora_sync_adapter(m->pool, v);
        if (w != PLORA_OK) return w;
        m->st.waited_for_busy += 1;
        const int ev = plora_evict(m->pool, v);
        if (ev == PLORA_ERR_BUSY) continue;  // held by an open batch
        if (ev != PLORA_OK) return ev;
        m->victims[k] = -1;
        evicted_now(v);
        evicted = true;
      }
    }
    if (!evicted) return 0;
  }
}

}  // namespace

extern "C" {

int plora_suggest_page_bytes(const plora_layout* lay, const int32_t* ranks, const double* weights, int32_t n,
                             double max_frag, size_t min_page, size_t max_page, size_t* page_out, double* frag_out) {
  if (!lay || !lay->d_in || !lay->d_out || lay->n_slots < 1 || !ranks || !weights || n < 1) return PLORA_ERR_INVAL;
  if (!(max_frag >= 0.0) || !(max_frag < 1.0)) return PLORA_ERR_INVAL;
  if (min_page < 4096 || (min_page & (min_page - 1)) || (max_page & (max_page - 1)) || max_page < min_page) return PLORA_ERR_INVAL;
  if (lay->dtype < 0 || lay->dtype > 2) return PLORA_ERR_INVAL;
  const uint64_t elt = lay->dtype == PLORA_F32 ? 4 : 2;
  uint64_t c = 0;
  for (int s = 0; s < lay->n_slots; ++s) {
    if (lay->d_in[s] <= 0 || lay->d_out[s] <= 0) return PLORA_ERR_INVAL;
    c += (uint64_t)lay->d_in[s] + (uint64_t)lay->d_out[s];
  }
  double wsum = 0.0;
  for (int32_t k = 0; k < n; ++k) {
    if (ranks[k] < 1 || !(weights[k] >= 0.0)) return PLORA_ERR_INVAL;
    wsum += weights[k];
  }
  if (!(wsum > 0.0)) return PLORA_ERR_INVAL;
  size_t best = 0, least = 0;
  double best_frag = 0.0, least_frag = 2.0;
  for (size_t P = min_page;; P <<= 1) {
    double wasted = 0.0, held = 0.0;
    for (int32_t k = 0; k < n; ++k) {
      const uint64_t S = (uint64_t)ranks[k] * elt * c;
      const uint64_t pages = (S + P - 1) / P;
      wasted += weights[k] * (double)(pages * P - S);
      held += weights[k] * (double)(pages * P);
    }
    const double frag = wasted / held;
    if (frag <= max_frag) { best = P; best_frag = frag; }            // candidates ascend: the last that meets the bound is the largest
    if (frag < least_frag) { least = P; least_frag = frag; }         // strict: the smaller page wins a tie
    if (P >= max_page) break;
  }
  if (!best) { best = least; best_frag = least_frag; }
  if (page_out) *page_out = best;
  if (frag_out) *frag_out = best_frag;
  return PLORA_OK;
}

int plora_manager_create(plora_pool* pool, int32_t n_adapters, const plora_manager_config* cfg, plora_manager** out) {
  if (!pool || !cfg || !out || n_adapters < 1) return PLORA_ERR_INVAL;
  if (!(cfg->alpha >= 0.0) || !(cfg->beta >= 0.0) || !(cfg->gamma >= 0.0) || cfg->window < 1 || !(cfg->theta >= 0.0) || !(cfg->theta <= 1.0))
    return PLORA_ERR_INVAL;
  plora_manager* m = new (std::nothrow) plora_manager;
  if (!m) return PLORA_ERR_NOMEM;
  m->pool = pool;
  m->cfg = *cfg;
  m->ad.resize(n_adapters);
  m->p_hat.assign(n_adapters, 0.f);
  *out = m;
  return PLORA_OK;
}

int plora_manager_destroy(plora_manager* m) {
  if (!m) return PLORA_ERR_INVAL;
  delete m;
  return PLORA_OK;
}

int plora_manager_set_adapter(plora_manager* m, int32_t id, int32_t rank, float scale, const void* pinned_host_ptr) {
  if (!m || id < 0 || id >= (int32_t)m->ad.size() || rank < 1) return PLORA_ERR_INVAL;
  if (m->ad[id].resident) return PLORA_ERR_BUSY;
  m->ad[id].rank = rank;
  m->ad[id].scale = scale;
  m->ad[id].host = pinned_host_ptr;
  return PLORA_OK;
}

int plora_manager_set_prediction(plora_manager* m, const float* p_hat) {
  if (!m) return PLORA_ERR_INVAL;
  m->have_p_hat = p_hat != nullptr;
  if (p_hat) std::memcpy(m->p_hat.data(), p_hat, m->p_hat.size() * sizeof(float));
  return PLORA_OK;
}

int plora_manager_request(plora_manager* m, int32_t id, plora_stream copy_stream, int32_t* hit_out) {
  if (!m || id < 0 || id >= (int32_t)m->ad.size() || m->ad[id].rank == 0) return PLORA_ERR_INVAL;
  Entry& e = m->ad[id];
  touch(m, id);
  const bool was_prefetched = e.prefetched;
  e.prefetched = false;
  if (e.resident) {
    e.last_use = m->clock;
    m->st.hits += 1;
    if (was_prefetched) m->st.useful_prefetches += 1;
    if (hit_out) *hit_out = 1;
    return PLORA_OK;
  }
  m->st.misses += 1;
  if (hit_out) *hit_out = 0;
  const int rc = load_with_eviction(m, id, copy_stream, false);
  if (rc < 0) return rc;
  if (rc == 0) m->st.failed_loads += 1;
  return PLORA_OK;
}

int plora_manager_prefetch(plora_manager* m, const float* p_hat, plora_stream prefetch_stream, int32_t* n_started_out) {
  if (!m || !p_hat) return PLORA_ERR_INVAL;
  plora_manager_set_prediction(m, p_hat);
  // most probable first; equal probabilities by id
  std::vector<int32_t> want;
  for (int32_t i = 0; i < (int32_t)m->ad.size(); ++i)
    if (predicted(m, i)) want.push_back(i);
  std::stable_sort(want.begin(), want.end(), [&](int32_t a, int32_t b) { return m->p_hat[a] > m->p_hat[b]; });
  int32_t started = 0;
  for (int32_t id : want) {
    Entry& e = m->ad[id];
    if (e.resident || e.rank == 0) continue;
    const int rc = load_with_eviction(m, id, prefetch_stream, true);
    if (rc < 0) { if (n_started_out) *n_started_out = started; return rc; }
    if (rc == 0) { m->st.prefetch_no_room += 1; break; }  // no unpredicted resident left to give up its pages
    e.prefetched = true;
    m->st.prefetch_loads += 1;
    ++started;
  }
  if (n_started_out) *n_started_out = started;
  return PLORA_OK;
}

int plora_manager_scores(plora_manager* m, int32_t* ids_out, double* scores_out, int32_t cap, int32_t* n_out) {
  if (!m || !n_out) return PLORA_ERR_INVAL;
  compute_scores(m);
  *n_out = (int32_t)m->order.size();
  for (int32_t k = 0; k < *n_out && k < cap; ++k) {
    if (ids_out) ids_out[k] = m->order[k];
    if (scores_out) scores_out[k] = m->score[k];
  }
  return PLORA_OK;
}

int plora_manager_residents(plora_manager* m, int32_t* ids_out, int32_t cap, int32_t* n_out) {
  if (!m || !n_out) return PLORA_ERR_INVAL;
  m->order.assign(m->residents.begin(), m->residents.end());
  std::sort(m->order.begin(), m->order.end());
  *n_out = (int32_t)m->order.size();
  for (int32_t k = 0; k < *n_out && k < cap; ++k)
    if (ids_out) ids_out[k] = m->order[k];
  return PLORA_OK;
}

int plora_manager_state(plora_manager* m, int32_t id) {
  if (!m || id < 0 || id >= (int32_t)m->ad.size()) return PLORA_ERR_INVAL;
  return (m->ad[id].resident ? 1 : 0) | (m->ad[id].prefetched ? 2 : 0);
}

int plora_manager_get_stats(plora_manager* m, plora_manager_stats* out) {
  if (!m || !out) return PLORA_ERR_INVAL;
  *out = m->st;
  return PLORA_OK;
}

int plora_manager_log(plora_manager* m, int32_t* out, int64_t cap_pairs, int64_t* n_pairs, int32_t clear) {
  if (!m || !n_pairs) return PLORA_ERR_INVAL;
  *n_pairs = (int64_t)(m->log.size() / 2);
  if (out) std::memcpy(out, m->log.data(), (size_t)std::min<int64_t>(cap_pairs, *n_pairs) * 2 * sizeof(int32_t));
  if (clear) m->log.clear();
  return PLORA_OK;
}

}  // extern "C"
