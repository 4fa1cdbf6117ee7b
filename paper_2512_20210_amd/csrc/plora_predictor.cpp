// Traffic predictor of Sec. III-A on the host (the paper runs it on CPU cores beside the GPU work):
// a stack of LSTM layers over a sliding window of per-interval access counts, a fully connected
// layer that gives one access probability per adapter, Eq. 2 as the loss, Adam, and a replay buffer
// of the most recent intervals for the online updates.  See include/plora.h for the contract.
//
// An interval's feature vector is sparse (an interval of 100 requests touches at most 100 of
// thousands of adapters), so intervals are kept as (adapter, feature) lists and the first layer's
// input weights as one row of 4H values per adapter — the learned embedding of that adapter: the
// gates of a step are the bias plus the feature-weighted sum of the rows of the adapters seen.
#include "../../include/plora.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <deque>
#include <new>
#include <thread>
#include <vector>

namespace {

struct Sparse {
  std::vector<int32_t> id;   // ascending
  std::vector<float> f;      // count / (1 + count)
};

inline float sigmoidf(float z) { return 1.0f / (1.0f + std::exp(-z)); }

// splitmix64: the counter-based generator behind parameter initialisation and minibatch sampling.
inline uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ULL;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ULL;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBULL;
  return x ^ (x >> 31);
}

}  // namespace

// Working state of one sample (one per worker thread): per step and layer the gate activations, cell
// and hidden states of the forward pass, the backward pass's carries, and a gradient accumulator.
struct Scratch {
  std::vector<float> gi, gf, gg, go, cs, hs, tc;  // [W][L][H] each
  std::vector<float> logits, dz, da, dh, dc, dh_up;
  std::vector<float> g;                           // gradient of this worker's samples
  double loss = 0.0;
};

struct plora_predictor {
  plora_predictor_config cfg;
  int n = 0, H = 0, L = 0, W = 0;
  std::vector<float> p, m, v;  // parameters, Adam moments
  struct Off { size_t w_in, w_hh, b; };
  std::vector<Off> off;
  size_t w_fc = 0, b_fc = 0;
  int64_t adam_t = 0;
  uint64_t draws = 0;               // minibatch samples drawn so far (counter of the generator)
  std::deque<Sparse> replay;        // the most recent intervals, oldest first
  int threads = 1;
  std::vector<Scratch> scr;         // scr[0] also holds the summed gradient
};

namespace {

size_t idx(const plora_predictor* q, int t, int l) { return ((size_t)t * q->L + l) * q->H; }

// Forward pass over the window `seq` (W entries, oldest first; a null entry is an all-zero interval).
void forward(const plora_predictor* q, Scratch& z, const Sparse* const* seq) {
  const int H = q->H, L = q->L, W = q->W, n = q->n;
  const float* P = q->p.data();
  std::vector<float> a(4 * H);
  for (int t = 0; t < W; ++t) {
    for (int l = 0; l < L; ++l) {
      const float* b = P + q->off[l].b;
      for (int k = 0; k < 4 * H; ++k) a[k] = b[k];
      if (l == 0) {
        if (seq[t])
          for (size_t e = 0; e < seq[t]->id.size(); ++e) {
            const float* row = P + q->off[0].w_in + (size_t)seq[t]->id[e] * 4 * H;
            const float f = seq[t]->f[e];
            for (int k = 0; k < 4 * H; ++k) a[k] += f * row[k];
          }
      } else {
        const float* x = z.hs.data() + idx(q, t, l - 1);
        const float* w = P + q->off[l].w_in;
        for (int k = 0; k < 4 * H; ++k) {
          float s = 0.f;
#pragma omp simd reduction(+ : s)
          for (int j = 0; j < H; ++j) s += w[(size_t)k * H + j] * x[j];
          a[k] += s;
        }
      }
      if (t > 0) {
        const float* hp = z.hs.data() + idx(q, t - 1, l);
        const float* w = P + q->off[l].w_hh;
        for (int k = 0; k < 4 * H; ++k) {
          float s = 0.f;
#pragma omp simd reduction(+ : s)
          for (int j = 0; j < H; ++j) s += w[(size_t)k * H + j] * hp[j];
          a[k] += s;
        }
      }
      const size_t o = idx(q, t, l);
      for (int j = 0; j < H; ++j) {
        const float i_ = sigmoidf(a[j]), f_ = sigmoidf(a[H + j]), g_ = std::tanh(a[2 * H + j]), o_ = sigmoidf(a[3 * H + j]);
        const float cp = t > 0 ? z.cs[idx(q, t - 1, l) + j] : 0.f;
        const float c = f_ * cp + i_ * g_;
        const float tch = std::tanh(c);
        z.gi[o + j] = i_; z.gf[o + j] = f_; z.gg[o + j] = g_; z.go[o + j] = o_;
        z.cs[o + j] = c; z.tc[o + j] = tch; z.hs[o + j] = o_ * tch;
      }
    }
  }
  const float* h = z.hs.data() + idx(q, W - 1, L - 1);
  const float* w = P + q->w_fc;
  const float* b = P + q->b_fc;
  for (int i = 0; i < n; ++i) {
    float s = 0.f;
#pragma omp simd reduction(+ : s)
    for (int j = 0; j < H; ++j) s += w[(size_t)i * H + j] * h[j];
    z.logits[i] = s + b[i];
  }
}

// Eq. 2 on the logits of the last forward pass; target: ascending ids of the adapters accessed.
float loss_of(const plora_predictor* q, const Scratch& z, const Sparse* target) {
  double s = 0.0;
  size_t e = 0;
  for (int i = 0; i < q->n; ++i) {
    const float zi = z.logits[i];
    const bool y = target && e < target->id.size() && target->id[e] == i;
    if (y) ++e;
    s += std::max(zi, 0.f) + std::log1p(std::exp(-std::fabs(zi))) - (y ? zi : 0.f);
  }
  return (float)s;
}

// Backward pass of the last forward pass in z: adds scale * dLoss/dparams to z.g.
void backward(const plora_predictor* q, Scratch& z, const Sparse* const* seq, const Sparse* target, float scale) {
  const int H = q->H, L = q->L, W = q->W, n = q->n;
  const float* P = q->p.data();
  float* G = z.g.data();
  size_t e = 0;
  for (int i = 0; i < n; ++i) {
    const bool y = target && e < target->id.size() && target->id[e] == i;
    if (y) ++e;
    z.dz[i] = scale * (sigmoidf(z.logits[i]) - (y ? 1.f : 0.f));
  }
  std::fill(z.dh.begin(), z.dh.end(), 0.f);  // [L][H]: from step t + 1
  std::fill(z.dc.begin(), z.dc.end(), 0.f);
  {  // output layer
    const float* h = z.hs.data() + idx(q, W - 1, L - 1);
    float* dht = z.dh.data() + (size_t)(L - 1) * H;
    for (int i = 0; i < n; ++i) {
      const float d = z.dz[i];
      G[q->b_fc + i] += d;
      float* gw = G + q->w_fc + (size_t)i * H;
      const float* w = P + q->w_fc + (size_t)i * H;
      for (int j = 0; j < H; ++j) { gw[j] += d * h[j]; dht[j] += d * w[j]; }
    }
  }
  for (int t = W - 1; t >= 0; --t) {
    std::fill(z.dh_up.begin(), z.dh_up.end(), 0.f);  // [L][H]: from the layer above at this step
    for (int l = L - 1; l >= 0; --l) {
      const size_t o = idx(q, t, l);
      float* dh = z.dh.data() + (size_t)l * H;
      float* dc = z.dc.data() + (size_t)l * H;
      const float* up = z.dh_up.data() + (size_t)l * H;
      float* da = z.da.data();
      for (int j = 0; j < H; ++j) {
        const float dht = dh[j] + up[j];
        const float i_ = z.gi[o + j], f_ = z.gf[o + j], g_ = z.gg[o + j], o_ = z.go[o + j], tch = z.tc[o + j];
        const float cp = t > 0 ? z.cs[idx(q, t - 1, l) + j] : 0.f;
        const float dct = dc[j] + dht * o_ * (1.f - tch * tch);
        da[j] = dct * g_ * i_ * (1.f - i_);
        da[H + j] = dct * cp * f_ * (1.f - f_);
        da[2 * H + j] = dct * i_ * (1.f - g_ * g_);
        da[3 * H + j] = dht * tch * o_ * (1.f - o_);
        dc[j] = dct * f_;
      }
      float* gb = G + q->off[l].b;
      for (int k = 0; k < 4 * H; ++k) gb[k] += da[k];
      // recurrent weights and the gradient that flows to step t - 1
      std::fill(dh, dh + H, 0.f);
      if (t > 0) {
        const float* hp = z.hs.data() + idx(q, t - 1, l);
        const float* w = P + q->off[l].w_hh;
        float* gw = G + q->off[l].w_hh;
        for (int k = 0; k < 4 * H; ++k) {
          const float d = da[k];
          for (int j = 0; j < H; ++j) { gw[(size_t)k * H + j] += d * hp[j]; dh[j] += d * w[(size_t)k * H + j]; }
        }
      }
      // input weights
      if (l == 0) {
        if (seq[t])
          for (size_t s = 0; s < seq[t]->id.size(); ++s) {
            float* row = G + q->off[0].w_in + (size_t)seq[t]->id[s] * 4 * H;
            const float f = seq[t]->f[s];
            for (int k = 0; k < 4 * H; ++k) row[k] += f * da[k];
          }
      } else {
        const float* x = z.hs.data() + idx(q, t, l - 1);
        const float* w = P + q->off[l].w_in;
        float* gw = G + q->off[l].w_in;
        float* below = z.dh_up.data() + (size_t)(l - 1) * H;
        for (int k = 0; k < 4 * H; ++k) {
          const float d = da[k];
          for (int j = 0; j < H; ++j) { gw[(size_t)k * H + j] += d * x[j]; below[j] += d * w[(size_t)k * H + j]; }
        }
      }
    }
  }
}

// The window of W intervals that ends just before replay position `end` (0 < end <= size): entries
// before the start of the buffer are empty intervals.
void window_before(const plora_predictor* q, size_t end, std::vector<const Sparse*>& seq) {
  seq.assign(q->W, nullptr);
  for (int k = 0; k < q->W; ++k) {
    const int64_t pos = (int64_t)end - q->W + k;
    if (pos >= 0) seq[k] = &q->replay[(size_t)pos];
  }
}

// Runs fn(worker) on `workers` threads (the caller is worker 0) and waits for all of them.
template <typename F>
void run_workers(int workers, F fn) {
  std::vector<std::thread> th;
  for (int t = 1; t < workers; ++t) th.emplace_back(fn, t);
  fn(0);
  for (auto& x : th) x.join();
}

void alloc_scratch(const plora_predictor* q, Scratch& z) {
  const size_t s = (size_t)q->W * q->L * q->H;
  for (auto* vec : {&z.gi, &z.gf, &z.gg, &z.go, &z.cs, &z.hs, &z.tc}) vec->assign(s, 0.f);
  z.logits.assign(q->n, 0.f); z.dz.assign(q->n, 0.f); z.da.assign(4 * (size_t)q->H, 0.f);
  z.dh.assign((size_t)q->L * q->H, 0.f); z.dc.assign((size_t)q->L * q->H, 0.f); z.dh_up.assign((size_t)q->L * q->H, 0.f);
  z.g.assign(q->p.size(), 0.f);
}

// Sums the workers' gradients (in worker order, so the result does not depend on timing), clears
// them, and applies one Adam update; every thread takes one slice of the parameter vector.
void reduce_and_adam(plora_predictor* q, int workers) {
  const float b1 = q->cfg.beta1, b2 = q->cfg.beta2, lr = q->cfg.lr, eps = q->cfg.eps;
  q->adam_t++;
  const double c1 = 1.0 - std::pow((double)b1, (double)q->adam_t), c2 = 1.0 - std::pow((double)b2, (double)q->adam_t);
  const float i1 = (float)(1.0 / c1), i2 = (float)(1.0 / c2);
  const size_t np = q->p.size();
  run_workers(workers, [&](int t) {
    const size_t lo = np * (size_t)t / workers, hi = np * (size_t)(t + 1) / workers;
    float* g0 = q->scr[0].g.data();
    for (int w = 1; w < workers; ++w) {
      float* gw = q->scr[w].g.data();
      for (size_t k = lo; k < hi; ++k) { g0[k] += gw[k]; gw[k] = 0.f; }
    }
    float* P = q->p.data();
    float* M = q->m.data();
    float* V = q->v.data();
    for (size_t k = lo; k < hi; ++k) {
      const float gk = g0[k];
      const float mk = b1 * M[k] + (1.f - b1) * gk;
      const float vk = b2 * V[k] + (1.f - b2) * gk * gk;
      M[k] = mk; V[k] = vk;
      P[k] -= lr * (mk * i1) / (std::sqrt(vk * i2) + eps);
      g0[k] = 0.f;
    }
  });
}

}  // namespace

extern "C" {

int plora_predictor_create(const plora_predictor_config* c, plora_predictor** out) {
  if (!c || !out) return PLORA_ERR_INVAL;
  if (c->n_adapters < 1 || c->window < 1 || c->window > 1024 || c->hidden < 1 || c->hidden > 1024 || c->layers < 1 ||
      c->layers > 8 || c->replay < 2 || c->batch < 1)
    return PLORA_ERR_INVAL;
  if (!(c->lr > 0.f) || !(c->beta1 >= 0.f && c->beta1 < 1.f) || !(c->beta2 >= 0.f && c->beta2 < 1.f) || !(c->eps > 0.f))
    return PLORA_ERR_INVAL;
  plora_predictor* q = new (std::nothrow) plora_predictor;
  if (!q) return PLORA_ERR_NOMEM;
  q->cfg = *c;
  q->n = c->n_adapters; q->H = c->hidden; q->L = c->layers; q->W = c->window;
  const size_t n = q->n, H = q->H;
  size_t o = 0;
  for (int l = 0; l < q->L; ++l) {
    plora_predictor::Off f;
    f.w_in = o; o += l == 0 ? n * 4 * H : 4 * H * H;
    f.w_hh = o; o += 4 * H * H;
    f.b = o; o += 4 * H;
    q->off.push_back(f);
  }
  q->w_fc = o; o += n * H;
  q->b_fc = o; o += n;
  q->p.assign(o, 0.f); q->m.assign(o, 0.f); q->v.assign(o, 0.f);
  // uniform in (-1/sqrt(H), 1/sqrt(H)), the usual LSTM initialisation; biases start at 0
  const float a = 1.0f / std::sqrt((float)H);
  for (size_t k = 0; k < o; ++k) {
    const bool bias = k >= q->b_fc;
    bool lstm_bias = false;
    for (int l = 0; l < q->L; ++l) lstm_bias |= k >= q->off[l].b && k < q->off[l].b + 4 * H;
    if (bias || lstm_bias) continue;
    const double u = (double)(mix64(c->seed ^ (0xA5A5ULL << 32) ^ k) >> 11) * (1.0 / 9007199254740992.0);
    q->p[k] = (float)((2.0 * u - 1.0) * a);
  }
  q->scr.resize(1);
  alloc_scratch(q, q->scr[0]);
  *out = q;
  return PLORA_OK;
}

int plora_predictor_destroy(plora_predictor* q) {
  if (!q) return PLORA_ERR_INVAL;
  delete q;
  return PLORA_OK;
}

int plora_predictor_observe(plora_predictor* q, const int32_t* ids, int32_t n_ids) {
  if (!q || n_ids < 0 || (n_ids > 0 && !ids)) return PLORA_ERR_INVAL;
  for (int32_t k = 0; k < n_ids; ++k)
    if (ids[k] < 0 || ids[k] >= q->n) return PLORA_ERR_INVAL;
  std::vector<int32_t> s(ids, ids + n_ids);
  std::sort(s.begin(), s.end());
  Sparse sp;
  for (size_t k = 0; k < s.size();) {
    size_t e = k;
    while (e < s.size() && s[e] == s[k]) ++e;
    const float c = (float)(e - k);
    sp.id.push_back(s[k]);
    sp.f.push_back(c / (1.0f + c));
    k = e;
  }
  q->replay.push_back(std::move(sp));
  while ((int64_t)q->replay.size() > (int64_t)q->cfg.replay) q->replay.pop_front();
  return PLORA_OK;
}

int64_t plora_predictor_observed(const plora_predictor* q) { return q ? (int64_t)q->replay.size() : PLORA_ERR_INVAL; }

int plora_predictor_predict(plora_predictor* q, float* p_hat) {
  if (!q || !p_hat) return PLORA_ERR_INVAL;
  std::vector<const Sparse*> seq;
  window_before(q, q->replay.size(), seq);
  forward(q, q->scr[0], seq.data());
  for (int i = 0; i < q->n; ++i) p_hat[i] = sigmoidf(q->scr[0].logits[i]);
  return PLORA_OK;
}

int plora_predictor_train_batch(plora_predictor* q, const int32_t* target_pos, int32_t n_samples, float* mean_loss) {
  if (!q || !target_pos || n_samples < 1) return PLORA_ERR_INVAL;
  for (int32_t k = 0; k < n_samples; ++k)
    if (target_pos[k] < 1 || (size_t)target_pos[k] >= q->replay.size()) return PLORA_ERR_INVAL;
  // sample k goes to worker k % workers; every worker's gradient buffer is all zeros on entry
  const int workers = std::max(1, std::min(q->threads, (int)n_samples));
  const float scale = 1.0f / (float)n_samples;
  run_workers(workers, [&](int t) {
    Scratch& z = q->scr[t];
    z.loss = 0.0;
    std::vector<const Sparse*> seq;
    for (int32_t k = t; k < n_samples; k += workers) {
      window_before(q, (size_t)target_pos[k], seq);
      forward(q, z, seq.data());
      const Sparse* y = &q->replay[(size_t)target_pos[k]];
      z.loss += loss_of(q, z, y);
      backward(q, z, seq.data(), y, scale);
    }
  });
  double total = 0.0;
  for (int t = 0; t < workers; ++t) total += q->scr[t].loss;
  reduce_and_adam(q, workers);
  if (mean_loss) *mean_loss = (float)(total / n_samples);
  return PLORA_OK;
}

int plora_predictor_train(plora_predictor* q, int32_t steps, float* mean_loss) {
  if (!q || steps < 0) return PLORA_ERR_INVAL;
  if (q->replay.size() < 2) { if (mean_loss) *mean_loss = 0.f; return PLORA_OK; }  // nothing to learn from yet
  std::vector<int32_t> pos(q->cfg.batch);
  double total = 0.0;
  for (int32_t s = 0; s < steps; ++s) {
    for (int32_t k = 0; k < q->cfg.batch; ++k)
      pos[k] = 1 + (int32_t)(mix64(q->cfg.seed + 0x51ED270BULL * (q->draws++)) % (q->replay.size() - 1));
    float l = 0.f;
    const int rc = plora_predictor_train_batch(q, pos.data(), q->cfg.batch, &l);
    if (rc != PLORA_OK) return rc;
    total += l;
  }
  if (mean_loss) *mean_loss = steps ? (float)(total / steps) : 0.f;
  return PLORA_OK;
}

int plora_predictor_set_threads(plora_predictor* q, int32_t threads) {
  if (!q || threads < 1 || threads > 64) return PLORA_ERR_INVAL;
  const size_t old = q->scr.size();
  if ((size_t)threads > old) {
    q->scr.resize(threads);
    for (size_t t = old; t < (size_t)threads; ++t) alloc_scratch(q, q->scr[t]);
  }
  q->threads = threads;
  return PLORA_OK;
}

int64_t plora_predictor_param_count(const plora_predictor* q) { return q ? (int64_t)q->p.size() : PLORA_ERR_INVAL; }

int plora_predictor_get_params(const plora_predictor* q, float* out) {
  if (!q || !out) return PLORA_ERR_INVAL;
  std::memcpy(out, q->p.data(), q->p.size() * sizeof(float));
  return PLORA_OK;
}

int plora_predictor_set_params(plora_predictor* q, const float* in) {
  if (!q || !in) return PLORA_ERR_INVAL;
  std::memcpy(q->p.data(), in, q->p.size() * sizeof(float));
  return PLORA_OK;
}

int plora_predictor_loss_grad(plora_predictor* q, const float* seq_dense, const float* target, float* loss, float* grad) {
  if (!q || !seq_dense || !target) return PLORA_ERR_INVAL;
  std::vector<Sparse> win(q->W);
  std::vector<const Sparse*> seq(q->W);
  for (int t = 0; t < q->W; ++t) {
    for (int i = 0; i < q->n; ++i) {
      const float f = seq_dense[(size_t)t * q->n + i];
      if (f != 0.f) { win[t].id.push_back(i); win[t].f.push_back(f); }
    }
    seq[t] = &win[t];
  }
  Sparse y;
  for (int i = 0; i < q->n; ++i) {
    if (target[i] != 0.f && target[i] != 1.f) return PLORA_ERR_INVAL;
    if (target[i] == 1.f) y.id.push_back(i);
  }
  Scratch& z = q->scr[0];
  forward(q, z, seq.data());
  if (loss) *loss = loss_of(q, z, &y);
  if (grad) {
    backward(q, z, seq.data(), &y, 1.0f);  // the buffer is all zeros between calls
    std::memcpy(grad, z.g.data(), z.g.size() * sizeof(float));
    std::fill(z.g.begin(), z.g.end(), 0.f);
  }
  return PLORA_OK;
}

}  // extern "C"
