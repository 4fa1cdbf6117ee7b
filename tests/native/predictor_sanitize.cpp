// The traffic predictor under AddressSanitizer / UBSan: random intervals observed, predictions and
// training steps interleaved, buffer limit exceeded, tiny and odd sizes.  No GPU call is involved.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "plora.h"

#define CHECK(c) do { if (!(c)) { std::printf("CHECK failed at line %d: %s\n", __LINE__, #c); std::exit(1); } } while (0)

int main() {
  std::mt19937 rng(99);
  const int shapes[4][4] = {{1, 1, 1, 1}, {7, 3, 5, 2}, {33, 8, 16, 3}, {300, 4, 64, 2}};  // n, window, hidden, layers
  for (const auto& s : shapes) {
    plora_predictor_config c{s[0], s[1], s[2], s[3], 12, 5, 1e-3f, 0.9f, 0.999f, 1e-8f, 42};
    plora_predictor* q = nullptr;
    CHECK(plora_predictor_create(&c, &q) == PLORA_OK);
    CHECK(plora_predictor_set_threads(q, 1 + s[0] % 4) == PLORA_OK);
    std::vector<float> p_hat(s[0]);
    for (int step = 0; step < 60; ++step) {
      std::vector<int32_t> ids(rng() % 9);
      for (auto& i : ids) i = (int32_t)(rng() % s[0]);
      CHECK(plora_predictor_predict(q, p_hat.data()) == PLORA_OK);
      for (float p : p_hat) CHECK(p >= 0.f && p <= 1.f && std::isfinite(p));
      CHECK(plora_predictor_observe(q, ids.data(), (int32_t)ids.size()) == PLORA_OK);
      CHECK(plora_predictor_observed(q) <= 12);
      float loss = -1.f;
      CHECK(plora_predictor_train(q, 1 + step % 2, &loss) == PLORA_OK);
      CHECK(std::isfinite(loss) && loss >= 0.f);
    }
    std::vector<float> params((size_t)plora_predictor_param_count(q)), grad(params.size());
    CHECK(plora_predictor_get_params(q, params.data()) == PLORA_OK);
    for (float v : params) CHECK(std::isfinite(v));
    std::vector<float> seq((size_t)s[1] * s[0], 0.5f), tgt(s[0], 1.f);
    float loss = 0.f;
    CHECK(plora_predictor_loss_grad(q, seq.data(), tgt.data(), &loss, grad.data()) == PLORA_OK);
    tgt[0] = 0.5f;
    CHECK(plora_predictor_loss_grad(q, seq.data(), tgt.data(), &loss, nullptr) == PLORA_ERR_INVAL);
    CHECK(plora_predictor_destroy(q) == PLORA_OK);
  }
  std::printf("predictor sanitize run OK\n");
  return 0;
}
