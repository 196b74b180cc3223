// Host-side exercise of the C ABI's argument layer for a build with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code (no GPU is touched: every call below either fails
// its argument checks on the host or is a host-only query).  Built and run by
// tests/test_host_sanitizers.py; exits 0 when every check holds and the sanitizers stay quiet.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "zeno.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
      return 1;                                                            \
    }                                                                      \
  } while (0)

static zeno_model_t* make(const std::vector<int>& dims, int bias, int loss, int fwd) {
  zeno_model_desc_t d;
  std::memset(&d, 0, sizeof(d));
  d.n_layers = (int)dims.size() - 1;
  for (size_t i = 0; i < dims.size(); ++i) d.dims[i] = dims[i];
  d.has_bias = bias;
  d.loss = loss;
  d.fwd = fwd;
  zeno_model_t* m = nullptr;
  return zeno_model_create(&d, &m) == ZENO_OK ? m : nullptr;
}

int main() {
  // model creation: good and bad descriptors
  CHECK(zeno_model_create(nullptr, nullptr) == ZENO_ERR_INVALID_ARG);
  zeno_model_desc_t bad;
  std::memset(&bad, 0, sizeof(bad));
  zeno_model_t* out = nullptr;
  bad.n_layers = ZENO_MAX_LAYERS + 1;
  CHECK(zeno_model_create(&bad, &out) == ZENO_ERR_INVALID_ARG);
  bad.n_layers = 2;
  bad.dims[0] = 4; bad.dims[1] = 0; bad.dims[2] = 3;
  CHECK(zeno_model_create(&bad, &out) == ZENO_ERR_INVALID_ARG);
  CHECK(make({4, 3}, 1, ZENO_LOSS_SQUARED, ZENO_FWD_FP32) == nullptr);   // squared loss needs width 1
  zeno_model_destroy(nullptr);

  const std::vector<std::vector<int>> shapes = {{64, 1}, {784, 10}, {3072, 512, 10}, {3072, 2048, 2048, 10},
                                               {4096, 4096, 4096, 4096, 1000}, {300, 129, 65, 33, 7},
                                               {64, 128, 64, 32, 16, 8, 4, 3, 2}};
  for (const auto& dims : shapes) {
    for (int fwd = 0; fwd < 2; ++fwd) {
      const int loss = dims.back() == 1 ? ZENO_LOSS_SQUARED : ZENO_LOSS_SOFTMAX_CE;
      zeno_model_t* m = make(dims, 1, loss, fwd);
      CHECK(m != nullptr);
      long long d = 0;
      for (size_t l = 1; l < dims.size(); ++l) d += (long long)dims[l] * dims[l - 1] + dims[l];
      CHECK(zeno_model_num_params(m) == d);
      for (int mm : {1, 7, 60, 100, 1024})
        for (int n_r : {1, 32, 33, 128, 300}) {
          CHECK(zeno_score_workspace_bytes(m, mm, n_r) > 0);
          CHECK(zeno_score_workspace_bytes(m, mm, n_r) % 256 == 0);
          CHECK(zeno_score_plan_check(m, mm, n_r) == ZENO_OK);
        }
      CHECK(zeno_score_workspace_bytes(m, 0, 4) == 0 && zeno_score_workspace_bytes(m, ZENO_MAX_CANDIDATES + 1, 4) == 0);
      CHECK(zeno_score_plan_check(m, 4, 0) == ZENO_ERR_INVALID_ARG);

      // zeno_score / zeno_score_static: every argument error is caught on the host.  The pointers below are
      // never dereferenced by a call that fails its checks.
      float dummy[64];
      int32_t labels[4] = {0, 0, 0, 0};
      zeno_batch_t b;
      std::memset(&b, 0, sizeof(b));
      b.n_r = 4;
      b.features = dummy;
      b.labels = labels;
      b.targets = dummy;
      CHECK(zeno_score(m, nullptr, dummy, d, 4, &b, 0.1f, 0.1f, dummy, dummy, 1 << 20, nullptr) == ZENO_ERR_INVALID_ARG);
      CHECK(zeno_score(m, dummy, dummy, d - 1, 4, &b, 0.1f, 0.1f, dummy, dummy, 1 << 20, nullptr) == ZENO_ERR_INVALID_ARG);
      CHECK(zeno_score(m, dummy, dummy, d, 0, &b, 0.1f, 0.1f, dummy, dummy, 1 << 20, nullptr) == ZENO_ERR_INVALID_ARG);
      CHECK(zeno_score(m, dummy, dummy, d, 4, &b, -1.f, 0.1f, dummy, dummy, 1 << 20, nullptr) == ZENO_ERR_INVALID_ARG);
      CHECK(zeno_score(m, dummy, dummy, d, 4, &b, 0.1f, 0.1f, dummy, nullptr, 0, nullptr) == ZENO_ERR_WORKSPACE);
      CHECK(zeno_score(m, dummy, dummy, d, 4, &b, 0.1f, 0.1f, dummy, dummy, 16, nullptr) == ZENO_ERR_WORKSPACE);
      CHECK(zeno_score(m, dummy, reinterpret_cast<float*>(reinterpret_cast<char*>(dummy) + 1), d, 4, &b, 0.1f, 0.1f, dummy,
                       dummy, 1 << 20, nullptr) == ZENO_ERR_INVALID_ARG);
      CHECK(zeno_score_static(m, dummy, dummy, d, 4, nullptr, 0.1f, 0.1f, dummy, nullptr) == ZENO_ERR_INVALID_ARG);
      b.n_r = 0;
      CHECK(zeno_score_static(m, dummy, dummy, d, 4, &b, 0.1f, 0.1f, dummy, nullptr) == ZENO_ERR_INVALID_ARG);
      zeno_model_destroy(m);
    }
  }

  float g[32], o[8];
  int32_t sel[8];
  CHECK(zeno_aggregate(nullptr, 8, g, 4, 8, 1, o, sel, nullptr) == ZENO_ERR_INVALID_ARG);
  CHECK(zeno_aggregate(g, 8, g, 4, 8, 4, o, sel, nullptr) == ZENO_ERR_INVALID_ARG);      // b >= m
  CHECK(zeno_aggregate(g, 7, g, 4, 8, 1, o, sel, nullptr) == ZENO_ERR_INVALID_ARG);      // ldg < d
  CHECK(zeno_aggregate_update(g, 8, g, 4, 8, 1, 0.1f, nullptr, o, o, sel, nullptr) == ZENO_ERR_INVALID_ARG);
  CHECK(zeno_mean(g, 8, 0, 8, o, nullptr) == ZENO_ERR_INVALID_ARG);
  CHECK(zeno_median(g, 8, 4, 0, o, nullptr) == ZENO_ERR_INVALID_ARG);
  CHECK(zeno_krum(g, 8, 4, 8, 2, o, sel, nullptr, g, 1 << 20, nullptr) == ZENO_ERR_INVALID_ARG);   // m - b - 2 < 1
  CHECK(zeno_krum_workspace_bytes(2) == 0 && zeno_krum_workspace_bytes(129) == 0);
  CHECK(std::strcmp(zeno_status_string(ZENO_OK), "ok") == 0);
  CHECK(std::strcmp(zeno_status_string(99), "unknown status") == 0);
  CHECK(zeno_profile_collect(nullptr, 0) == 0);
  std::puts("host checks passed");
  return 0;
}
