// Host-side exercise of the C ABI for a sanitizer build (AddressSanitizer + UndefinedBehaviorSanitizer on the host
// code of csrc/api.hip; no GPU is needed and none is touched): every size query over a sweep of configurations, every
// compute entry point with arguments it must refuse before any launch, empty inputs, the host-side penalty-weight
// feedback (Algorithm 1) and the status strings.  Exit status 0 = every call returned what the header promises;
// a sanitizer report aborts the run.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ltea.h"

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } } while (0)

static void* fake(uintptr_t a = 0x10000) { return reinterpret_cast<void*>(a); }

static ltea_cfg make_cfg(int Hq, int Hkv, int D, int window, int budget, int sink, int dtype) {
  ltea_cfg c;
  std::memset(&c, 0, sizeof(c));
  c.Hq = Hq; c.Hkv = Hkv; c.D = D; c.window = window; c.budget = budget; c.sink = sink;
  c.tau_logit = 0.f; c.softmax_scale = 0.f; c.dtype = dtype;
  return c;
}

static ltea_cnn make_cnn(int L, const int* ks, const int* dil, const int* co) {
  ltea_cnn c;
  std::memset(&c, 0, sizeof(c));
  c.n_layers = L;
  for (int l = 0; l < L && l < LTEA_MAX_CNN_LAYERS; ++l) {
    c.kernel[l] = ks[l]; c.dilation[l] = dil[l]; c.c_out[l] = co[l];
    c.w[l] = fake(); c.bias[l] = static_cast<const float*>(fake());
  }
  c.w_out = fake(); c.b_out = static_cast<const float*>(fake());
  return c;
}

static ltea_cache fake_cache() {
  ltea_cache c;
  c.k_win = c.v_win = c.k_ret = c.v_ret = fake();
  c.win_score = c.ret_score = static_cast<float*>(fake());
  c.ret_pos = c.ret_count = c.n_seen = c.n_scored = static_cast<int32_t*>(fake());
  return c;
}

int main() {
  long calls = 0;
  // ---- size queries over a sweep of configurations (host arithmetic only) ----------------------------------------
  const int stacks[][3][4] = {
      {{5}, {1}, {32}}, {{7}, {1}, {32}}, {{3}, {2}, {16}}, {{1}, {1}, {8}},
      {{3, 3, 3}, {2, 2, 2}, {64, 32, 16}}, {{5, 3}, {1, 2}, {32, 16}}, {{3, 3, 3, 3}, {1, 2, 4, 8}, {64, 64, 32, 16}},
      {{7, 7}, {4, 4}, {48, 24}}};
  const int layers[] = {1, 1, 1, 1, 3, 2, 4, 2};
  for (int dtype = 0; dtype < 2; ++dtype)
    for (int D : {64, 128})
      for (int s = 0; s < 8; ++s)
        for (int window : {64, 512, 2048})
          for (int budget : {0, 33, 1024})
            for (int n_seqs : {1, 4, 300})
              for (int64_t total : {(int64_t)1, (int64_t)5000, (int64_t)3 << 20}) {
                ltea_cfg cfg = make_cfg(8, 2, D, window, budget, 4, dtype);
                ltea_cnn cnn = make_cnn(layers[s], stacks[s][0], stacks[s][1], stacks[s][2]);
                const int32_t max_len = (int32_t)(total < 100000 ? total : 100000);
                volatile size_t sink = 0;
                sink += ltea_workspace_bytes(&cfg, &cnn, n_seqs, total, max_len);
                sink += ltea_workspace_bytes(&cfg, nullptr, n_seqs, total, max_len);
                sink += ltea_decode_workspace_bytes(&cfg, &cnn, n_seqs);
                sink += ltea_decode_workspace_bytes(&cfg, nullptr, n_seqs);
                sink += ltea_append_workspace_bytes(&cfg, &cnn, n_seqs, total, max_len);
                sink += ltea_rescore_workspace_bytes(&cfg, &cnn, n_seqs);
                sink += ltea_decode_feat_workspace_bytes(&cfg, &cnn, n_seqs);
                sink += ltea_train_workspace_bytes(&cfg, &cnn, n_seqs, total, max_len);
                sink += ltea_cnn_backward_workspace_bytes(&cfg, &cnn, total);
                sink += ltea_cnn_panels_bytes(&cfg, &cnn);
                sink += (size_t)ltea_lazy_period(&cfg, &cnn);
                calls += 11;
              }
  // degenerate and hostile structures: the queries must not read past the arrays or overflow
  {
    ltea_cfg cfg = make_cfg(8, 2, 64, 512, 256, 0, LTEA_BF16);
    const int ks[] = {5, 5, 5, 5}, dil[] = {1, 1, 1, 1}, co[] = {32, 32, 32, 32};
    for (int L : {-3, 0, 5, 1000, INT32_MAX}) {
      ltea_cnn cnn = make_cnn(4, ks, dil, co);
      cnn.n_layers = L;
      (void)ltea_workspace_bytes(&cfg, &cnn, 4, 1000, 500);
      (void)ltea_decode_workspace_bytes(&cfg, &cnn, 4);
      (void)ltea_cnn_panels_bytes(&cfg, &cnn);
      (void)ltea_lazy_period(&cfg, &cnn);
      EXPECT(ltea_score(&cfg, &cnn, fake(), fake(), 128, 64, static_cast<const int32_t*>(fake()), 1, 32, 32,
                        static_cast<float*>(fake()), fake(), (size_t)1 << 30, nullptr) == LTEA_EINVAL);
      calls += 5;
    }
    ltea_cnn cnn = make_cnn(1, ks, dil, co);
    for (int big : {INT32_MAX, INT32_MAX - 1, 1 << 30}) {
      ltea_cfg c2 = make_cfg(big, big, 64, big, big, big, LTEA_BF16);
      (void)ltea_workspace_bytes(&c2, &cnn, INT32_MAX, INT64_MAX / 4, INT32_MAX);
      (void)ltea_decode_workspace_bytes(&c2, &cnn, INT32_MAX);
      (void)ltea_append_workspace_bytes(&c2, &cnn, INT32_MAX, INT64_MAX / 4, INT32_MAX);
      (void)ltea_train_workspace_bytes(&c2, &cnn, INT32_MAX, INT64_MAX / 4, INT32_MAX);
      (void)ltea_rescore_workspace_bytes(&c2, &cnn, INT32_MAX);
      (void)ltea_cnn_backward_workspace_bytes(&c2, &cnn, INT64_MAX / 4);
      calls += 6;
    }
    (void)ltea_workspace_bytes(nullptr, &cnn, 1, 1, 1);
    (void)ltea_decode_workspace_bytes(nullptr, nullptr, 1);
    (void)ltea_lazy_period(nullptr, nullptr);
    calls += 3;
  }
  // ---- entry points must refuse these before any launch -----------------------------------------------------------
  {
    const int ks[] = {5}, dil[] = {1}, co[] = {16};
    ltea_cfg cfg = make_cfg(4, 2, 64, 16, 8, 0, LTEA_BF16);
    ltea_cnn cnn = make_cnn(1, ks, dil, co);
    ltea_cache cache = fake_cache();
    const int32_t* cu = static_cast<const int32_t*>(fake());
    float* fl = static_cast<float*>(fake());
    const size_t big = (size_t)1 << 30;
    EXPECT(ltea_score(nullptr, &cnn, fake(), fake(), 128, 64, cu, 1, 32, 32, fl, fake(), big, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_score(&cfg, nullptr, fake(), fake(), 128, 64, cu, 1, 32, 32, fl, fake(), big, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_score(&cfg, &cnn, nullptr, fake(), 128, 64, cu, 1, 32, 32, fl, fake(), big, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_score(&cfg, &cnn, fake(), fake(), 127, 64, cu, 1, 32, 32, fl, fake(), big, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_score(&cfg, &cnn, fake(), fake(), 128, 64, cu, 1, 32, 32, fl, nullptr, 0, nullptr) == LTEA_EWORKSPACE);
    EXPECT(ltea_score(&cfg, &cnn, fake(), fake(), 128, 64, cu, 1, -1, 32, fl, fake(), big, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_score(&cfg, &cnn, fake(), fake(), (int64_t)1 << 21, 64, cu, 1, 32, 32, fl, fake(), big, nullptr) == LTEA_EUNSUPPORTED);
    EXPECT(ltea_retain(&cfg, nullptr, fake(), fake(), 128, 64, cu, 1, 32, 32, 2, &cache, nullptr, 0, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_retain(&cfg, fl, fake(), fake(), 128, 64, cu, 1, 32, 32, 2, nullptr, nullptr, 0, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_sparse_attention(&cfg, nullptr, 256, 64, fake(), fake(), 128, 64, cu, 1, 32, 32, &cache, fake(), nullptr, 0, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_decode_step(&cfg, &cnn, nullptr, fake(), fake(), fake(), &cache, 1, fake(), big, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_decode_step(&cfg, &cnn, fake(), fake(), fake(), fake(), &cache, 1, nullptr, 0, nullptr) == LTEA_EWORKSPACE);
    EXPECT(ltea_decode_step(&cfg, &cnn, fake(), fake(), fake(), fake(), &cache, -1, fake(), big, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_decode_step_static(&cfg, &cnn, nullptr, fake(), fake(), fake(), &cache, 1, nullptr) == LTEA_EINVAL);
    EXPECT(ltea_decode_step_static(&cfg, &cnn, fake(), fake(), fake(), fake(), &cache, 1 << 20, nullptr) == LTEA_EWORKSPACE);
    ltea_cfg bad = cfg;
    bad.D = 96;
    EXPECT(ltea_score(&bad, &cnn, fake(), fake(), 128, 64, cu, 1, 32, 32, fl, fake(), big, nullptr) == LTEA_EUNSUPPORTED);
    bad = cfg;
    bad.dtype = 7;
    EXPECT(ltea_score(&bad, &cnn, fake(), fake(), 128, 64, cu, 1, 32, 32, fl, fake(), big, nullptr) == LTEA_EINVAL);
    bad = cfg;
    bad.Hq = 5;
    EXPECT(ltea_decode_step(&bad, &cnn, fake(), fake(), fake(), fake(), &cache, 1, fake(), big, nullptr) == LTEA_EINVAL);
    // empty inputs are fine and touch nothing
    EXPECT(ltea_score(&cfg, &cnn, fake(), fake(), 128, 64, cu, 0, 0, 0, fl, fake(), big, nullptr) == LTEA_OK);
    EXPECT(ltea_decode_step(&cfg, &cnn, fake(), fake(), fake(), fake(), &cache, 0, nullptr, 0, nullptr) == LTEA_OK);
    calls += 21;
  }
  // ---- penalty-weight feedback on host arrays (Algorithm 1) --------------------------------------------------------
  {
    const int n = 1000;
    std::vector<float> lam(n), cbar(n);
    for (int i = 0; i < n; ++i) {
      lam[i] = i % 7 == 0 ? 0.f : std::ldexp(1.0f, -(i % 40));
      cbar[i] = (float)(i % 13) * 50.f;
    }
    for (int it = 0; it < 200; ++it) EXPECT(ltea_lambda_update(lam.data(), cbar.data(), n, 256.f, 1.05f) == LTEA_OK);
    for (int i = 0; i < n; ++i) EXPECT(lam[i] >= 0.f && lam[i] <= 1.f && (lam[i] == 0.f || lam[i] >= 1e-9f));
    EXPECT(ltea_lambda_update(nullptr, cbar.data(), n, 256.f, 1.05f) == LTEA_EINVAL);
    EXPECT(ltea_lambda_update(lam.data(), cbar.data(), -1, 256.f, 1.05f) == LTEA_EINVAL);
    EXPECT(ltea_lambda_update(lam.data(), cbar.data(), 0, 256.f, 1.05f) == LTEA_OK);
    calls += 204;
  }
  for (int s = -10; s <= 2; ++s) { EXPECT(ltea_strerror(s) != nullptr && std::strlen(ltea_strerror(s)) > 1); ++calls; }
  EXPECT(ltea_diag_sink_bytes() > 0);
  std::printf("%ld calls, %d failures\n", calls, failures);
  return failures == 0 ? 0 : 1;
}
