// Drives the C ABI of libmoonwalk on a machine without a GPU, for the AddressSanitizer / UBSan build of the
// library's host code (linked against fake_hip.cpp instead of the HIP runtime). Two parts: the argument
// validation that must answer before anything touches a device, and whole calls (setup, the gradient
// drivers, training step, refreshes, statistics, fetches, destroy) on small networks of every kind, which
// run all of the host-side planning: buffer plans, pointer tables, slot sharing between segments, fragment
// tables, image chunking. Kernels do not run, so no number is checked here; the sanitizers are the check.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/moonwalk.h"
#include "../../include/moonwalk_bench.h"

extern "C" unsigned long long fake_hip_launches();
extern "C" unsigned long long fake_hip_bad_launches();
extern "C" int fake_hip_pending_configurations();

static int g_failures = 0;
#define EXPECT(cond)                                                    \
  do {                                                                  \
    if (!(cond)) {                                                      \
      fprintf(stderr, "%s:%d: expectation failed: %s\n", __FILE__, __LINE__, #cond); \
      ++g_failures;                                                     \
    }                                                                   \
  } while (0)

static size_t g_live_blocks = 0;
static void* test_alloc(size_t bytes, void*) {
  ++g_live_blocks;
  return calloc(bytes ? bytes : 1, 1);
}
static void test_free(void* p, void*) {
  if (p) --g_live_blocks;
  free(p);
}
static int g_fail_after = -1;  // the allocator starts to fail after this many calls (< 0: never)
static void* failing_alloc(size_t bytes, void* ctx) {
  if (g_fail_after == 0) return nullptr;
  if (g_fail_after > 0) --g_fail_after;
  return test_alloc(bytes, ctx);
}

static mw_config_t base_config(int batch) {
  mw_config_t c;
  memset(&c, 0, sizeof(c));
  c.batch = batch;
  c.loss_scale = 1.f;
  c.fuse = 1;
  c.frag_capacity_factor = 1.0;
  c.dev_alloc = test_alloc;
  c.dev_free = test_free;
  return c;
}

static void validation() {
  mw_handle_t* h = nullptr;
  float* fake = reinterpret_cast<float*>(0x1000);  // never dereferenced: validation fails first
  mw_layer_t ok{8, 8, fake, nullptr, 0.1f};
  mw_config_t cfg = base_config(4);
  EXPECT(moonwalk_setup(nullptr, &ok, 1, &cfg, nullptr) == MW_ERR_INVALID_ARG);
  EXPECT(moonwalk_setup(&h, nullptr, 1, &cfg, nullptr) == MW_ERR_INVALID_ARG);
  EXPECT(moonwalk_setup(&h, &ok, 0, &cfg, nullptr) == MW_ERR_INVALID_ARG);
  EXPECT(moonwalk_setup(&h, &ok, 1, nullptr, nullptr) == MW_ERR_INVALID_ARG);
  mw_layer_t wide{8, 9, fake, nullptr, 0.1f};
  EXPECT(moonwalk_setup(&h, &wide, 1, &cfg, nullptr) == MW_ERR_NOT_SUBMERSIVE);
  mw_layer_t huge{32768, 16384, fake, nullptr, 0.1f};
  EXPECT(moonwalk_setup(&h, &huge, 1, &cfg, nullptr) == MW_ERR_INVALID_ARG);
  mw_config_t bad = cfg;
  bad.debug_keep = 3;
  EXPECT(moonwalk_setup(&h, &ok, 1, &bad, nullptr) == MW_ERR_INVALID_ARG);
  bad = cfg;
  bad.refresh_precision = 2;
  EXPECT(moonwalk_setup(&h, &ok, 1, &bad, nullptr) == MW_ERR_INVALID_ARG);
  bad = cfg;
  bad.batch = 1 << 30;
  EXPECT(moonwalk_setup(&h, &ok, 1, &bad, nullptr) == MW_ERR_INVALID_ARG);
  EXPECT(h == nullptr);
  EXPECT(moonwalk_grad(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == MW_ERR_INVALID_ARG);
  EXPECT(backprop_grad(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == MW_ERR_INVALID_ARG);
  EXPECT(moonwalk_memory_stats(nullptr, nullptr) == MW_ERR_INVALID_ARG);
  EXPECT(moonwalk_debug_fetch(nullptr, 0, MW_FETCH_MASK, nullptr, 0, nullptr) == MW_ERR_INVALID_ARG);
  moonwalk_destroy(nullptr);
  EXPECT(mw_gemm_f32(MW_GEMM_NT, 0, 1024, 64, 64, 1.f, fake, 64, fake, 64, 0.f, fake, 1 << 20, nullptr) == MW_ERR_INVALID_ARG);
  EXPECT(mw_colsum_wide_noalloc(fake, 2, (int32_t)mw_colsum_noalloc_max_floats() + 4, 1.f, fake, nullptr) == MW_ERR_TOO_LARGE);
  for (int code = -9; code <= 0; ++code) EXPECT(strlen(moonwalk_strerror(code)) > 1);
}

// One dense network through every entry point. widths: d_0 .. d_L.
static void dense_network(const std::vector<int>& widths, int batch, const std::vector<float>& alphas, int K, int S, int fuse,
                          int debug_keep, int plan, int group = 1, int overlap = 0, int refresh_precision = 0) {
  const int L = (int)widths.size() - 1;
  std::vector<std::vector<float>> W(L), b(L);
  std::vector<mw_layer_t> layers(L);
  for (int i = 0; i < L; ++i) {
    W[i].assign((size_t)widths[i + 1] * widths[i], 0.f);
    b[i].assign(widths[i + 1], 0.f);
    layers[i] = mw_layer_t{widths[i], widths[i + 1], W[i].data(), (i % 2) ? nullptr : b[i].data(), alphas[i]};
  }
  mw_config_t cfg = base_config(batch);
  cfg.reseed_interval = K;
  cfg.segment_length = S;
  cfg.fuse = fuse;
  cfg.debug_keep = debug_keep;
  cfg.plan = plan;
  cfg.phase3_parallel_segments = group;
  cfg.phase3_overlap = overlap;
  cfg.refresh_precision = refresh_precision;
  mw_handle_t* h = nullptr;
  const int rc = moonwalk_setup(&h, layers.data(), L, &cfg, nullptr);
  EXPECT(rc == MW_OK && h != nullptr);
  if (rc != MW_OK) return;
  size_t total = 0;
  std::vector<size_t> dW_off(L), db_off(L);
  EXPECT(moonwalk_grad_layout(h, &total, dW_off.data(), db_off.data()) == MW_OK);
  EXPECT(db_off[L - 1] + (size_t)widths[L] == total);
  std::vector<float> x((size_t)batch * widths[0]), t((size_t)batch * widths[L]), grads(total), scalars(2);
  const bool mw_planned = plan == 0 || (plan & MW_PLAN_MOONWALK), bp_planned = plan == 0 || (plan & MW_PLAN_BACKPROP);
  EXPECT(moonwalk_grad(h, x.data(), t.data(), grads.data(), &scalars[0], nullptr) == (mw_planned ? MW_OK : MW_ERR_NOT_PLANNED));
  EXPECT(backprop_grad(h, x.data(), t.data(), grads.data(), nullptr, nullptr) == (bp_planned ? MW_OK : MW_ERR_NOT_PLANNED));
  if (mw_planned) {
    for (int kclass = 0; kclass < MW_KCLASS_COUNT; ++kclass) {
      uint64_t n = 0;
      EXPECT(moonwalk_profile_filter(h, kclass) == MW_OK);
      EXPECT(moonwalk_grad(h, x.data(), t.data(), grads.data(), nullptr, nullptr) == MW_OK);
      EXPECT(moonwalk_profile_launches(h, kclass, &n) == MW_OK);
    }
    EXPECT(moonwalk_profile_filter(h, -1) == MW_OK);
    if (fuse) {
      EXPECT(moonwalk_sgd_step(h, x.data(), t.data(), 0.01f, 2, &scalars[0], &scalars[1], nullptr) == MW_OK);
      EXPECT(moonwalk_sgd_step(h, x.data(), t.data(), 0.01f, -1, nullptr, nullptr, nullptr) == MW_OK);
    } else {
      EXPECT(moonwalk_sgd_step(h, x.data(), t.data(), 0.01f, 2, nullptr, nullptr, nullptr) == MW_ERR_NOT_PLANNED);
    }
    for (int iters = 0; iters <= 3; ++iters) EXPECT(moonwalk_refresh_incremental(h, iters, &scalars[1], nullptr) == MW_OK);
    EXPECT(moonwalk_refresh(h, nullptr) == MW_OK);
  }
  mw_memstats_t st;
  EXPECT(moonwalk_memory_stats(h, &st) == MW_OK);
  EXPECT(st.bytes_live <= st.bytes_peak);
  EXPECT(st.nonfinite_loss == 0 && st.reserved == 0);
  EXPECT((st.bytes_debug != 0) == (debug_keep != 0 && mw_planned));
  // every kind of fetch on every layer: size query, exact buffer, buffer one byte short
  for (int i = 0; i < L; ++i)
    for (int what = MW_FETCH_MASK; what <= MW_FETCH_H_FORWARD; ++what) {
      size_t n = 0;
      const int q = moonwalk_debug_fetch(h, i, what, nullptr, 0, &n);
      if (q != MW_OK) continue;  // not kept for this layer or this plan
      std::vector<unsigned char> dst(n ? n : 1);
      EXPECT(moonwalk_debug_fetch(h, i, what, dst.data(), n, &n) == MW_OK);
      if (n > 0) EXPECT(moonwalk_debug_fetch(h, i, what, dst.data(), n - 1, nullptr) == MW_ERR_INVALID_ARG);
    }
  EXPECT(moonwalk_debug_fetch(h, L, MW_FETCH_MASK, nullptr, 0, nullptr) == MW_ERR_INVALID_ARG);
  EXPECT(moonwalk_debug_fetch(h, 0, 99, nullptr, 0, nullptr) == MW_ERR_INVALID_ARG);
  moonwalk_destroy(h);
  EXPECT(g_live_blocks == 0);
}

static void dense_allocation_failures() {
  // the allocator gives out after n calls, for every n until setup succeeds: everything taken so far must go back
  std::vector<float> W(64 * 64, 0.f);
  mw_layer_t layers[3] = {{64, 64, W.data(), nullptr, 0.f}, {64, 64, W.data(), nullptr, 0.1f}, {64, 64, W.data(), nullptr, 0.f}};
  for (int n = 0; n < 200; ++n) {
    mw_config_t cfg = base_config(8);
    cfg.reseed_interval = 1;
    cfg.dev_alloc = failing_alloc;
    g_fail_after = n;
    mw_handle_t* h = nullptr;
    const int rc = moonwalk_setup(&h, layers, 3, &cfg, nullptr);
    g_fail_after = -1;
    if (rc == MW_OK) {
      moonwalk_destroy(h);
      EXPECT(g_live_blocks == 0);
      EXPECT(n > 10);
      return;
    }
    EXPECT(rc == MW_ERR_OOM && h == nullptr && g_live_blocks == 0);
  }
  EXPECT(!"setup never succeeded");
}

static void conv_network(int kind, int channels, int k, int s, int p, int H, int Wd, int batch, int depth, int K, int kernels,
                         int h0, int block, int max_images) {
  std::vector<std::vector<float>> w(depth), b(depth);
  std::vector<mw_conv_layer_t> layers(depth);
  const int taps = kind == MW_CONV_FRAGMENTAL_1D ? k : k * k;
  for (int i = 0; i < depth; ++i) {
    w[i].assign((size_t)taps * channels * channels, 0.f);
    b[i].assign(channels, 0.f);
    layers[i] = mw_conv_layer_t{channels, channels, k, s, p, w[i].data(), b[i].data(), 0.3f, kind, block};
  }
  mw_conv_config_t cfg;
  memset(&cfg, 0, sizeof(cfg));
  cfg.batch = batch;
  cfg.height = H;
  cfg.width = Wd;
  cfg.reseed_interval = K;
  cfg.loss_scale = 1.f;
  cfg.kernels = kernels;
  cfg.input_cotangent = h0;
  cfg.max_images_per_launch = max_images;
  cfg.dev_alloc = test_alloc;
  cfg.dev_free = test_free;
  mw_conv_handle_t* h = nullptr;
  const int rc = moonwalk_conv_setup(&h, layers.data(), depth, &cfg, nullptr);
  EXPECT(rc == MW_OK && h != nullptr);
  if (rc != MW_OK) return;
  size_t total = 0;
  std::vector<size_t> dW_off(depth), db_off(depth);
  EXPECT(moonwalk_conv_grad_layout(h, &total, dW_off.data(), db_off.data()) == MW_OK);
  int Ho = H, Wo = Wd;
  for (int i = 0; i < depth; ++i) {
    if (kind == MW_CONV_SUBMERSIVE) Ho = (Ho + 2 * p - k) / s + 1;
    Wo = (Wo + 2 * p - k) / s + 1;
  }
  std::vector<float> x((size_t)batch * H * Wd * channels), t((size_t)batch * Ho * Wo * channels), grads(total), loss(1);
  EXPECT(moonwalk_conv_grad(h, x.data(), t.data(), grads.data(), loss.data(), nullptr) == MW_OK);
  EXPECT(backprop_conv_grad(h, x.data(), t.data(), grads.data(), nullptr, nullptr) == MW_OK);
  EXPECT(moonwalk_conv_refresh(h, nullptr) == MW_OK);
  const int step = moonwalk_conv_sgd_step(h, x.data(), t.data(), 0.01f, loss.data(), nullptr);
  EXPECT(step == MW_OK || step == MW_ERR_NOT_PLANNED);
  mw_conv_memstats_t st;
  EXPECT(moonwalk_conv_memory_stats(h, &st) == MW_OK);
  for (int i = 0; i < depth; ++i)
    for (int what : {MW_FETCH_MASK, MW_FETCH_H0, MW_FETCH_P, MW_FETCH_FRAG, MW_FETCH_CHECKPOINT}) {
      size_t n = 0;
      if (moonwalk_conv_fetch(h, i, what, nullptr, 0, &n) != MW_OK) continue;
      std::vector<unsigned char> dst(n ? n : 1);
      EXPECT(moonwalk_conv_fetch(h, i, what, dst.data(), n, &n) == MW_OK);
    }
  moonwalk_conv_destroy(h);
  EXPECT(g_live_blocks == 0);
}

int main() {
  validation();
  // leaky, every tile choice of a taper, a re-seed every two layers, no bias on odd layers
  dense_network({96, 96, 80, 64, 64, 33, 7}, 5, {0.1f, 0.1f, 0.5f, 1.f, 0.1f, 0.1f}, 2, 0, 1, 0, 0);
  // ReLU layers (fragment tables), mixed with leaky ones; adaptive re-seeds
  dense_network({128, 128, 128, 96, 96}, 33, {0.f, 0.1f, 0.f, 0.f}, -1, 0, 1, 0, 0);
  // segments of two and three layers over seven layers (shared mask and offset slots, a short last segment)
  dense_network({64, 64, 64, 64, 48, 48, 32, 32}, 16, {0.f, 0.1f, 0.f, 0.1f, 0.f, 0.1f, 0.f}, 0, 2, 1, 0, 0);
  dense_network({64, 64, 64, 64, 48, 48, 32, 32}, 16, {0.1f, 0.1f, 0.1f, 0.1f, 0.1f, 0.1f, 0.f}, 2, 3, 1, 1, MW_PLAN_MOONWALK);
  // the unfused path, kept tensors, one plan at a time
  dense_network({70, 50, 33, 33, 7}, 5, {0.f, 0.1f, 0.f, 0.3f}, 2, 0, 0, 1, 0);
  dense_network({40, 24}, 3, {0.1f}, 0, 0, 1, 1, MW_PLAN_MOONWALK);
  dense_network({40, 24}, 3, {0.1f}, 0, 0, 1, 0, MW_PLAN_BACKPROP);
  // shapes of the large configurations (host arithmetic in size_t / int64): 1024-wide, batch 256, 9 layers of one shape
  dense_network(std::vector<int>(10, 1024), 256, std::vector<float>(9, 0.1f), 4, 0, 1, 0, MW_PLAN_MOONWALK);
  // Phase III side by side: stretches of 4, 4, 4 and 2 layers (the short one alone), two or three or all at a
  // time, on one stream and with the side stream; a ReLU layer at the same place of every stretch; kept tensors
  for (int group : {0, 2, 3, 16})
    for (int overlap = 0; overlap <= 1; ++overlap)
      dense_network(std::vector<int>(15, 256), 64, std::vector<float>(14, 0.1f), 4, 0, 1, 0, MW_PLAN_MOONWALK, group, overlap);
  dense_network(std::vector<int>(13, 256), 77, {0.1f, 0.f, 0.1f, 0.3f, 0.1f, 0.f, 0.1f, 0.3f, 0.1f, 0.f, 0.1f, 0.3f}, 4, 0, 1, 1, 0, 3, 1);
  // the refresh with the correction product in bf16: square and narrowing runs of layers, a ragged layer that stays in fp32
  dense_network({200, 136, 136, 136, 96, 96, 70, 50}, 9, {0.1f, 0.1f, 0.1f, 0.1f, 0.1f, 0.1f, 0.1f}, 2, 0, 1, 0, MW_PLAN_MOONWALK, 1, 0, 1);
  dense_network(std::vector<int>(12, 1024), 64, std::vector<float>(11, 0.1f), 4, 0, 1, 0, MW_PLAN_MOONWALK, 0, 0, 1);
  dense_allocation_failures();
  // convolutional chains: gathered kernels and patch buffer, as-read input cotangent, image chunks of 3,
  // a kernel wider than padding + stride (the sweep), 1-D fragmental layers in blocks of 4
  conv_network(MW_CONV_SUBMERSIVE, 32, 3, 2, 1, 32, 32, 8, 3, 2, MW_CONV_KERNELS_AUTO, MW_CONV_H0_FULL, 0, 0);
  conv_network(MW_CONV_SUBMERSIVE, 32, 3, 2, 1, 32, 32, 8, 3, 1, MW_CONV_KERNELS_AUTO, MW_CONV_H0_AS_READ, 0, 3);
  conv_network(MW_CONV_SUBMERSIVE, 8, 3, 2, 1, 16, 24, 5, 2, 0, MW_CONV_KERNELS_AUTO, MW_CONV_H0_FULL, 0, 0);
  conv_network(MW_CONV_SUBMERSIVE, 32, 3, 2, 1, 16, 16, 4, 2, 0, MW_CONV_KERNELS_PATCH_MATRIX, MW_CONV_H0_FULL, 0, 0);
  conv_network(MW_CONV_SUBMERSIVE, 32, 5, 2, 1, 33, 29, 6, 2, 1, MW_CONV_KERNELS_AUTO, MW_CONV_H0_FULL, 0, 4);
  conv_network(MW_CONV_FRAGMENTAL_1D, 32, 3, 1, 1, 1, 64, 6, 3, 2, MW_CONV_KERNELS_AUTO, MW_CONV_H0_FULL, 4, 0);
  conv_network(MW_CONV_FRAGMENTAL_1D, 64, 5, 1, 2, 1, 48, 3, 2, 0, MW_CONV_KERNELS_AUTO, MW_CONV_H0_FULL, 8, 2);
  EXPECT(fake_hip_bad_launches() == 0);
  EXPECT(fake_hip_pending_configurations() == 0);
  EXPECT(fake_hip_launches() > 500);
  if (g_failures) {
    fprintf(stderr, "abi_driver: %d expectation(s) failed\n", g_failures);
    return 1;
  }
  printf("abi_driver: ok, %llu launches checked\n", fake_hip_launches());
  return 0;
}
