// libmoonwalk: handle, buffer plan and the three gradient drivers behind the C ABI.
//
// Everything here is host code that enqueues kernels; the only synchronising calls are setup,
// refresh, memory_stats, debug_fetch and destroy.
#include "../../include/moonwalk.h"
#include "../../include/moonwalk_bench.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <functional>
#include <string>
#include <utility>
#include <vector>

#include "mw_internal.h"

namespace mw {

hipError_t gemm_plain_nt(int tile, int M, int N, int K, float alpha, const float* A, int64_t lda, const float* B,
                         int64_t ldb, float beta, float* C, int64_t ldc, const float* bias, hipStream_t stream);
hipError_t gemm_plain_nn(int tile, int M, int N, int K, float alpha, const float* A, int64_t lda, const float* B,
                         int64_t ldb, float beta, float* C, int64_t ldc, const float* bias, hipStream_t stream);
hipError_t gemm_plain_tn(int tile, int M, int N, int K, float alpha, const float* A, int64_t lda, const float* B,
                         int64_t ldb, float beta, float* C, int64_t ldc, const float* bias, hipStream_t stream);

int pick_tile(int M, int N, int K) {
  auto tiles = [](int m, int n, int tm, int tn) { return (int64_t)((m + tm - 1) / tm) * ((n + tn - 1) / tn); };
  // Measured on MI355X (256 CUs) over the layer shapes of the five configurations: take the
  // largest tile that still gives every CU about two workgroups, with eight wavefronts per
  // workgroup; below that the 64x64 tile, whose eight-wavefront form splits K over two groups
  // (it pays when K is long); outputs too small even for that split K over the four wavefronts
  // of a 32x32 tile.
  if (tiles(M, N, 128, 128) >= 512) return TILE_128W8;
  if (tiles(M, N, 64, 128) >= 512) return TILE_64X128;
  const int64_t t64 = tiles(M, N, 64, 64);
  if (t64 >= 192) return K >= 1024 ? TILE_64K2 : TILE_64;
  if (K >= 256) return TILE_32K4;
  return TILE_64;
}

// The weight-gradient tile next to a kernel of tile `partner` (TILE_AUTO: none); `phase3` says
// whether that kernel is a Phase-III layer kernel or backprop's reverse product. Both tasks of a
// launch need the same workgroup size, so the choice is made among the tiles with as many
// wavefronts as the partner's; within those it follows what was measured for the pairs. It
// depends on the shapes alone: launched together or apart, a product gets the same tile and
// therefore the same bits.
int pick_tile_dw(int M, int N, int K, int partner, bool phase3) {
  (void)K;
  const int64_t t128 = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
  // eight wavefronts: beside a layer kernel the 128x128 tile (few, long workgroups on both sides
  // share the CUs evenly), beside the single reverse product the 64x128 one
  if (tile_has_8_waves(partner)) return phase3 ? TILE_128W8 : TILE_64X128;
  return t128 >= 512 ? TILE_128 : TILE_64;
}

hipError_t gemm_plain(int op, int tile, int M, int N, int K, float alpha, const float* A, int64_t lda,
                      const float* B, int64_t ldb, float beta, float* C, int64_t ldc, const float* bias,
                      hipStream_t stream) {
  switch (op) {
    case OP_NT: return gemm_plain_nt(tile, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, bias, stream);
    case OP_NN: return gemm_plain_nn(tile, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, bias, stream);
    case OP_TN: return gemm_plain_tn(tile, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, bias, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mw

using namespace mw;

namespace {

thread_local std::string g_hip_error_text = "no HIP error recorded";

int hip_fail(hipError_t e, const char* where) {
  g_hip_error_text = std::string(where) + ": " + hipGetErrorString(e);
  return MW_ERR_HIP;
}

}  // namespace

namespace mw {
int record_hip_failure(hipError_t e, const char* where) { return hip_fail(e, where); }
}  // namespace mw

namespace {

#define MW_HIP(expr)                                   \
  do {                                                 \
    hipError_t e__ = (expr);                           \
    if (e__ != hipSuccess) return hip_fail(e__, #expr); \
  } while (0)

// Launch `expr` (a launcher returning hipError_t) unless a class filter excludes it.
#define MW_LAUNCH(h, s, kclass, expr)                                   \
  do {                                                                  \
    if ((h)->class_filter < 0 || (h)->class_filter == (kclass)) {       \
      MW_HIP(expr);                                                     \
      (h)->launches[(kclass)] += 1;                                     \
    }                                                                   \
  } while (0)

void* default_alloc(size_t bytes, void*) {
  void* p = nullptr;
  if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
  return p;
}
void default_free(void* p, void*) { (void)hipFree(p); }

struct Layer {
  int d_in = 0, d_out = 0;
  const float* W = nullptr;
  const float* b = nullptr;
  float alpha = 0.f;
  float* P = nullptr;
  uint64_t* mask = nullptr;
  size_t mask_words = 0;
  uint32_t* offsets = nullptr;  // ReLU layers: [mask_words + 1]
  int relu_slot = -1;           // position in reverse-pass order among the ReLU layers
  float* ckpt = nullptr;        // kept cotangent at this layer's OUTPUT (h_i), if any
  float* xck = nullptr;         // kept activation at this layer's OUTPUT (x_i): segment boundaries only
  float* act = nullptr;         // backprop: stored x_i
  // cfg.debug_keep only: this layer's Phase-I pre-activations z_i, the Phase-II cotangent at its output
  // (NULL where ckpt already holds it), and the Phase-III cotangent at its output
  float *dbg_z = nullptr, *dbg_h = nullptr, *dbg_h3 = nullptr;
  size_t dW_off = 0, db_off = 0;
};

}  // namespace

struct mw_handle {
  std::vector<Layer> layers;
  int B = 0, L = 0, K = 0, fuse = 1, plan = 0;
  int S = 0;                        // segment length (0: the whole network is one run)
  int debug_keep = 0;               // per-layer z, Phase-II and Phase-III cotangents kept for moonwalk_debug_fetch
  int refresh_bf16 = 0;             // incremental refresh: the correction product of a Schulz iteration in bf16 matrix instructions
  float* hseg[2] = {nullptr, nullptr};  // cotangents at segment boundaries, alternating
  float loss_scale = 1.f;
  double frag_factor = 1.0;
  void* (*dev_alloc)(size_t, void*) = nullptr;
  void (*dev_free)(void*, void*) = nullptr;
  void* alloc_ctx = nullptr;
  std::vector<std::pair<void*, size_t>> allocs;
  uint64_t live = 0, peak = 0, setup_peak = 0;
  mw_memstats_t st{};
  size_t total_floats = 0;
  int dmax = 0;  // max over d_1..d_L

  // Moonwalk workspace
  float *xa = nullptr, *xb = nullptr, *ha = nullptr, *hb = nullptr, *ctz = nullptr, *zbuf = nullptr, *h0 = nullptr;
  float* frag = nullptr;
  uint64_t frag_capacity = 0;
  int n_relu = 0;
  uint64_t* frag_bases = nullptr;         // [n_relu + 1]; last = total
  const uint32_t** count_ptrs = nullptr;  // device array [n_relu]
  FragLayer* frag_layers = nullptr;       // device array [n_relu]: mask, offsets and size of every ReLU layer
  int64_t frag_max_n = 0;                 // largest B * d_out among them
  uint32_t* status = nullptr;             // [0..1] sign mismatches (u64), [2] fragment overflow, [3] non-finite loss, [4] bad pivot
  double* loss_scratch = nullptr;
  float* refresh_work = nullptr;  // incremental refresh of P: allocated on first use
  const float** refresh_tab = nullptr;  // device table of pointers for the grouped products of that refresh:
                                        // P of every layer, W of every layer, then the S and the Q slots
  struct RefreshRun {             // consecutive layers of one shape
    int l0, len, sets;            // first layer, layers, layers refreshed side by side
    bool vec;                     // grouped products (16-byte aligned operands, widths in fours); else one plain layer at a time
    size_t tab_off;               // the run's S slot pointers in refresh_tab, its Q slot pointers `sets` further on
    size_t slot, q_off;           // floats per slot of refresh_work, and where Q starts inside a slot
  };
  std::vector<RefreshRun> refresh_runs;
  // Phase III runs layer i's kernel and layer i-1's weight-gradient product in one launch: the
  // latter still reads ct_z_{i-1} and x_{i-2} while the former writes ct_z_i and x_i, so the
  // activation buffers rotate over three and the ct_z buffers over two.
  float *xc = nullptr, *ctz2 = nullptr;
  // backprop workspace
  float *bp_ha = nullptr, *bp_hb = nullptr;

  // Phase III side by side (cfg.phase3_parallel_segments): the stretches between re-seed points, top first,
  // and how they are taken: `count` > 1 consecutive stretches of one signature in grouped launches, or one
  // stretch through the ordinary sweep.
  struct Stretch { int lo, hi; };
  struct StretchGroup { int first, count; };   // indices into `stretches`
  std::vector<Stretch> stretches;
  std::vector<StretchGroup> groups;
  int group_width = 0;                          // most stretches in one launch (0: grouping off)
  int overlap = 0;                              // grouped stretches run on `side` while Phase II goes on
  std::vector<float*> gx, gh, gc;               // per group slot: 3 activation, 2 cotangent, 2 ct_z buffers
  hipStream_t side = nullptr;
  std::vector<hipEvent_t> events;               // one per group, and one to join

  // measurement aid: run only the launches of one kernel class (-1 = all), count launches
  int class_filter = -1;
  uint64_t launches[MW_KCLASS_COUNT] = {0, 0, 0, 0, 0, 0};

  void* alloc(size_t bytes, uint64_t* item) {
    if (bytes == 0) bytes = 4;
    void* p = dev_alloc(bytes, alloc_ctx);
    if (!p) return nullptr;
    allocs.emplace_back(p, bytes);
    live += bytes;
    if (live > peak) peak = live;
    if (item) *item += bytes;
    return p;
  }
  void release(void* p) {
    if (!p) return;
    for (size_t i = 0; i < allocs.size(); ++i)
      if (allocs[i].first == p) {
        live -= allocs[i].second;
        dev_free(p, alloc_ctx);
        allocs.erase(allocs.begin() + i);
        return;
      }
  }
  void release_all() {
    for (auto& a : allocs) dev_free(a.first, alloc_ctx);
    allocs.clear();
    live = 0;
    for (auto e : events) (void)hipEventDestroy(e);
    events.clear();
    if (side) (void)hipStreamDestroy(side);
    side = nullptr;
  }
};

namespace {

template <class T>
bool alloc_t(mw_handle* h, T** out, size_t count, uint64_t* item) {
  *out = static_cast<T*>(h->alloc(count * sizeof(T), item));
  return *out != nullptr;
}

// Right inverses for every layer; scratch is taken and given back within the call. Consecutive layers of
// one shape are factored side by side, up to SETUP_GROUP of them and SETUP_GROUP_BYTES of scratch at a time.
constexpr int SETUP_GROUP = 16;
constexpr size_t SETUP_GROUP_BYTES = (size_t)1 << 30;

int build_right_inverses(mw_handle* h, hipStream_t stream) {
  const int L = (int)h->layers.size();
  std::vector<int> group(L, 1);  // group[i]: layers factored together starting at layer i (0: inside a group)
  size_t work_floats = 0;
  for (int i = 0; i < L;) {
    const Layer& f = h->layers[i];
    const size_t w = setup_work_floats(f.d_out, f.d_in);
    int most = (int)(SETUP_GROUP_BYTES / (w * sizeof(float)));
    if (most > SETUP_GROUP) most = SETUP_GROUP;
    if (most < 1) most = 1;
    int g = 1;
    while (i + g < L && g < most && h->layers[i + g].d_out == f.d_out && h->layers[i + g].d_in == f.d_in) ++g;
    group[i] = g;
    for (int j = 1; j < g; ++j) group[i + j] = 0;
    if ((size_t)g * w > work_floats) work_floats = (size_t)g * w;
    i += g;
  }
  uint64_t before = h->live;
  float* work = static_cast<float*>(h->alloc(work_floats * sizeof(float), nullptr));
  if (!work) return MW_ERR_OOM;
  if (h->live > h->setup_peak) h->setup_peak = h->live;
  (void)before;
  int32_t* bad = reinterpret_cast<int32_t*>(h->status + 4);
  int rc = MW_OK;
  hipError_t e = ew_fill_u32(h->status + 4, 0u, 1, stream);
  for (int i = 0; e == hipSuccess && i < L; ++i) {
    if (group[i] == 0) continue;
    const float* Ws[SETUP_GROUP];
    float* Ps[SETUP_GROUP];
    for (int j = 0; j < group[i]; ++j) {
      Ws[j] = h->layers[i + j].W;
      Ps[j] = h->layers[i + j].P;
    }
    e = setup_right_inverse_group(group[i], Ws, h->layers[i].d_out, h->layers[i].d_in, Ps, work, bad, stream);
  }
  int32_t bad_host = 0;
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  if (e == hipSuccess) e = hipMemcpy(&bad_host, bad, sizeof(int32_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) rc = hip_fail(e, "right-inverse setup");
  else if (bad_host) rc = MW_ERR_NOT_SUBMERSIVE;
  h->release(work);
  return rc;
}

// Phase III side by side. The re-seed points cut the network into stretches that Phase III can sweep
// independently of each other once the activation at a stretch's first layer is kept too (Phase I writes it
// there anyway; with a plan it is kept for every stretch). Consecutive stretches (top first, the order in which Phase II releases them) with the same
// layer shapes and slopes, all of them shapes the grouped kernel takes, are swept in one launch per layer
// position, at most `width` of them; everything else goes through the ordinary sweep, one stretch at a time.
// width 0 (automatic): as many as it takes to give every CU one 64 x 64 tile of the layer kernel.
void plan_stretches(mw_handle* h, int width) {
  const int L = h->L, B = h->B;
  h->stretches.clear();
  h->groups.clear();
  h->group_width = 0;
  if (!h->fuse || h->S > 0 || width == 1) return;
  std::vector<int> bounds;  // 0 = b_0 < b_1 < ... < L
  bounds.push_back(0);
  for (int j = 1; j < L; ++j)
    if (h->layers[j - 1].ckpt) bounds.push_back(j);
  bounds.push_back(L);
  if (bounds.size() < 3) return;  // one stretch: nothing to run side by side
  for (size_t k = bounds.size() - 1; k >= 1; --k) h->stretches.push_back({bounds[k - 1], bounds[k]});
  auto eligible = [&](const mw_handle::Stretch& st) {
    for (int i = st.lo; i < st.hi; ++i) {
      const Layer& l = h->layers[i];
      if (!phase3_group_ok(B, l.d_out, l.d_in)) return false;
      if ((reinterpret_cast<uintptr_t>(l.W) | reinterpret_cast<uintptr_t>(l.P)) & 15) return false;
    }
    return true;
  };
  auto same = [&](const mw_handle::Stretch& a, const mw_handle::Stretch& b) {
    if (a.hi - a.lo != b.hi - b.lo) return false;
    for (int j = 0; j < a.hi - a.lo; ++j) {
      const Layer &p = h->layers[a.lo + j], &q = h->layers[b.lo + j];
      if (p.d_in != q.d_in || p.d_out != q.d_out || p.alpha != q.alpha) return false;
    }
    return true;
  };
  const int n = (int)h->stretches.size();
  int widest = 0;
  for (int k = 0; k < n;) {
    int count = 1;
    if (eligible(h->stretches[k])) {
      int most = width;
      if (most == 0) {
        const Layer& l = h->layers[h->stretches[k].lo];
        const int tiles = ((B + 63) / 64) * ((l.d_out + 63) / 64);
        most = (256 + tiles - 1) / tiles;
      }
      if (most > 16) most = 16;
      while (k + count < n && count < most && same(h->stretches[k], h->stretches[k + count])) ++count;
    }
    h->groups.push_back({k, count});
    if (count > widest) widest = count;
    k += count;
  }
  if (widest < 2) {  // nothing to gain: the ordinary sweep, no kept activations
    h->stretches.clear();
    h->groups.clear();
    return;
  }
  h->group_width = widest;
}

int validate_layers(const mw_layer_t* layers, int32_t n_layers, const mw_config_t* cfg) {
  if (!layers || n_layers <= 0 || !cfg || cfg->batch <= 0) return MW_ERR_INVALID_ARG;
  if (cfg->reseed_interval < -1 || cfg->segment_length < 0) return MW_ERR_INVALID_ARG;
  if (cfg->segment_length > 0 && !cfg->fuse) return MW_ERR_INVALID_ARG;
  if (!(cfg->loss_scale > 0.f) || !std::isfinite(cfg->loss_scale)) return MW_ERR_INVALID_ARG;
  if ((cfg->dev_alloc == nullptr) != (cfg->dev_free == nullptr)) return MW_ERR_INVALID_ARG;
  if (cfg->plan & ~(MW_PLAN_MOONWALK | MW_PLAN_BACKPROP)) return MW_ERR_INVALID_ARG;
  if (cfg->debug_keep != 0 && cfg->debug_keep != 1) return MW_ERR_INVALID_ARG;
  if (cfg->phase3_parallel_segments < 0 || cfg->phase3_parallel_segments > 16) return MW_ERR_INVALID_ARG;
  if (cfg->phase3_overlap < 0 || cfg->phase3_overlap > 1) return MW_ERR_INVALID_ARG;
  if (cfg->refresh_precision < 0 || cfg->refresh_precision > 1) return MW_ERR_INVALID_ARG;
  for (int i = 0; i < n_layers; ++i) {
    const mw_layer_t& l = layers[i];
    if (l.d_in <= 0 || l.d_out <= 0 || !l.W) return MW_ERR_INVALID_ARG;
    if (!(l.alpha >= 0.f && l.alpha <= 1.f)) return MW_ERR_INVALID_ARG;
    if (i > 0 && l.d_in != layers[i - 1].d_out) return MW_ERR_INVALID_ARG;
  }
  // the kernels address every operand with 31-bit byte offsets: each matrix must stay below 2 GiB
  const int64_t limit = (int64_t)0x7FFFFFFF;
  for (int i = 0; i < n_layers; ++i) {
    const mw_layer_t& l = layers[i];
    if ((int64_t)l.d_out * l.d_in * 4 >= limit) return MW_ERR_INVALID_ARG;
    if ((int64_t)cfg->batch * l.d_in * 4 >= limit || (int64_t)cfg->batch * l.d_out * 4 >= limit) return MW_ERR_INVALID_ARG;
  }
  for (int i = 0; i < n_layers; ++i)
    if (layers[i].d_out > layers[i].d_in) return MW_ERR_NOT_SUBMERSIVE;
  return MW_OK;
}

}  // namespace

// =============================================================================================== C ABI

extern "C" {

int moonwalk_setup(mw_handle_t** out, const mw_layer_t* layers, int32_t n_layers, const mw_config_t* cfg,
                   void* hip_stream) {
  if (!out) return MW_ERR_INVALID_ARG;
  *out = nullptr;
  int rc = validate_layers(layers, n_layers, cfg);
  if (rc != MW_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  mw_handle* h = new mw_handle();
  h->B = cfg->batch;
  h->L = n_layers;
  h->K = cfg->reseed_interval;
  h->S = (cfg->segment_length > 0 && cfg->segment_length < n_layers) ? cfg->segment_length : 0;
  h->fuse = cfg->fuse ? 1 : 0;
  h->debug_keep = cfg->debug_keep;
  h->refresh_bf16 = cfg->refresh_precision;
  h->plan = cfg->plan ? cfg->plan : (MW_PLAN_MOONWALK | MW_PLAN_BACKPROP);
  h->loss_scale = cfg->loss_scale;
  h->frag_factor = cfg->frag_capacity_factor > 0.0 ? cfg->frag_capacity_factor : 1.0;
  h->dev_alloc = cfg->dev_alloc ? cfg->dev_alloc : default_alloc;
  h->dev_free = cfg->dev_free ? cfg->dev_free : default_free;
  h->alloc_ctx = cfg->alloc_ctx;
  h->layers.resize(n_layers);
  size_t off = 0;
  const size_t B = (size_t)h->B;
  for (int i = 0; i < n_layers; ++i) {
    Layer& l = h->layers[i];
    l.d_in = layers[i].d_in;
    l.d_out = layers[i].d_out;
    l.W = layers[i].W;
    l.b = layers[i].b;
    l.alpha = layers[i].alpha;
    l.dW_off = off;
    off += (size_t)l.d_out * l.d_in;
    l.db_off = off;
    off += (size_t)l.d_out;
    if (l.d_out > h->dmax) h->dmax = l.d_out;
  }
  h->total_floats = off;

  auto fail = [&](int code) {
    h->release_all();
    delete h;
    return code;
  };
  mw_memstats_t& st = h->st;
  bool ok = alloc_t(h, &h->status, 5, &st.bytes_mw_scratch);
  if (!ok) return fail(MW_ERR_OOM);
  hipError_t e = ew_fill_u32(h->status, 0u, 5, stream);
  if (e != hipSuccess) return fail(hip_fail(e, "status init"));

  if (h->plan & MW_PLAN_MOONWALK) {
    // right inverses
    for (auto& l : h->layers) ok = ok && alloc_t(h, &l.P, (size_t)l.d_out * l.d_in, &st.bytes_P);
    if (!ok) return fail(MW_ERR_OOM);
    rc = build_right_inverses(h, stream);
    if (rc != MW_OK) return fail(rc);

    // Sign masks (zeroed once: the padding bits of the last word are never written afterwards),
    // and for ReLU layers the per-word erased offsets. Without segments every layer has its own;
    // with segments the layers at the same position of their segments share a slot sized for the
    // largest of them.
    const int S = h->S;
    const int n_slots = S > 0 ? S : n_layers;
    std::vector<uint64_t*> mask_slot(n_slots, nullptr);
    std::vector<uint32_t*> off_slot(n_slots, nullptr);
    {
      std::vector<size_t> words(n_slots, 0);
      std::vector<bool> relu(n_slots, false);
      for (int i = 0; i < n_layers; ++i) {
        Layer& l = h->layers[i];
        l.mask_words = (B * l.d_out + 63) / 64;
        const int p = S > 0 ? i % S : i;
        if (l.mask_words > words[p]) words[p] = l.mask_words;
        if (l.alpha == 0.f) relu[p] = true;
      }
      for (int p = 0; p < n_slots; ++p) {
        ok = ok && alloc_t(h, &mask_slot[p], words[p], &st.bytes_masks);
        if (ok) {
          e = ew_fill_u32(reinterpret_cast<uint32_t*>(mask_slot[p]), 0u, (int64_t)words[p] * 2, stream);
          if (e != hipSuccess) return fail(hip_fail(e, "mask init"));
        }
        if (relu[p]) ok = ok && alloc_t(h, &off_slot[p], words[p] + 1, &st.bytes_frag_index);
      }
      if (!ok) return fail(MW_ERR_OOM);
    }
    // fragment store (ReLU layers): room for the erased cotangents of one run of layers
    size_t relu_elems = 0, run_elems = 0;
    for (int i = 0; i < n_layers; ++i) {
      Layer& l = h->layers[i];
      const int p = S > 0 ? i % S : i;
      l.mask = mask_slot[p];
      if (S > 0 && p == 0) run_elems = 0;
      if (l.alpha == 0.f) {
        ++h->n_relu;
        l.offsets = off_slot[p];
        run_elems += B * l.d_out;
        if (run_elems > relu_elems) relu_elems = run_elems;
      }
    }
    if (ok && h->n_relu > 0) {
      h->frag_capacity = (uint64_t)std::ceil(h->frag_factor * (double)relu_elems);
      if (h->frag_capacity < 1) h->frag_capacity = 1;
      ok = ok && alloc_t(h, &h->frag, h->frag_capacity, &st.bytes_fragments);
      ok = ok && alloc_t(h, &h->frag_bases, (size_t)h->n_relu + 1, &st.bytes_frag_index);
      ok = ok && alloc_t(h, &h->count_ptrs, (size_t)h->n_relu, &st.bytes_frag_index);
      ok = ok && alloc_t(h, &h->frag_layers, (size_t)h->n_relu, &st.bytes_frag_index);
      if (ok) {
        std::vector<const uint32_t*> ptrs;
        std::vector<FragLayer> table;
        int slot = 0;
        for (int i = n_layers - 1; i >= 0; --i) {  // reverse-pass order: layer L first
          Layer& l = h->layers[i];
          if (l.alpha == 0.f) {
            l.relu_slot = slot++;
            ptrs.push_back(l.offsets + l.mask_words);
            const int64_t n = (int64_t)(B * l.d_out);
            uint32_t* sums = nullptr;
            ok = ok && alloc_t(h, &sums, ew_frag_scan_words(n), &st.bytes_frag_index);
            table.push_back(FragLayer{l.mask, l.offsets, n, sums});
            if (n > h->frag_max_n) h->frag_max_n = n;
          }
        }
        if (!ok) return fail(MW_ERR_OOM);
        e = hipMemcpy(h->count_ptrs, ptrs.data(), ptrs.size() * sizeof(ptrs[0]), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(h->frag_layers, table.data(), table.size() * sizeof(table[0]), hipMemcpyHostToDevice);
        if (e != hipSuccess) return fail(hip_fail(e, "fragment index init"));
      }
    }
    // Re-seed checkpoints: the cotangent at the output of layer j (1-based), kept in the reverse
    // pass and taken up again by Phase III. K > 0: j = K, 2K, ... < L. K = -1: placed where the
    // predicted growth of the rounding error since the last seed, prod (alpha + 1/alpha)/2 over
    // the layers in between, would pass 700 (what four alpha = 0.1 layers give; measured to keep
    // the gradients at 1e-4 of the oracle's). Segment boundaries are exact seeds by themselves.
    {
      double growth = 1.0;
      for (int j = 1; j < n_layers; ++j) {
        const float a = h->layers[j - 1].alpha;
        growth *= (a > 0.f) ? 0.5 * ((double)a + 1.0 / (double)a) : 1.0;
        const bool boundary = S > 0 && j % S == 0;
        bool keep = false;
        if (boundary) {
          growth = 1.0;
        } else if (h->K > 0) {
          keep = (j % h->K == 0);
        } else if (h->K < 0) {
          const float an = h->layers[j].alpha;
          const double next = growth * ((an > 0.f) ? 0.5 * ((double)an + 1.0 / (double)an) : 1.0);
          if (next > 700.0) {
            keep = true;
            growth = 1.0;
          }
        }
        if (keep) ok = ok && alloc_t(h, &h->layers[j - 1].ckpt, B * h->layers[j - 1].d_out, &st.bytes_checkpoints);
        if (boundary) ok = ok && alloc_t(h, &h->layers[j - 1].xck, B * h->layers[j - 1].d_out, &st.bytes_checkpoints);
      }
    }
    // Phase III side by side: the plan, the activations kept at the first layer of every stretch that is
    // swept in a group, the groups' own rotating buffers, and the side stream with its events
    plan_stretches(h, cfg->phase3_parallel_segments);
    if (h->group_width > 0) {
      const size_t nmax = B * (size_t)h->dmax;
      for (const auto& sg : h->stretches)
        if (sg.lo > 0) ok = ok && alloc_t(h, &h->layers[sg.lo - 1].xck, B * h->layers[sg.lo - 1].d_out, &st.bytes_checkpoints);
      h->gx.assign((size_t)3 * h->group_width, nullptr);
      h->gh.assign((size_t)2 * h->group_width, nullptr);
      h->gc.assign((size_t)2 * h->group_width, nullptr);
      for (auto& p : h->gx) ok = ok && alloc_t(h, &p, nmax, &st.bytes_mw_scratch);
      for (auto& p : h->gh) ok = ok && alloc_t(h, &p, nmax, &st.bytes_mw_scratch);
      for (auto& p : h->gc) ok = ok && alloc_t(h, &p, nmax, &st.bytes_mw_scratch);
      if (!ok) return fail(MW_ERR_OOM);
      h->overlap = cfg->phase3_overlap;
      if (h->overlap) {
        e = hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking);  // default priority
        if (e != hipSuccess) return fail(hip_fail(e, "side stream"));
        h->events.resize(h->groups.size() + 2, nullptr);
        for (auto& ev : h->events) {
          e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
          if (e != hipSuccess) return fail(hip_fail(e, "event"));
        }
      }
    }
    // ping-pong buffers
    const size_t nmax = B * (size_t)h->dmax;
    ok = ok && alloc_t(h, &h->xa, nmax, &st.bytes_mw_scratch) && alloc_t(h, &h->xb, nmax, &st.bytes_mw_scratch) &&
         alloc_t(h, &h->ha, nmax, &st.bytes_mw_scratch) && alloc_t(h, &h->hb, nmax, &st.bytes_mw_scratch) &&
         alloc_t(h, &h->ctz, nmax, &st.bytes_mw_scratch) &&
         alloc_t(h, &h->h0, B * (size_t)h->layers[0].d_in, &st.bytes_mw_scratch);
    if (!h->fuse) ok = ok && alloc_t(h, &h->zbuf, nmax, &st.bytes_mw_scratch);
    if (h->debug_keep)
      for (auto& l : h->layers) {
        const size_t n = B * (size_t)l.d_out;
        ok = ok && alloc_t(h, &l.dbg_z, n, &st.bytes_debug) && alloc_t(h, &l.dbg_h3, n, &st.bytes_debug);
        if (!l.ckpt) ok = ok && alloc_t(h, &l.dbg_h, n, &st.bytes_debug);
      }
    if (h->fuse) ok = ok && alloc_t(h, &h->xc, nmax, &st.bytes_mw_scratch) && alloc_t(h, &h->ctz2, nmax, &st.bytes_mw_scratch);
    if (h->S > 0) ok = ok && alloc_t(h, &h->hseg[0], nmax, &st.bytes_mw_scratch) && alloc_t(h, &h->hseg[1], nmax, &st.bytes_mw_scratch);
    if (!ok) return fail(MW_ERR_OOM);
  }
  ok = ok && alloc_t(h, &h->loss_scratch, (size_t)LOSS_BLOCKS, &st.bytes_mw_scratch);
  if (h->plan & MW_PLAN_BACKPROP) {
    for (auto& l : h->layers) ok = ok && alloc_t(h, &l.act, B * l.d_out, &st.bytes_bp_activations);
    const size_t nmax = B * (size_t)h->dmax;
    ok = ok && alloc_t(h, &h->bp_ha, nmax, &st.bytes_bp_scratch) && alloc_t(h, &h->bp_hb, nmax, &st.bytes_bp_scratch);
  }
  if (!ok) return fail(MW_ERR_OOM);
  e = hipStreamSynchronize(stream);
  if (e != hipSuccess) return fail(hip_fail(e, "setup sync"));
  *out = h;
  return MW_OK;
}

int moonwalk_refresh(mw_handle_t* h, void* hip_stream) {
  if (!h) return MW_ERR_INVALID_ARG;
  if (!(h->plan & MW_PLAN_MOONWALK)) return MW_ERR_NOT_PLANNED;
  return build_right_inverses(h, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"

namespace {

// One gradient step is assembled from four pieces that work on a run of layers [lo, hi).
// Without segments the run is the whole network; with segments (cfg.segment_length = S) Phase I
// keeps x at every S-th layer boundary and no masks, and the segments are then finished one by
// one from the top: forward again inside the segment (masks, fragment index), reverse through
// it, Phase III through it. Only one segment's masks and fragments exist at a time.
#define MW_TRY_RC(expr)          \
  do {                           \
    int rc__ = (expr);           \
    if (rc__ != MW_OK) return rc__; \
  } while (0)

struct Step {
  mw_handle* h;
  hipStream_t s;
  const float* x;
  float* grads_out;
  float apply_lr;  // 0: gradients to grads_out; else W_i -= apply_lr dW_i, b_i -= apply_lr db_i in place
};

// Forward through layers [lo, hi) from xin. Layers i >= mask_from also write their sign masks.
// A layer with an activation checkpoint writes its output there. *x_end = x_{hi}.
int forward_range(const Step& c, int lo, int hi, const float* xin, int mask_from, const float** x_end) {
  mw_handle* h = c.h;
  hipStream_t s = c.s;
  const int B = h->B;
  float* xbuf[2] = {h->xa, h->xb};
  for (int i = lo; i < hi; ++i) {
    Layer& l = h->layers[i];
    float* xout = l.xck ? l.xck : xbuf[i & 1];
    const bool want_mask = i >= mask_from;
    // mask slots are shared between segments: clear what this layer's packing will not overwrite
    if (want_mask && h->S > 0 && (((size_t)B * l.d_out) % 64) != 0)
      MW_LAUNCH(h, s, MW_KCLASS_EW, ew_fill_u32(reinterpret_cast<uint32_t*>(l.mask + l.mask_words - 1), 0u, 2, s));
    if (h->fuse) {
      if (want_mask && l.d_out % 32 == 0) {
        MW_LAUNCH(h, s, MW_KCLASS_FWD, gemm_fwd_act(TILE_AUTO, B, l.d_out, l.d_in, xin, l.W, l.b, l.alpha, xout, l.mask, s, l.dbg_z));
      } else {
        MW_LAUNCH(h, s, MW_KCLASS_FWD, gemm_fwd_act(TILE_AUTO, B, l.d_out, l.d_in, xin, l.W, l.b, l.alpha, xout, nullptr, s, l.dbg_z));
        if (want_mask) MW_LAUNCH(h, s, MW_KCLASS_EW, ew_mask_from_act(xout, (int64_t)B * l.d_out, l.mask, s));
      }
    } else {
      float* z = l.dbg_z ? l.dbg_z : h->zbuf;
      MW_LAUNCH(h, s, MW_KCLASS_FWD, gemm_plain(OP_NT, TILE_AUTO, B, l.d_out, l.d_in, 1.f, xin, l.d_in, l.W, l.d_in, 0.f, z, l.d_out,
                        l.b, s));
      MW_LAUNCH(h, s, MW_KCLASS_EW, ew_bias_act_mask(z, nullptr, B, l.d_out, l.alpha, xout, want_mask ? l.mask : nullptr, s));
    }
    xin = xout;
  }
  *x_end = xin;
  return MW_OK;
}

// Fragment index (erased-element offsets, then the bases of the store) of the ReLU layers in
// [lo, hi): one scan launch and one tiny scan. The per-layer tables are in reverse-pass order,
// so the layers of a run are a contiguous stretch of them; bases restart at 0 for every run.
int frag_index_range(const Step& c, int lo, int hi) {
  mw_handle* h = c.h;
  int first = -1, count = 0;
  for (int i = hi - 1; i >= lo; --i)
    if (h->layers[i].alpha == 0.f) {
      if (first < 0) first = h->layers[i].relu_slot;
      ++count;
    }
  if (count == 0) return MW_OK;
  MW_LAUNCH(h, c.s, MW_KCLASS_EW, ew_frag_offsets_layers(h->frag_layers + first, count, h->frag_max_n, c.s));
  MW_LAUNCH(h, c.s, MW_KCLASS_EW, ew_frag_bases(h->count_ptrs + first, count, h->frag_bases + first, h->frag_bases + h->n_relu, c.s));
  return MW_OK;
}

// Phase II through layers [lo, hi): h_top holds the raw cotangent at the output of layer hi-1
// (overwritten), the cotangent at the input of layer lo goes to h_bottom.
// `released` (may be empty) is called after the launch that produced the cotangent at layer boundary i
// (the input of layer i), for every i in [lo, hi), top down.
int reverse_range(const Step& c, int lo, int hi, float* h_top, float* h_bottom,
                  const std::function<int(int)>& released = nullptr) {
  mw_handle* h = c.h;
  hipStream_t s = c.s;
  const int B = h->B;
  int32_t* overflow = reinterpret_cast<int32_t*>(h->status + 2);
  float* hbuf[2] = {h->ha, h->hb};
  {
    Layer& top = h->layers[hi - 1];  // debugging aid: the raw cotangent at the top of the run
    if (top.dbg_h) MW_LAUNCH(h, s, MW_KCLASS_EW, ew_copy(h_top, top.dbg_h, (int64_t)B * top.d_out, s));
  }
  if (h->fuse) {
    // The top layer's slope (and fragments) are applied by the elementwise kernels; every
    // reverse product then applies the slope of the layer below it in its own epilogue.
    {
      Layer& l = h->layers[hi - 1];
      const int64_t n = (int64_t)B * l.d_out;
      if (l.alpha == 0.f)
        MW_LAUNCH(h, s, MW_KCLASS_EW, ew_frag_compact(h_top, l.mask, l.offsets, n, h->frag, h->frag_bases + l.relu_slot,
                                                      h->frag_capacity, overflow, s));
      MW_LAUNCH(h, s, MW_KCLASS_EW, ew_rev_scale(h_top, l.mask, n, l.alpha, h_top, s));
    }
    const float* ctcur = h_top;
    for (int i = hi - 1; i >= lo; --i) {
      Layer& l = h->layers[i];
      if (i == lo) {
        MW_LAUNCH(h, s, MW_KCLASS_REV, gemm_plain(OP_NN, TILE_AUTO, B, l.d_in, l.d_out, 1.f, ctcur, l.d_out, l.W, l.d_in, 0.f,
                                                  h_bottom, l.d_in, nullptr, s));
      } else {
        Layer& below = h->layers[i - 1];
        float* ctout = (ctcur == hbuf[0]) ? hbuf[1] : hbuf[0];
        const bool relu = below.alpha == 0.f;
        RevArgs r{ctout, below.ckpt ? below.ckpt : below.dbg_h, below.mask, below.alpha, below.offsets, h->frag,
                  relu ? h->frag_bases + below.relu_slot : nullptr, h->frag_capacity, overflow};
        MW_LAUNCH(h, s, MW_KCLASS_REV, gemm_rev_fused(TILE_AUTO, B, l.d_in, l.d_out, ctcur, l.W, r, s));
        ctcur = ctout;
      }
      if (released) MW_TRY_RC(released(i));
    }
  } else {
    const float* hcur = h_top;
    for (int i = hi - 1; i >= lo; --i) {
      Layer& l = h->layers[i];
      const int64_t n = (int64_t)B * l.d_out;
      if (l.alpha == 0.f)
        MW_LAUNCH(h, s, MW_KCLASS_EW, ew_frag_compact(hcur, l.mask, l.offsets, n, h->frag, h->frag_bases + l.relu_slot,
                                                      h->frag_capacity, overflow, s));
      float* hout;
      if (i == lo) hout = h_bottom;
      else if (h->layers[i - 1].ckpt) hout = h->layers[i - 1].ckpt;
      else if (h->layers[i - 1].dbg_h) hout = h->layers[i - 1].dbg_h;
      else hout = (hcur == hbuf[0]) ? hbuf[1] : hbuf[0];
      MW_LAUNCH(h, s, MW_KCLASS_EW, ew_rev_scale(hcur, l.mask, n, l.alpha, h->ctz, s));
      MW_LAUNCH(h, s, MW_KCLASS_REV, gemm_plain(OP_NN, TILE_AUTO, B, l.d_in, l.d_out, 1.f, h->ctz, l.d_out, l.W, l.d_in, 0.f,
                                                hout, l.d_in, nullptr, s));
      hcur = hout;
      if (released) MW_TRY_RC(released(i));
    }
  }
  return MW_OK;
}

// Phase III through layers [lo, hi) from the input xin and the input cotangent hin of layer lo.
// apply_lr != 0 (fused path only): each layer's gradient is applied to the caller's W_i, b_i as
// soon as it exists (Algorithm 1, "Apply g_i"). W_i is last read by layer i's own kernel, one
// launch before the launch that carries its weight gradient, so updating it in place is safe.
int phase3_range(const Step& c, int lo, int hi, const float* xin, const float* hin) {
  mw_handle* h = c.h;
  hipStream_t s = c.s;
  const int B = h->B;
  unsigned long long* mismatches = reinterpret_cast<unsigned long long*>(h->status);
  float* hbuf[2] = {h->ha, h->hb};
  float* xbuf[2] = {h->xa, h->xb};
  const float inv_scale = 1.0f / h->loss_scale;
  if (h->fuse) {
    // Launch k carries layer k's kernel and layer k-1's weight gradient (see the buffer rotation
    // at the handle); a last launch carries the final weight gradient alone. With a class filter
    // set the two are launched separately so that each can be timed alone.
    const bool paired = h->class_filter < 0 || h->class_filter == MW_KCLASS_PHASE3;
    float* xrot[3] = {h->xa, h->xb, h->xc};
    float* crot[2] = {h->ctz, h->ctz2};
    DwArgs pending{};
    bool have_pending = false;
    for (int i = lo; i < hi; ++i) {
      Layer& l = h->layers[i];
      if (i > lo && h->layers[i - 1].ckpt) hin = h->layers[i - 1].ckpt;  // re-seed
      float* xout = xrot[i % 3];
      float* ctz = crot[i & 1];
      float* hout = l.dbg_h3 ? l.dbg_h3 : hbuf[i & 1];
      const bool relu = (l.alpha == 0.f);
      VijpArgs a{xin, l.W, l.b, hin, l.P, l.alpha, l.mask, l.offsets, h->frag,
                 relu ? h->frag_bases + l.relu_slot : nullptr, h->frag_capacity, xout, hout, ctz, mismatches};
      DwArgs d{l.d_out, l.d_in, B, ctz, xin, inv_scale, nullptr, nullptr};
      if (c.apply_lr != 0.f) {
        d.scale = -c.apply_lr * inv_scale;
        d.dW = const_cast<float*>(l.W);
        d.db = const_cast<float*>(l.b);  // NULL: the layer has no bias
        d.beta = 1.f;
      } else {
        d.dW = c.grads_out + l.dW_off;
        d.db = c.grads_out + l.db_off;
      }
      if (paired) {
        MW_LAUNCH(h, s, MW_KCLASS_PHASE3, gemm_phase3_pair(&a, B, l.d_out, l.d_in, have_pending ? &pending : nullptr, s));
        pending = d;
        have_pending = true;
      } else {
        // same tiles as in the paired launches: the weight gradient's follows the next layer's kernel
        const int partner = (i + 1 < hi) ? pick_tile(B, h->layers[i + 1].d_out, h->layers[i + 1].d_in) : TILE_AUTO;
        MW_LAUNCH(h, s, MW_KCLASS_VIJP, gemm_vijp_dual(TILE_AUTO, B, l.d_out, l.d_in, a, s));
        MW_LAUNCH(h, s, MW_KCLASS_DW, gemm_dw(pick_tile_dw(d.M, d.N, d.K, partner, true), d.M, d.N, d.K, d.CTZ, d.X, d.scale,
                                              d.dW, d.db, s, d.beta));
      }
      xin = xout;
      hin = hout;
    }
    if (have_pending) MW_LAUNCH(h, s, MW_KCLASS_PHASE3, gemm_phase3_pair(nullptr, 0, 0, 0, &pending, s));
  } else {
    for (int i = lo; i < hi; ++i) {
      Layer& l = h->layers[i];
      if (i > lo && h->layers[i - 1].ckpt) hin = h->layers[i - 1].ckpt;  // re-seed
      float* xout = xbuf[i & 1];
      float* hout = l.dbg_h3 ? l.dbg_h3 : hbuf[i & 1];
      const bool relu = (l.alpha == 0.f);
      MW_LAUNCH(h, s, MW_KCLASS_FWD, gemm_plain(OP_NT, TILE_AUTO, B, l.d_out, l.d_in, 1.f, xin, l.d_in, l.W, l.d_in, 0.f, h->zbuf, l.d_out,
                        l.b, s));
      MW_LAUNCH(h, s, MW_KCLASS_FWD, gemm_plain(OP_NT, TILE_AUTO, B, l.d_out, l.d_in, 1.f, hin, l.d_in, l.P, l.d_in, 0.f, h->ctz, l.d_out,
                        nullptr, s));
      MW_LAUNCH(h, s, MW_KCLASS_EW, ew_vijp_epilogue(h->zbuf, h->ctz, B, l.d_out, l.alpha, l.mask, l.offsets, h->frag,
                              relu ? h->frag_bases + l.relu_slot : nullptr, h->frag_capacity, xout, hout, mismatches,
                              s));
      const int partner = (i + 1 < hi) ? pick_tile(B, h->layers[i + 1].d_out, h->layers[i + 1].d_in) : TILE_AUTO;
      MW_LAUNCH(h, s, MW_KCLASS_DW, gemm_dw(pick_tile_dw(l.d_out, l.d_in, B, partner, true), l.d_out, l.d_in, B, h->ctz, xin, inv_scale,
                                            c.grads_out + l.dW_off, nullptr, s));
      MW_LAUNCH(h, s, MW_KCLASS_EW, ew_colsum(h->ctz, B, l.d_out, inv_scale, c.grads_out + l.db_off, s));
      xin = xout;
      hin = hout;
    }
  }
  return MW_OK;
}

// Phase III of the stretches [first, first + count) of the plan, side by side on stream `s`: position j of all of
// them in one launch, which also carries the weight gradients of position j - 1 (the rotation of phase3_range,
// per stretch, over the group's own buffers). A stretch starts from the activation and the cotangent kept at
// its first layer. The weight gradients of a group's last position would need a launch of their own: they are
// handed on in `carry` instead and ride in the next group's first launch (the caller flushes what is left),
// unless they read a buffer that launch writes (the groups share their rotating buffers).
struct CarriedDw {
  DwArgs d[MAX_PHASE3_GROUP];
  int n = 0;
};

int flush_carried(const Step& c, CarriedDw* carry, hipStream_t s) {
  if (carry->n > 0) MW_LAUNCH(c.h, s, MW_KCLASS_PHASE3, gemm_phase3_group(0, nullptr, 0, 0, 0, carry->n, carry->d, s));
  carry->n = 0;
  return MW_OK;
}

int phase3_group(const Step& c, int first, int count, hipStream_t s, CarriedDw* carry) {
  mw_handle* h = c.h;
  const int B = h->B;
  unsigned long long* mismatches = reinterpret_cast<unsigned long long*>(h->status);
  const float inv_scale = 1.0f / h->loss_scale;
  const bool paired = h->class_filter < 0 || h->class_filter == MW_KCLASS_PHASE3;
  const int len = h->stretches[first].hi - h->stretches[first].lo;
  VijpArgs v[MAX_PHASE3_GROUP];
  DwArgs pending[MAX_PHASE3_GROUP], fresh[MAX_PHASE3_GROUP];
  int n_pending = 0;
  if (paired) {
    for (int g = 0; g < carry->n; ++g) pending[g] = carry->d[g];
    n_pending = carry->n;
    carry->n = 0;
  }
  for (int j = 0; j < len; ++j) {
    for (int g = 0; g < count; ++g) {
      const int lo = h->stretches[first + g].lo, i = lo + j;
      Layer& l = h->layers[i];
      float* const* xrot = &h->gx[(size_t)3 * g];
      float* const* hrot = &h->gh[(size_t)2 * g];
      float* const* crot = &h->gc[(size_t)2 * g];
      const float* xin = j > 0 ? xrot[(j - 1) % 3] : (lo == 0 ? c.x : h->layers[lo - 1].xck);
      const float* hin = j > 0 ? (h->layers[i - 1].dbg_h3 ? h->layers[i - 1].dbg_h3 : hrot[(j - 1) & 1])
                               : (lo == 0 ? h->h0 : h->layers[lo - 1].ckpt);
      float* hout = l.dbg_h3 ? l.dbg_h3 : hrot[j & 1];
      const bool relu = (l.alpha == 0.f);
      v[g] = VijpArgs{xin, l.W, l.b, hin, l.P, l.alpha, l.mask, l.offsets, h->frag,
                      relu ? h->frag_bases + l.relu_slot : nullptr, h->frag_capacity, xrot[j % 3], hout, crot[j & 1], mismatches};
      DwArgs d{l.d_out, l.d_in, B, crot[j & 1], xin, inv_scale, nullptr, nullptr};
      if (c.apply_lr != 0.f) {
        d.scale = -c.apply_lr * inv_scale;
        d.dW = const_cast<float*>(l.W);
        d.db = const_cast<float*>(l.b);
        d.beta = 1.f;
      } else {
        d.dW = c.grads_out + l.dW_off;
        d.db = c.grads_out + l.db_off;
      }
      fresh[g] = d;
    }
    const Layer& l0 = h->layers[h->stretches[first].lo + j];
    if (paired) {
      MW_LAUNCH(h, s, MW_KCLASS_PHASE3, gemm_phase3_group(count, v, B, l0.d_out, l0.d_in, n_pending, pending, s));
    } else {
      MW_LAUNCH(h, s, MW_KCLASS_VIJP, gemm_phase3_group(count, v, B, l0.d_out, l0.d_in, 0, nullptr, s));
      MW_LAUNCH(h, s, MW_KCLASS_DW, gemm_phase3_group(0, nullptr, 0, 0, 0, count, fresh, s));
    }
    for (int g = 0; g < count; ++g) pending[g] = fresh[g];
    n_pending = count;
  }
  if (!paired) return MW_OK;
  // The last position's weight gradients read ct_z buffer (len - 1) & 1 and activation buffer (len - 2) % 3 of
  // their slot (the kept activation when len == 1); the next group's first launch writes buffers 0 of each.
  const bool safe_to_carry = len >= 2 && ((len - 1) & 1) != 0 && ((len - 2) % 3) != 0;
  for (int g = 0; g < count; ++g) carry->d[g] = pending[g];
  carry->n = count;
  if (!safe_to_carry) return flush_carried(c, carry, s);
  return MW_OK;
}

// Phases II and III with the plan of plan_stretches. Phase II runs on `s`. A group of stretches can be swept as
// soon as Phase II has passed its lowest boundary: with overlap it is then issued on the side stream (behind an
// event) and shares the machine with the rest of Phase II; otherwise, and for stretches taken one at a time
// (they use the buffers Phase II uses), it is issued on `s` after Phase II, top first.
int reverse_and_sweep(const Step& c) {
  mw_handle* h = c.h;
  hipStream_t s = c.s;
  const int L = h->L;
  const bool overlap = h->overlap && h->class_filter < 0;
  size_t next = 0;  // next group Phase II will release
  int side_used = 0;
  CarriedDw carry;
  auto released = [&](int boundary) -> int {
    while (next < h->groups.size()) {
      const auto& g = h->groups[next];
      if (h->stretches[g.first + g.count - 1].lo != boundary) break;
      if (overlap && g.count > 1) {
        MW_HIP(hipEventRecord(h->events[next], s));
        MW_HIP(hipStreamWaitEvent(h->side, h->events[next], 0));
        MW_TRY_RC(phase3_group(c, g.first, g.count, h->side, &carry));
        side_used = 1;
      }
      ++next;
    }
    return MW_OK;
  };
  // (every launch on the side stream follows a wait for an event recorded on the caller's stream inside this call,
  // and the last call ended with the caller's stream waiting for the side stream: no further fence is needed here)
  MW_TRY_RC(reverse_range(c, 0, L, h->ha, h->h0, released));
  if (side_used) MW_TRY_RC(flush_carried(c, &carry, h->side));
  for (size_t k = 0; k < h->groups.size(); ++k) {
    const auto& g = h->groups[k];
    if (g.count > 1) {
      if (!overlap) MW_TRY_RC(phase3_group(c, g.first, g.count, s, &carry));
    } else {
      MW_TRY_RC(flush_carried(c, &carry, s));
      const auto& st = h->stretches[g.first];
      MW_TRY_RC(phase3_range(c, st.lo, st.hi, st.lo == 0 ? c.x : h->layers[st.lo - 1].xck,
                             st.lo == 0 ? h->h0 : h->layers[st.lo - 1].ckpt));
    }
  }
  MW_TRY_RC(flush_carried(c, &carry, s));
  if (side_used) {
    MW_HIP(hipEventRecord(h->events[h->groups.size() + 1], h->side));
    MW_HIP(hipStreamWaitEvent(s, h->events[h->groups.size() + 1], 0));
  }
  return MW_OK;
}

int run_moonwalk(mw_handle* h, const float* x, const float* target, float* grads_out, float* loss_out, hipStream_t s,
                 float apply_lr) {
  const int B = h->B, L = h->L;
  const Step c{h, s, x, grads_out, apply_lr};
  for (auto& n : h->launches) n = 0;
  MW_LAUNCH(h, s, MW_KCLASS_EW, ew_fill_u32(h->status, 0u, 3, s));
  const float* x_L = nullptr;

  if (h->S <= 0) {
    // Phase I: forward, keep sign masks only; loss and output cotangent; Phase II; Phase III
    MW_TRY_RC(forward_range(c, 0, L, x, 0, &x_L));
    MW_TRY_RC(frag_index_range(c, 0, L));
    MW_LAUNCH(h, s, MW_KCLASS_EW, ew_loss_grad(x_L, target, B, h->layers[L - 1].d_out, h->loss_scale, h->ha, loss_out, h->loss_scratch, s, h->status + 3));
    if (h->group_width > 0) return reverse_and_sweep(c);
    MW_TRY_RC(reverse_range(c, 0, L, h->ha, h->h0));
    return phase3_range(c, 0, L, x, h->h0);
  }

  // Segments of S layers. Phase I keeps x_{S}, x_{2S}, ... (and, for the top segment, already the
  // masks); then the segments are finished from the top down, each with the exact cotangent at
  // its output as the seed of its reverse pass and the exact cotangent at its input as the seed
  // of its Phase III.
  const int S = h->S, nseg = (L + S - 1) / S;
  MW_TRY_RC(forward_range(c, 0, L, x, (nseg - 1) * S, &x_L));
  MW_LAUNCH(h, s, MW_KCLASS_EW, ew_loss_grad(x_L, target, B, h->layers[L - 1].d_out, h->loss_scale, h->hseg[(nseg - 1) & 1], loss_out,
                                             h->loss_scratch, s, h->status + 3));
  for (int k = nseg - 1; k >= 0; --k) {
    const int lo = k * S, hi = (lo + S < L) ? lo + S : L;
    const float* x_seg = (lo == 0) ? x : h->layers[lo - 1].xck;
    if (k != nseg - 1) {
      const float* unused = nullptr;
      MW_TRY_RC(forward_range(c, lo, hi, x_seg, lo, &unused));
    }
    MW_TRY_RC(frag_index_range(c, lo, hi));
    float* h_bottom = (lo == 0) ? h->h0 : h->hseg[(k - 1) & 1];
    MW_TRY_RC(reverse_range(c, lo, hi, h->hseg[k & 1], h_bottom));
    MW_TRY_RC(phase3_range(c, lo, hi, x_seg, h_bottom));
  }
  return MW_OK;
}

// ||E - I||_F of an n x n matrix, folded into *out as a running maximum (stream-ordered).
// P <- right inverse of the CURRENT W, starting from the P held (right inverse of nearby weights):
//   P_0 = (P P^T) W            P P^T = (W_old W_old^T)^{-1}: a first-order guess whose rows lie in the
//                              row space of the new W, so that every iterate stays the minimum-norm one
//                              (a square layer has one inverse only: there P_0 = P, no start products)
//   P_{k+1} = (2 I - P_k W^T) P_k     Newton-Schulz; the residual I - P W^T squares per iteration
// Consecutive layers of one shape are refreshed side by side, as many (up to REFRESH_SETS) as it takes to
// fill the chip with 128 x 128 tiles: each step is then one grouped product over all of them (a
// 1024 x 1024 x 1024 product alone fills a quarter of the chip with the tile that suits it). Scratch
// (d_out^2 + d_out d_in floats per layer in flight) and the pointer table are allocated on first use and kept.
constexpr int REFRESH_SETS = 8;

int refresh_one_layer(mw_handle* h, Layer& l, int iters, float* residual_out, hipStream_t s) {
  const int n = l.d_out, m = l.d_in;
  float* S = h->refresh_work;
  float* Q = S + (((size_t)n * n + 63) / 64) * 64;
  float* cur = (iters % 2 == 1) ? Q : l.P;
  float* other = (cur == Q) ? l.P : Q;
  if (n == m) {  // a square layer starts from the inverse it has
    if (cur != l.P) MW_HIP(ew_copy(l.P, cur, (int64_t)n * m, s));
  } else {
    MW_HIP(gemm_plain(OP_NT, TILE_AUTO, n, n, m, 1.f, l.P, m, l.P, m, 0.f, S, n, nullptr, s));
    MW_HIP(gemm_plain(OP_NN, TILE_AUTO, n, m, n, 1.f, S, n, l.W, m, 0.f, cur, m, nullptr, s));
  }
  for (int it = 0; it < iters; ++it) {
    MW_HIP(gemm_plain(OP_NT, TILE_AUTO, n, n, m, 1.f, cur, m, l.W, m, 0.f, S, n, nullptr, s));
    if (residual_out && it == iters - 1) MW_HIP(ew_identity_residual(S, n, h->loss_scratch, residual_out, s));
    MW_HIP(ew_copy(cur, other, (int64_t)n * m, s));
    MW_HIP(gemm_plain(OP_NN, TILE_AUTO, n, m, n, -1.f, S, n, cur, m, 2.f, other, m, nullptr, s));
    float* t = cur;
    cur = other;
    other = t;
  }
  return MW_OK;
}

int refresh_plan(mw_handle* h) {
  auto round64 = [](size_t v) { return (v + 63) / 64 * 64; };  // slots start on 256-byte boundaries
  const int L = h->L;
  std::vector<mw_handle::RefreshRun> runs;
  size_t total = 0, n_tab = 2 * (size_t)L;
  for (int l0 = 0; l0 < L;) {
    const int n = h->layers[l0].d_out, m = h->layers[l0].d_in;
    int len = 0;
    bool vec = n % 4 == 0 && m % 4 == 0;
    while (l0 + len < L && h->layers[l0 + len].d_out == n && h->layers[l0 + len].d_in == m) {
      vec = vec && ((reinterpret_cast<uintptr_t>(h->layers[l0 + len].P) | reinterpret_cast<uintptr_t>(h->layers[l0 + len].W)) & 15) == 0;
      ++len;
    }
    // layers side by side: enough for two 128 x 128 tiles per CU in the smaller of the two products
    const int64_t tiles = (int64_t)((n + 127) / 128) * ((n + 127) / 128);
    int sets = (int)((512 + tiles - 1) / tiles);
    if (sets > REFRESH_SETS) sets = REFRESH_SETS;
    if (sets > len) sets = len;
    if (!vec || sets < 1) sets = 1;
    const size_t q_off = round64((size_t)n * n), slot = q_off + round64((size_t)n * m);
    runs.push_back({l0, len, sets, vec, n_tab, slot, q_off});
    if ((size_t)sets * slot > total) total = (size_t)sets * slot;
    if (vec) n_tab += 2 * (size_t)sets;
    l0 += len;
  }
  float* work = static_cast<float*>(h->alloc(total * sizeof(float), &h->st.bytes_mw_scratch));
  if (!work) return MW_ERR_OOM;
  const float** tab = static_cast<const float**>(h->alloc(n_tab * sizeof(float*), &h->st.bytes_mw_scratch));
  if (!tab) return MW_ERR_OOM;
  std::vector<const float*> host(n_tab);
  for (int i = 0; i < L; ++i) {
    host[i] = h->layers[i].P;
    host[L + i] = h->layers[i].W;
  }
  for (auto& r : runs)
    for (int j = 0; r.vec && j < r.sets; ++j) {
      host[r.tab_off + j] = work + (size_t)j * r.slot;
      host[r.tab_off + r.sets + j] = work + (size_t)j * r.slot + r.q_off;
    }
  MW_HIP(hipMemcpy(tab, host.data(), n_tab * sizeof(float*), hipMemcpyHostToDevice));
  h->refresh_work = work;
  h->refresh_tab = tab;
  h->refresh_runs = std::move(runs);
  return MW_OK;
}

int refresh_newton_schulz(mw_handle* h, int iters, float* residual_out, hipStream_t s) {
  const int L = h->L;
  if (!h->refresh_work) {
    int rc = refresh_plan(h);
    if (rc != MW_OK) return rc;
  }
  if (residual_out) MW_HIP(ew_fill_f32(residual_out, iters >= 1 ? 0.f : -1.f, 1, s));
  auto out = [](const float* const* t) { return reinterpret_cast<float* const*>(const_cast<float**>(const_cast<const float**>(t))); };
  for (const auto& r : h->refresh_runs) {
    const int n = h->layers[r.l0].d_out, m = h->layers[r.l0].d_in;
    for (int l0 = r.l0; l0 < r.l0 + r.len;) {
      const int g = (r.l0 + r.len - l0 < r.sets) ? r.l0 + r.len - l0 : r.sets;
      if (!r.vec) {
        int rc = refresh_one_layer(h, h->layers[l0], iters, residual_out, s);
        if (rc != MW_OK) return rc;
        l0 += 1;
        continue;
      }
      const float* const* Pt = h->refresh_tab + l0;
      const float* const* Wt = h->refresh_tab + L + l0;
      const float* const* St = h->refresh_tab + r.tab_off;
      const float* const* Qt = St + r.sets;
      const float* const* cur = (iters % 2 == 1) ? Qt : Pt;
      const float* const* other = (cur == Qt) ? Pt : Qt;
      if (n == m) {  // square layers start from the inverses they have
        if (cur != Pt)
          for (int j = 0; j < g; ++j)
            MW_HIP(ew_copy(h->layers[l0 + j].P, h->refresh_work + (size_t)j * r.slot + r.q_off, (int64_t)n * m, s));
      } else {
        MW_HIP(gemm_grouped(OP_NT, g, n, n, m, 1.f, Pt, m, Pt, m, 0.f, nullptr, out(St), n, s));
        MW_HIP(gemm_grouped(OP_NN, g, n, m, n, 1.f, St, n, Wt, m, 0.f, nullptr, out(cur), m, s));
      }
      for (int it = 0; it < iters; ++it) {
        if (h->refresh_bf16) {
          // S = I - cur W^T in fp32 (the difference is where the digits are lost); other = cur + S cur, the small
          // correction S cur with its operands rounded to bf16 in front of the matrix unit, summed and added in fp32
          MW_HIP(gemm_grouped(OP_NT, g, n, n, m, -1.f, cur, m, Wt, m, 0.f, nullptr, out(St), n, s, 1.f));
          if (residual_out && it == iters - 1)
            MW_HIP(ew_identity_residual_sets(h->refresh_work, (int64_t)r.slot, g, n, h->loss_scratch, residual_out, s, false));
          MW_HIP(gemm_grouped(OP_NN, g, n, m, n, 1.f, St, n, cur, m, 1.f, cur, out(other), m, s, 0.f, true));
          const float* const* t = cur;
          cur = other;
          other = t;
          continue;
        }
        MW_HIP(gemm_grouped(OP_NT, g, n, n, m, 1.f, cur, m, Wt, m, 0.f, nullptr, out(St), n, s));
        if (residual_out && it == iters - 1)
          MW_HIP(ew_identity_residual_sets(h->refresh_work, (int64_t)r.slot, g, n, h->loss_scratch, residual_out, s));
        // other = 2 cur - S cur, the addend read from cur by the epilogue
        MW_HIP(gemm_grouped(OP_NN, g, n, m, n, -1.f, St, n, cur, m, 2.f, cur, out(other), m, s));
        const float* const* t = cur;
        cur = other;
        other = t;
      }
      l0 += g;
    }
  }
  return MW_OK;
}

}  // namespace

extern "C" {

int moonwalk_grad(mw_handle_t* h, const float* x, const float* target, float* grads_out, float* loss_out,
                  void* hip_stream) {
  if (!h || !x || !target || !grads_out) return MW_ERR_INVALID_ARG;
  if (!(h->plan & MW_PLAN_MOONWALK)) return MW_ERR_NOT_PLANNED;
  return run_moonwalk(h, x, target, grads_out, loss_out, static_cast<hipStream_t>(hip_stream), 0.f);
}

int moonwalk_refresh_incremental(mw_handle_t* h, int32_t iters, float* residual_out, void* hip_stream) {
  if (!h || iters < 0 || iters > 16) return MW_ERR_INVALID_ARG;
  if (!(h->plan & MW_PLAN_MOONWALK)) return MW_ERR_NOT_PLANNED;
  return refresh_newton_schulz(h, iters, residual_out, static_cast<hipStream_t>(hip_stream));
}

int moonwalk_sgd_step(mw_handle_t* h, const float* x, const float* target, float lr, int32_t refresh_iters,
                      float* loss_out, float* residual_out, void* hip_stream) {
  if (!h || !x || !target || !std::isfinite(lr) || lr == 0.f || refresh_iters > 16) return MW_ERR_INVALID_ARG;
  if (!(h->plan & MW_PLAN_MOONWALK) || !h->fuse) return MW_ERR_NOT_PLANNED;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int rc = run_moonwalk(h, x, target, nullptr, loss_out, s, lr);
  if (rc != MW_OK || refresh_iters < 0) return rc;
  return refresh_newton_schulz(h, refresh_iters, residual_out, s);
}

int backprop_grad(mw_handle_t* h, const float* x, const float* target, float* grads_out, float* loss_out,
                  void* hip_stream) {
  if (!h || !x || !target || !grads_out) return MW_ERR_INVALID_ARG;
  if (!(h->plan & MW_PLAN_BACKPROP)) return MW_ERR_NOT_PLANNED;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int B = h->B, L = h->L;
  for (auto& c : h->launches) c = 0;
  // forward, every activation stored
  const float* xin = x;
  for (int i = 0; i < L; ++i) {
    Layer& l = h->layers[i];
    MW_LAUNCH(h, s, MW_KCLASS_FWD, gemm_fwd_act(TILE_AUTO, B, l.d_out, l.d_in, xin, l.W, l.b, l.alpha, l.act, nullptr, s));
    xin = l.act;
  }
  float* hbuf[2] = {h->bp_ha, h->bp_hb};
  MW_LAUNCH(h, s, MW_KCLASS_EW, ew_loss_grad(xin, target, B, h->layers[L - 1].d_out, h->loss_scale, hbuf[0], loss_out, h->loss_scratch, s,
                                             h->status + 3));
  const float inv_scale = 1.0f / h->loss_scale;
  int sel = 0;
  for (int i = L - 1; i >= 0; --i) {
    Layer& l = h->layers[i];
    const float* xprev = (i == 0) ? x : h->layers[i - 1].act;
    // dW_i = (h_i .* f'(x_i))^T x_{i-1}, db_i = column sums, and (except for the first layer, whose
    // input cotangent nobody needs) h_{i-1} = (h_i .* f'(x_i)) W_i: one launch for both products
    BpLayerArgs a{B, l.d_out, l.d_in, hbuf[sel], l.act, l.alpha, xprev, l.W, inv_scale,
                  grads_out + l.dW_off, grads_out + l.db_off, i > 0 ? hbuf[sel ^ 1] : nullptr};
    if (h->class_filter < 0) {
      MW_LAUNCH(h, s, MW_KCLASS_PHASE3, gemm_bp_layer(a, s));
    } else {
      const int tile_r = (i > 0) ? pick_tile(B, l.d_in, l.d_out) : TILE_AUTO;
      MW_LAUNCH(h, s, MW_KCLASS_DW, gemm_dw_act(pick_tile_dw(l.d_out, l.d_in, B, tile_r, false), l.d_out, l.d_in, B, a.Hy, a.act, a.alpha,
                                                a.Xprev, a.scale, a.dW, a.db, s));
      if (i > 0) MW_LAUNCH(h, s, MW_KCLASS_REV, gemm_rev_act(tile_r, B, l.d_in, l.d_out, a.Hy, a.act, a.alpha, a.W, a.Hout, s));
    }
    if (i > 0) sel ^= 1;
  }
  return MW_OK;
}

int moonwalk_grad_layout(const mw_handle_t* h, size_t* total_floats, size_t* dW_off, size_t* db_off) {
  if (!h) return MW_ERR_INVALID_ARG;
  if (total_floats) *total_floats = h->total_floats;
  for (int i = 0; i < h->L; ++i) {
    if (dW_off) dW_off[i] = h->layers[i].dW_off;
    if (db_off) db_off[i] = h->layers[i].db_off;
  }
  return MW_OK;
}

int moonwalk_memory_stats(mw_handle_t* h, mw_memstats_t* out) {
  if (!h || !out) return MW_ERR_INVALID_ARG;
  uint32_t status[4] = {0, 0, 0, 0};  // the words a gradient step writes
  uint64_t frag_total = 0;
  MW_HIP(hipDeviceSynchronize());
  MW_HIP(hipMemcpy(status, h->status, sizeof(status), hipMemcpyDeviceToHost));
  if (h->n_relu > 0)
    MW_HIP(hipMemcpy(&frag_total, h->frag_bases + h->n_relu, sizeof(uint64_t), hipMemcpyDeviceToHost));
  *out = h->st;
  out->bytes_live = h->live;
  out->bytes_peak = h->peak;
  out->bytes_setup_peak = h->setup_peak;
  out->frag_used = frag_total;
  out->sign_mismatches = (uint64_t)status[0] | ((uint64_t)status[1] << 32);
  out->frag_overflow = status[2] ? 1 : 0;
  out->nonfinite_loss = status[3] ? 1 : 0;
  out->phase3_group_width = h->group_width;
  if (out->frag_overflow) return MW_ERR_FRAG_OVERFLOW;
  if (out->nonfinite_loss) return MW_ERR_NONFINITE;
  if (out->sign_mismatches) return MW_ERR_SIGN_MISMATCH;
  return MW_OK;
}

int moonwalk_debug_fetch(mw_handle_t* h, int32_t layer, int32_t what, void* host_dst, size_t cap, size_t* n_bytes) {
  if (!h) return MW_ERR_INVALID_ARG;
  if (what != MW_FETCH_H0 && (layer < 0 || layer >= h->L)) return MW_ERR_INVALID_ARG;
  MW_HIP(hipDeviceSynchronize());
  const size_t B = (size_t)h->B;
  const void* src = nullptr;
  size_t bytes = 0;
  const Layer* l = (what == MW_FETCH_H0) ? nullptr : &h->layers[layer];
  // with segments, masks and fragments exist for one segment at a time: after a step, the first one
  if (h->S > 0 && layer >= h->S &&
      (what == MW_FETCH_MASK || what == MW_FETCH_FRAG_OFFSETS || what == MW_FETCH_FRAG_BASE || what == MW_FETCH_FRAG))
    return MW_ERR_INVALID_ARG;
  uint64_t base = 0;
  switch (what) {
    case MW_FETCH_MASK:
      src = l->mask; bytes = l->mask_words * 8; break;
    case MW_FETCH_FRAG_OFFSETS:
      src = l->offsets; bytes = l->offsets ? (l->mask_words + 1) * 4 : 0; break;
    case MW_FETCH_FRAG_BASE:
      if (l->relu_slot < 0) return MW_ERR_INVALID_ARG;
      src = h->frag_bases + l->relu_slot; bytes = 8; break;
    case MW_FETCH_FRAG: {
      if (l->relu_slot < 0) return MW_ERR_INVALID_ARG;
      uint32_t n0 = 0;
      MW_HIP(hipMemcpy(&base, h->frag_bases + l->relu_slot, 8, hipMemcpyDeviceToHost));
      MW_HIP(hipMemcpy(&n0, l->offsets + l->mask_words, 4, hipMemcpyDeviceToHost));
      if (base + n0 > h->frag_capacity) return MW_ERR_FRAG_OVERFLOW;
      src = h->frag + base; bytes = (size_t)n0 * 4; break;
    }
    case MW_FETCH_H0:
      src = h->h0; bytes = B * h->layers[0].d_in * 4; break;
    case MW_FETCH_P:
      src = l->P; bytes = (size_t)l->d_out * l->d_in * 4; break;
    case MW_FETCH_CHECKPOINT:
      src = l->ckpt; bytes = B * l->d_out * 4; break;
    case MW_FETCH_Z:
      src = l->dbg_z; bytes = B * l->d_out * 4; break;
    case MW_FETCH_H:
      src = h->debug_keep ? (l->ckpt ? l->ckpt : l->dbg_h) : nullptr; bytes = B * l->d_out * 4; break;
    case MW_FETCH_H_FORWARD:
      src = l->dbg_h3; bytes = B * l->d_out * 4; break;
    default:
      return MW_ERR_INVALID_ARG;
  }
  if (!src) return MW_ERR_INVALID_ARG;
  if (n_bytes) *n_bytes = bytes;
  if (!host_dst && cap == 0) return MW_OK;  // size query
  if (!host_dst || cap < bytes) return MW_ERR_INVALID_ARG;
  if (bytes) MW_HIP(hipMemcpy(host_dst, src, bytes, hipMemcpyDeviceToHost));
  return MW_OK;
}

int moonwalk_profile_filter(mw_handle_t* h, int32_t kclass) {
  if (!h || kclass < -1 || kclass >= MW_KCLASS_COUNT) return MW_ERR_INVALID_ARG;
  h->class_filter = kclass;
  return MW_OK;
}

int moonwalk_profile_launches(const mw_handle_t* h, int32_t kclass, uint64_t* launches) {
  if (!h || !launches || kclass < 0 || kclass >= MW_KCLASS_COUNT) return MW_ERR_INVALID_ARG;
  *launches = h->launches[kclass];
  return MW_OK;
}

void moonwalk_destroy(mw_handle_t* h) {
  if (!h) return;
  (void)hipDeviceSynchronize();
  h->release_all();
  delete h;
}

const char* moonwalk_strerror(int code) {
  switch (code) {
    case MW_OK: return "ok";
    case MW_ERR_INVALID_ARG: return "invalid argument";
    case MW_ERR_NOT_SUBMERSIVE: return "layer is not a submersion (d_out > d_in or W W^T not positive definite)";
    case MW_ERR_OOM: return "device allocator returned NULL";
    case MW_ERR_FRAG_OVERFLOW: return "fragment store overflow";
    case MW_ERR_HIP: return g_hip_error_text.c_str();
    case MW_ERR_SIGN_MISMATCH: return "recomputed activation signs differ from the stored masks";
    case MW_ERR_NOT_PLANNED: return "handle was planned without this entry point";
    case MW_ERR_TOO_LARGE: return "input larger than the fixed scratch array of an entry point that allocates nothing";
    case MW_ERR_NONFINITE: return "the loss of the last gradient step was NaN or infinite";
    default: return "unknown error code";
  }
}

// ------------------------------------------------------------------------------ kernel-level entries

int mw_gemm_f32(int32_t op, int32_t tile, int32_t M, int32_t N, int32_t K, float alpha, const float* A, int32_t lda,
                const float* B, int32_t ldb, float beta, float* C, int32_t ldc, void* hip_stream) {
  if (M < 0 || N < 0 || K < 0 || !C || (K > 0 && (!A || !B))) return MW_ERR_INVALID_ARG;
  if (op < MW_GEMM_NT || op > MW_GEMM_TN || tile < MW_TILE_AUTO || tile > MW_TILE_64X128) return MW_ERR_INVALID_ARG;
  // leading dimensions must cover the fast index of each operand
  const int a_fast = (op == MW_GEMM_TN) ? M : K, b_fast = (op == MW_GEMM_NT) ? K : N;
  if (lda < a_fast || ldb < b_fast || ldc < N) return MW_ERR_INVALID_ARG;
  // the kernels address every operand with 31-bit byte offsets, row strides included
  auto too_large = [](int64_t n_outer, int64_t n_inner, int64_t ld) {
    return n_outer > 0 && n_inner > 0 && ((n_outer - 1) * ld + n_inner) * 4 >= (int64_t)0x7FFFFFFF;
  };
  if (too_large(op == MW_GEMM_TN ? K : M, a_fast, lda) || too_large(op == MW_GEMM_NT ? N : K, b_fast, ldb) ||
      too_large(M, N, ldc))
    return MW_ERR_INVALID_ARG;
  MW_HIP(gemm_plain(op, tile, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, nullptr, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

int mw_bias_act_mask(const float* zin, const float* bias, int64_t rows, int32_t d, float alpha, float* x,
                     uint64_t* mask, void* hip_stream) {
  if (rows < 0 || d <= 0 || (rows > 0 && (!zin || !x || !mask))) return MW_ERR_INVALID_ARG;
  MW_HIP(ew_bias_act_mask(zin, bias, rows, d, alpha, x, mask, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

int mw_rev_scale(const float* h, const uint64_t* mask, int64_t n, float alpha, float* ct_z, void* hip_stream) {
  if (n < 0 || (n > 0 && (!h || !mask || !ct_z))) return MW_ERR_INVALID_ARG;
  MW_HIP(ew_rev_scale(h, mask, n, alpha, ct_z, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

size_t mw_frag_offsets_work_words(int64_t n) { return ew_frag_scan_words(n); }

int mw_frag_offsets(const uint64_t* mask, int64_t n, uint32_t* offsets, uint32_t* work, void* hip_stream) {
  if (n < 0 || !offsets || !work || (n > 0 && !mask)) return MW_ERR_INVALID_ARG;
  if (n > (int64_t)0xFFFFFFFFll) return MW_ERR_INVALID_ARG;
  MW_HIP(ew_frag_offsets(mask, n, offsets, work, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

int mw_frag_compact(const float* h, const uint64_t* mask, const uint32_t* offsets, int64_t n, float* frag,
                    uint64_t capacity, int32_t* overflow_flag, void* hip_stream) {
  if (n < 0 || (n > 0 && (!h || !mask || !offsets || !frag))) return MW_ERR_INVALID_ARG;
  MW_HIP(ew_frag_compact(h, mask, offsets, n, frag, nullptr, capacity, overflow_flag, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

int mw_vijp_epilogue(const float* z, float* ct_z, int64_t rows, int32_t d, float alpha, const uint64_t* mask,
                     const uint32_t* offsets, const float* frag, float* x, float* h_y, void* hip_stream) {
  if (rows < 0 || d <= 0 || !(alpha >= 0.f)) return MW_ERR_INVALID_ARG;
  if (rows > 0 && (!z || !ct_z || !x || !h_y)) return MW_ERR_INVALID_ARG;
  if (rows > 0 && alpha == 0.f && (!mask || !offsets || !frag)) return MW_ERR_INVALID_ARG;
  MW_HIP(ew_vijp_epilogue(z, ct_z, rows, d, alpha, mask, offsets, frag, nullptr, ~0ull, x, h_y, nullptr,
                          static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

int mw_colsum(const float* a, int64_t rows, int32_t d, float scale, float* out, void* hip_stream) {
  if (rows < 0 || d <= 0 || !out || (rows > 0 && !a)) return MW_ERR_INVALID_ARG;
  MW_HIP(ew_colsum(a, rows, d, scale, out, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

size_t mw_colsum_work_floats(int32_t d) { return d > 0 ? (size_t)COLSUM_MAX_SLICES * (size_t)d : 0; }

int mw_colsum_wide(const float* a, int64_t rows, int32_t d, float scale, float* out, float* work, void* hip_stream) {
  if (rows < 0 || d <= 0 || !out || !work || (rows > 0 && !a)) return MW_ERR_INVALID_ARG;
  MW_HIP(ew_colsum_wide(a, rows, d, scale, 0.f, out, work, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

size_t mw_colsum_noalloc_max_floats(void) { return ew_colsum_static_floats(); }

int mw_colsum_wide_noalloc(const float* a, int64_t rows, int32_t d, float scale, float* out, void* hip_stream) {
  if (rows < 0 || d <= 0 || !out || (rows > 0 && !a)) return MW_ERR_INVALID_ARG;
  bool too_large = false;
  MW_HIP(ew_colsum_wide_static(a, rows, d, scale, out, static_cast<hipStream_t>(hip_stream), &too_large));
  if (too_large) return MW_ERR_TOO_LARGE;
  return MW_OK;
}

size_t mw_loss_scratch_doubles(void) { return (size_t)LOSS_BLOCKS; }

int mw_loss_grad(const float* xL, const float* t, int64_t rows, int32_t d, float scale, float* hL, float* loss,
                 double* scratch, void* hip_stream) {
  if (rows <= 0 || d <= 0 || !xL || !t || !hL || !scratch) return MW_ERR_INVALID_ARG;
  MW_HIP(ew_loss_grad(xL, t, rows, d, scale, hL, loss, scratch, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

int mw_copy_f32(const float* src, float* dst, int64_t n, void* hip_stream) {
  if (n < 0 || (n > 0 && (!src || !dst))) return MW_ERR_INVALID_ARG;
  MW_HIP(ew_copy(src, dst, n, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

int mw_probe_operand_stream(int32_t M, int32_t N, int32_t K, int32_t tile, const float* A, const float* B, float* sink,
                            int32_t repeats, void* hip_stream) {
  if (!A || !B || !sink || repeats < 1) return MW_ERR_INVALID_ARG;
  if (M <= 0 || N <= 0 || K <= 0 || (tile != 16 && tile != 32 && tile != 64) || M % tile || N % tile || K % 256)
    return MW_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 15) return MW_ERR_INVALID_ARG;
  for (int32_t i = 0; i < repeats; ++i)
    MW_HIP(ew_operand_stream(A, B, M, N, K, tile, sink, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

}  // extern "C"
