// Moonwalk on convolutional layers: handle, buffer plan and the gradient drivers behind the C ABI.
// Two kinds of layer: submersive 2-D convolutions (lemma on submersive convolutional layers; the
// paper's fully parallel 2-D setting), and length-preserving 1-D convolutions with fragmental
// checkpointing (section on fragmental gradient checkpointing and its appendix).
//
// A convolution is run as the library's fp32 MFMA GEMMs on patch matrices. Where the channel
// counts allow it (C_in and C_out multiples of 32) the patch matrix never exists in memory: the
// products gather their operand from the image (conv_gemm.h). The forward product ends in the
// activation and the sign mask; the input cotangent is one product per stride class of input
// pixels, ending in the previous layer's slope; Phase III of a submersive layer is one kernel
// (recomputed forward, channel solve, vijp epilogue), of a fragmental layer the block-wise rebuild
// of ct_z followed by one kernel (recomputed forward, vijp epilogue); the weight gradient is split
// over the patch rows. Submersive layers with other channel counts go through a bounded patch
// buffer in image chunks instead (im2col, plain GEMMs, col2im, a fixed-order sum).
// The vijp of a submersive convolution, in the fully parallel case k <= p + s, is a triangular
// solve over channels at every output position, done as a product with the inverse of the
// channel-triangular tap; the cotangents Phase III starts from are kept in the form it reads them.
// Wider kernels couple each output position with earlier ones: the same solve for all positions,
// then a sweep over the anti-diagonals of the output grid that subtracts the earlier positions'
// contributions (one gathered product per diagonal), on cotangents kept whole.
#include "../../include/moonwalk.h"

#include <cmath>
#include <utility>
#include <vector>

#include "mw_internal.h"

using namespace mw;

namespace {

#define CV_HIP(expr)                                              \
  do {                                                            \
    hipError_t e__ = (expr);                                      \
    if (e__ != hipSuccess) return record_hip_failure(e__, #expr); \
  } while (0)

void* cv_default_alloc(size_t bytes, void*) {
  void* p = nullptr;
  if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
  return p;
}
void cv_default_free(void* p, void*) { (void)hipFree(p); }

struct ConvLayer {
  int Cin = 0, Cout = 0, k = 0, s = 0, p = 0;
  int kind = MW_CONV_SUBMERSIVE;
  int kh = 0, kw = 0, ph = 0, pw = 0;  // the kernel as the products see it: k x k with padding p, or 1 x k for a 1-D layer
  int block = 0;                // fragmental layers: positions per block
  float* frag = nullptr;        // fragmental layers: [B W / block][k - 1][Cout], the first k - 1 positions of every block of ct_z
  float* Arec = nullptr;        // fragmental layers: [Cout][(k - 1) Cout], T^{-1} w[u][:Cout] side by side for u = k - 1 .. 1
  int reach = 0;                // submersive layers: earlier output positions per dimension in a vijp equation, (k - 1 - p) / s;
                                // 0 is the fully parallel case
  float* Asweep = nullptr;      // reach > 0: [Cout][((reach + 1)^2 - 1) Cout], T^{-1} w[p + a s][p + b s][:Cout] by tap slot
  bool whole_h() const { return kind == MW_CONV_FRAGMENTAL_1D || reach > 0; }  // the vijp reads more of h than sub(h)
  int Hin = 0, Win = 0, Ho = 0, Wo = 0;
  int K = 0;            // k k Cin: columns of the patch matrix
  int64_t rows = 0;     // B Ho Wo: rows of the patch matrix
  int64_t n_in = 0, n_out = 0;  // elements of the input / output activation
  const float* w = nullptr;     // [k][k][Cin][Cout] = [K][Cout]
  const float* b = nullptr;
  float alpha = 0.f;
  float* Tinv = nullptr;        // inverse of the tap at (p, p), [Cout][Cout]
  float* wrev = nullptr;        // taps regrouped for the gathered input-cotangent product, [K][Cout] floats
  bool gather_rev = false;      // that product instead of patches + col2im
  uint64_t* mask = nullptr;
  size_t mask_words = 0;
  float* ckpt = nullptr;        // kept cotangent at this layer's output, as the next layer's vijp reads it:
                                // [next.rows][next.Cout] = the strided positions, the first next.Cout channels
  float* act = nullptr;         // backprop: stored output activation
  size_t dW_off = 0, db_off = 0;
  int chunk_images = 1;         // images per patch-buffer fill
  bool gather = false;          // gathered-operand kernels for forward, Phase III and dW
  int gchunk = 1;               // images per launch of those kernels (2 GiB operand limit)
  ConvGeom geom() const { return ConvGeom{Hin, Win, Cin, Ho, Wo, kh, kw, s, ph, pw}; }
  // the tap whose first Cout rows are the triangular T: (p, p) of a submersive layer, u = 0 of a fragmental one
  const float* tri_tap() const {
    return kind == MW_CONV_FRAGMENTAL_1D ? w : w + ((size_t)(p * k + p) * Cin) * Cout;
  }
  int64_t in_img() const { return (int64_t)Hin * Win * Cin; }     // floats per input image
  int64_t out_img() const { return (int64_t)Ho * Wo * Cout; }     // floats per output image
};

}  // namespace

struct mw_conv_handle {
  std::vector<ConvLayer> layers;
  int B = 0, L = 0, Kre = 0, plan = 0;
  bool h0_full = true;          // h_0 for every input element (else only what the first layer's vijp reads)
  float loss_scale = 1.f;
  void* (*dev_alloc)(size_t, void*) = nullptr;
  void (*dev_free)(void*, void*) = nullptr;
  void* alloc_ctx = nullptr;
  std::vector<std::pair<void*, size_t>> allocs;
  uint64_t live = 0, peak = 0;
  mw_conv_memstats_t st{};
  size_t total_floats = 0;
  float *patches = nullptr, *zbuf = nullptr, *ctz = nullptr, *hsub = nullptr;
  float *dw_part = nullptr, *colsum_part = nullptr;
  float *xa = nullptr, *xb = nullptr, *ha = nullptr, *hb = nullptr, *h0 = nullptr;
  uint32_t* status = nullptr;  // [0..1] sign mismatches (u64), [2] kernel not triangular / zero diagonal, [3] non-finite loss
  double* loss_scratch = nullptr;

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
  void release_all() {
    for (auto& a : allocs) dev_free(a.first, alloc_ctx);
    allocs.clear();
    live = 0;
  }
};

namespace {

template <class T>
bool cv_alloc(mw_conv_handle* h, T** out, size_t count, uint64_t* item) {
  *out = static_cast<T*>(h->alloc(count * sizeof(T), item));
  return *out != nullptr;
}

// everything the library derives from the weights: the tap inverses (Moonwalk) and the regrouped taps
int build_from_weights(mw_conv_handle* h, hipStream_t s) {
  int32_t* flag = reinterpret_cast<int32_t*>(h->status + 2);
  CV_HIP(ew_fill_u32(h->status + 2, 0u, 1, s));
  for (auto& l : h->layers) {
    if (l.wrev) CV_HIP(cv_pack_rev_weights(l.w, l.kh, l.kw, l.s, l.Cin, l.Cout, l.wrev, s));
    if (!l.Tinv) continue;
    CV_HIP(cv_tri_inverse(l.tri_tap(), l.Cout, l.Cout, l.Tinv, flag, s));
    // general vijp: T^{-1} w[p + a s][p + b s][:Cout] for the earlier positions (a, b) != (0, 0), slot (reach - a, reach - b)
    if (l.Asweep) {
      const int n1 = l.reach + 1, Ktot = (n1 * n1 - 1) * l.Cout;
      for (int ky = 0; ky < n1; ++ky)
        for (int kx = 0; kx < n1; ++kx) {
          if (ky == l.reach && kx == l.reach) continue;
          const int u = l.p + (l.reach - ky) * l.s, v = l.p + (l.reach - kx) * l.s;
          CV_HIP(gemm_plain(OP_NN, TILE_AUTO, l.Cout, l.Cout, l.Cout, 1.f, l.Tinv, l.Cout,
                            l.w + ((size_t)(u * l.k + v) * l.Cin) * l.Cout, l.Cout, 0.f,
                            l.Asweep + (size_t)(ky * n1 + kx) * l.Cout, Ktot, nullptr, s));
        }
    }
    // fragmental layers: the recurrence matrices T^{-1} w[u][:Cout] side by side, u = k - 1 .. 1, in the
    // order of the positions j - k + 1 .. j - 1 they multiply: one [Cout][(k - 1) Cout] matrix
    for (int u = 1; l.Arec && u < l.k; ++u)
      CV_HIP(gemm_plain(OP_NN, TILE_AUTO, l.Cout, l.Cout, l.Cout, 1.f, l.Tinv, l.Cout, l.w + (size_t)u * l.Cin * l.Cout, l.Cout, 0.f,
                        l.Arec + (size_t)(l.k - 1 - u) * l.Cout, (int64_t)(l.k - 1) * l.Cout, nullptr, s));
  }
  int32_t bad = 0;
  CV_HIP(hipStreamSynchronize(s));
  CV_HIP(hipMemcpy(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost));
  return bad ? MW_ERR_NOT_SUBMERSIVE : MW_OK;
}

// z (rows [r0, r0 + R) of the layer's output, bias added) = patches(x) w, through the patch buffer
int conv_rows(mw_conv_handle* h, const ConvLayer& l, const float* xin, int64_t r0, int64_t R, float* zout, hipStream_t s) {
  CV_HIP(cv_im2col(xin, l.Hin, l.Win, l.Cin, l.Ho, l.Wo, l.k, l.s, l.p, r0, R, h->patches, s));
  CV_HIP(gemm_plain(OP_NN, TILE_AUTO, (int)R, l.Cout, l.K, 1.f, h->patches, l.K, l.w, l.Cout, 0.f, zout + r0 * l.Cout, l.Cout,
                    l.b, s));
  return MW_OK;
}

// input cotangent of the layer from ct_z (whole layer), image chunk by image chunk: hout (may be NULL
// with ct_out) = h; ct_out (may be NULL) = h times the slope selected by the previous layer's mask.
// Returns through *fused whether ct_out was written (only the gathered kernel can do that).
int conv_input_grad(mw_conv_handle* h, const ConvLayer& l, const float* ctz, float* hout, float* ct_out,
                    const ConvLayer* prev, bool* fused, hipStream_t s) {
  if (fused) *fused = false;
  if (l.gather_rev) {
    // the mask of an image chunk must start on a 32-bit word
    const bool fuse = ct_out && prev && l.Cin % 32 == 0;
    if (!fuse && !hout) return MW_ERR_INVALID_ARG;
    for (int64_t img0 = 0; img0 < h->B; img0 += l.gchunk) {
      const int n_img = (int)((img0 + l.gchunk <= h->B) ? l.gchunk : h->B - img0);
      const int64_t o = img0 * l.in_img();
      CV_HIP(conv_input_cotangent(l.geom(), n_img, l.Cout, ctz + img0 * l.out_img(), l.wrev, hout ? hout + o : nullptr,
                                  fuse ? ct_out + o : nullptr,
                                  fuse ? reinterpret_cast<const uint32_t*>(prev->mask) + o / 32 : nullptr,
                                  fuse ? prev->alpha : 1.f, s));
    }
    if (fused) *fused = fuse;
    return MW_OK;
  }
  if (!hout) return MW_ERR_INVALID_ARG;
  const int64_t per_img = (int64_t)l.Ho * l.Wo;
  for (int64_t img0 = 0; img0 < h->B; img0 += l.chunk_images) {
    const int64_t n_img = (img0 + l.chunk_images <= h->B) ? l.chunk_images : h->B - img0;
    const int64_t r0 = img0 * per_img, R = n_img * per_img;
    // patch cotangents = ct_z w^T: (R x Cout) (K x Cout)^T
    CV_HIP(gemm_plain(OP_NT, TILE_AUTO, (int)R, l.K, l.Cout, 1.f, ctz + r0 * l.Cout, l.Cout, l.w, l.Cout, 0.f, h->patches, l.K,
                      nullptr, s));
    CV_HIP(cv_col2im(h->patches, l.Hin, l.Win, l.Cin, l.Ho, l.Wo, l.k, l.s, l.p, img0, n_img, hout, s));
  }
  return MW_OK;
}

// The part of the layer's input cotangent its own vijp reads, sub(h)[:, :Cout] (the strided positions,
// the first Cout channels), straight from ct_z: in the fully parallel case only the tap at (p, p)
// reaches those entries, so it is ct_z T^T with T the first Cout rows of that tap (Alg. 2 read backwards).
int conv_kept_cotangent(mw_conv_handle* h, const ConvLayer& l, const float* ctz, float* kept, hipStream_t s) {
  const float* tap = l.tri_tap();  // [Cin][Cout]; rows c < Cout are T
  const int64_t per_img = (int64_t)l.Ho * l.Wo;
  for (int64_t img0 = 0; img0 < h->B; img0 += l.gchunk) {
    const int64_t n_img = (img0 + l.gchunk <= h->B) ? l.gchunk : h->B - img0;
    const int64_t r0 = img0 * per_img, R = n_img * per_img;
    CV_HIP(gemm_plain(OP_NT, TILE_AUTO, (int)R, l.Cout, l.Cout, 1.f, ctz + r0 * l.Cout, l.Cout, tap, l.Cout, 0.f,
                      kept + r0 * l.Cout, l.Cout, nullptr, s));
  }
  return MW_OK;
}

// Fragmental layer: ct_z of the whole layer from the incoming cotangent hin [B][1][W][Cin] and the stored
// fragments (section on fragmental gradient checkpointing, its appendix and the fragmental vijp
// algorithm). Rows are (sample, block); position j of every block is one column group of a matrix with
// row stride block * C, so each step of the recurrence
//     ct[., j] = hin[., j - p][:Cout] T^{-T} - sum_{u = 1}^{k-1} ct[., j - u] (T^{-1} w[u][:Cout])^T
// is k plain products over all blocks at once; the steps j = k - 1 .. block - 1 follow one another.
int frag_rebuild(mw_conv_handle* h, const ConvLayer& l, const float* hin, float* ctz, hipStream_t s) {
  const int64_t blocks_per_img = l.Wo / l.block;
  const int64_t ld_ct = (int64_t)l.block * l.Cout, ld_h = (int64_t)l.block * l.Cin;
  const int nfrag = (l.k - 1) * l.Cout;
  for (int64_t img0 = 0; img0 < h->B; img0 += l.gchunk) {
    const int64_t n_img = (img0 + l.gchunk <= h->B) ? l.gchunk : h->B - img0;
    const int64_t r0 = img0 * blocks_per_img, R = n_img * blocks_per_img;
    float* ct = ctz + r0 * ld_ct;
    const float* hi = hin + r0 * ld_h;
    if (nfrag > 0) CV_HIP(cv_copy_rows(l.frag + r0 * nfrag, nfrag, ct, ld_ct, R, nfrag, s));
    for (int j = l.k - 1; j < l.block; ++j) {
      CV_HIP(gemm_plain(OP_NT, TILE_AUTO, (int)R, l.Cout, l.Cout, 1.f, hi + (int64_t)(j - l.p) * l.Cin, ld_h, l.Tinv, l.Cout, 0.f,
                        ct + (int64_t)j * l.Cout, ld_ct, nullptr, s));
      // the k - 1 positions before j are neighbours in a row of ct: one product over all of them
      if (l.k > 1)
        CV_HIP(gemm_plain(OP_NT, TILE_AUTO, (int)R, l.Cout, (l.k - 1) * l.Cout, -1.f, ct + (int64_t)(j - l.k + 1) * l.Cout, ld_ct,
                          l.Arec, (int64_t)(l.k - 1) * l.Cout, 1.f, ct + (int64_t)j * l.Cout, ld_ct, nullptr, s));
    }
  }
  return MW_OK;
}

// Phase II of a fragmental layer: keep the first k - 1 positions of every block of ct_z
int frag_store(mw_conv_handle* h, const ConvLayer& l, const float* ctz, hipStream_t s) {
  const int nfrag = (l.k - 1) * l.Cout;
  if (nfrag == 0) return MW_OK;
  const int64_t rows = (int64_t)h->B * (l.Wo / l.block);
  CV_HIP(cv_copy_rows(ctz, (int64_t)l.block * l.Cout, l.frag, nfrag, rows, nfrag, s));
  return MW_OK;
}

// forward of one layer for the whole batch: xout = act(conv(xin) + b); mask (may be NULL) gets the signs
int conv_forward_layer(mw_conv_handle* h, const ConvLayer& l, const float* xin, float* xout, uint64_t* mask, hipStream_t s) {
  if (l.gather) {
    for (int64_t img0 = 0; img0 < h->B; img0 += l.gchunk) {
      const int n_img = (int)((img0 + l.gchunk <= h->B) ? l.gchunk : h->B - img0);
      uint32_t* m32 = mask ? reinterpret_cast<uint32_t*>(mask) + img0 * l.out_img() / 32 : nullptr;
      CV_HIP(conv_fwd_act(l.geom(), n_img, xin + img0 * l.in_img(), l.w, l.b, l.alpha, l.Cout, xout + img0 * l.out_img(), m32, s));
    }
    return MW_OK;
  }
  const int64_t per_img = (int64_t)l.Ho * l.Wo;
  for (int64_t img0 = 0; img0 < h->B; img0 += l.chunk_images) {
    const int64_t n_img = (img0 + l.chunk_images <= h->B) ? l.chunk_images : h->B - img0;
    int rc = conv_rows(h, l, xin, img0 * per_img, n_img * per_img, xout, s);
    if (rc != MW_OK) return rc;
  }
  CV_HIP(ew_bias_act_mask(xout, nullptr, l.rows, l.Cout, l.alpha, xout, mask, s));  // in place: z -> x, signs packed
  return MW_OK;
}

// dW (+ db) of one layer from its input activation and ct_z, both for the whole batch
// dW = scale * (parameter vjp) + beta0 * dW, likewise db (db may be NULL: not wanted)
int conv_weight_grad(mw_conv_handle* h, const ConvLayer& l, const float* xin, const float* ctz, float scale, float* dW,
                     float* db, hipStream_t s, float beta0 = 0.f) {
  bool first = true;
  if (l.gather) {
    for (int64_t img0 = 0; img0 < h->B; img0 += l.gchunk) {
      const int n_img = (int)((img0 + l.gchunk <= h->B) ? l.gchunk : h->B - img0);
      CV_HIP(conv_dw(l.geom(), n_img, xin + img0 * l.in_img(), ctz + img0 * l.out_img(), l.Cout, scale, first ? beta0 : 1.f, dW,
                     h->dw_part, s));
      first = false;
    }
  } else {
    const int64_t per_img = (int64_t)l.Ho * l.Wo;
    for (int64_t img0 = 0; img0 < h->B; img0 += l.chunk_images) {
      const int64_t n_img = (img0 + l.chunk_images <= h->B) ? l.chunk_images : h->B - img0;
      const int64_t r0 = img0 * per_img, R = n_img * per_img;
      CV_HIP(cv_im2col(xin, l.Hin, l.Win, l.Cin, l.Ho, l.Wo, l.k, l.s, l.p, r0, R, h->patches, s));
      CV_HIP(gemm_plain(OP_TN, TILE_AUTO, l.K, l.Cout, (int)R, scale, h->patches, l.K, ctz + r0 * l.Cout, l.Cout,
                        first ? beta0 : 1.f, dW, l.Cout, nullptr, s));
      first = false;
    }
  }
  if (db) CV_HIP(ew_colsum_wide(ctz, l.rows, l.Cout, scale, beta0, db, h->colsum_part, s));
  return MW_OK;
}

int run_conv_moonwalk(mw_conv_handle* h, const float* x, const float* target, float* grads_out, float* loss_out, bool apply,
                      float lr, hipStream_t s);

}  // namespace

extern "C" {

int moonwalk_conv_setup(mw_conv_handle_t** out, const mw_conv_layer_t* layers, int32_t n_layers,
                        const mw_conv_config_t* cfg, void* hip_stream) {
  if (!out) return MW_ERR_INVALID_ARG;
  *out = nullptr;
  if (!layers || n_layers <= 0 || !cfg || cfg->batch <= 0 || cfg->height <= 0 || cfg->width <= 0) return MW_ERR_INVALID_ARG;
  if (cfg->reseed_interval < 0 || !(cfg->loss_scale > 0.f) || !std::isfinite(cfg->loss_scale)) return MW_ERR_INVALID_ARG;
  if ((cfg->dev_alloc == nullptr) != (cfg->dev_free == nullptr)) return MW_ERR_INVALID_ARG;
  if (cfg->plan & ~(MW_PLAN_MOONWALK | MW_PLAN_BACKPROP)) return MW_ERR_INVALID_ARG;
  if (cfg->kernels != MW_CONV_KERNELS_AUTO && cfg->kernels != MW_CONV_KERNELS_PATCH_MATRIX) return MW_ERR_INVALID_ARG;
  if (cfg->input_cotangent != MW_CONV_H0_FULL && cfg->input_cotangent != MW_CONV_H0_AS_READ) return MW_ERR_INVALID_ARG;
  if (cfg->max_images_per_launch < 0) return MW_ERR_INVALID_ARG;
  int Hc = cfg->height, Wc = cfg->width;
  const int64_t limit = (int64_t)0x7FFFFFFF;
  for (int i = 0; i < n_layers; ++i) {
    const mw_conv_layer_t& l = layers[i];
    if (l.channels_in <= 0 || l.channels_out <= 0 || l.k <= 0 || l.stride <= 0 || l.pad < 0 || !l.w) return MW_ERR_INVALID_ARG;
    if (!(l.alpha > 0.f && l.alpha <= 1.f)) return MW_ERR_INVALID_ARG;
    if (i > 0 && l.channels_in != layers[i - 1].channels_out) return MW_ERR_INVALID_ARG;
    if (l.kind != MW_CONV_SUBMERSIVE && l.kind != MW_CONV_FRAGMENTAL_1D) return MW_ERR_INVALID_ARG;
    if (l.kind != layers[0].kind) return MW_ERR_INVALID_ARG;  // one kind of layer per chain
    if (l.kind == MW_CONV_FRAGMENTAL_1D) {
      // a length-preserving 1-D convolution on a one-row image, cut into whole blocks of at least k - 1
      // positions; channel counts the gathered kernels take; h_0 is needed whole (the rebuild reads every position)
      if (Hc != 1 || l.stride != 1 || l.k % 2 != 1 || l.pad != (l.k - 1) / 2) return MW_ERR_INVALID_ARG;
      if (l.block < l.k - 1 || l.block < 1 || Wc % l.block) return MW_ERR_INVALID_ARG;
      if (l.channels_out > l.channels_in) return MW_ERR_INVALID_ARG;
      if (l.channels_in % 32 || l.channels_out % 32 || cfg->kernels != MW_CONV_KERNELS_AUTO) return MW_ERR_INVALID_ARG;
      if (cfg->input_cotangent != MW_CONV_H0_FULL) return MW_ERR_INVALID_ARG;
      if ((int64_t)l.k * l.channels_in * l.channels_out * 4 >= limit) return MW_ERR_INVALID_ARG;
      if ((int64_t)Wc * l.channels_in >= limit / 4) return MW_ERR_INVALID_ARG;
      continue;  // the length and the single row are kept
    }
    if (Hc + 2 * l.pad < l.k || Wc + 2 * l.pad < l.k) return MW_ERR_INVALID_ARG;
    const int Ho = (Hc + 2 * l.pad - l.k) / l.stride + 1, Wo = (Wc + 2 * l.pad - l.k) / l.stride + 1;
    // conditions (i) of the lemma, and m' <= m
    if (!(l.k > l.pad && l.stride > l.pad && Hc > l.stride * (Ho - 1) && Wc > l.stride * (Wo - 1))) return MW_ERR_NOT_SUBMERSIVE;
    if (l.channels_out > l.channels_in) return MW_ERR_NOT_SUBMERSIVE;
    // k > p + s: earlier output positions enter the equations of the vijp; that sweep exists for the
    // gathered kernels only, and reads every position of the layer's input cotangent
    if (l.k > l.pad + l.stride &&
        (l.channels_in % 32 || l.channels_out % 32 || cfg->kernels != MW_CONV_KERNELS_AUTO || cfg->input_cotangent != MW_CONV_H0_FULL))
      return MW_ERR_INVALID_ARG;
    if ((int64_t)l.k * l.k * l.channels_in * l.channels_out * 4 >= limit) return MW_ERR_INVALID_ARG;
    if ((int64_t)Ho * Wo * l.channels_out >= limit) return MW_ERR_INVALID_ARG;
    Hc = Ho;
    Wc = Wo;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  mw_conv_handle* h = new mw_conv_handle();
  h->B = cfg->batch;
  h->L = n_layers;
  h->Kre = cfg->reseed_interval;
  h->plan = cfg->plan ? cfg->plan : (MW_PLAN_MOONWALK | MW_PLAN_BACKPROP);
  h->loss_scale = cfg->loss_scale;
  h->h0_full = cfg->input_cotangent == MW_CONV_H0_FULL;
  h->dev_alloc = cfg->dev_alloc ? cfg->dev_alloc : cv_default_alloc;
  h->dev_free = cfg->dev_free ? cfg->dev_free : cv_default_free;
  h->alloc_ctx = cfg->alloc_ctx;
  h->layers.resize(n_layers);
  const size_t patch_cap_floats = (cfg->patch_bytes > 0 ? cfg->patch_bytes : ((size_t)256 << 20)) / 4;
  size_t off = 0, max_out = 0, max_odd = 1, max_patch = 0, max_part = 1, max_cout = 1;
  bool any_patch_layer = false, need_patches = false;
  Hc = cfg->height;
  Wc = cfg->width;
  for (int i = 0; i < n_layers; ++i) {
    ConvLayer& l = h->layers[i];
    l.Cin = layers[i].channels_in;
    l.Cout = layers[i].channels_out;
    l.k = layers[i].k;
    l.s = layers[i].stride;
    l.p = layers[i].pad;
    l.kind = layers[i].kind;
    l.block = layers[i].block;
    const bool frag1d = l.kind == MW_CONV_FRAGMENTAL_1D;
    l.reach = frag1d ? 0 : (l.k - 1 - l.p) / l.s;
    l.kh = frag1d ? 1 : l.k;
    l.kw = l.k;
    l.ph = frag1d ? 0 : l.p;
    l.pw = l.p;
    l.w = layers[i].w;
    l.b = layers[i].b;
    l.alpha = layers[i].alpha;
    l.Hin = Hc;
    l.Win = Wc;
    l.Ho = (Hc + 2 * l.ph - l.kh) / l.s + 1;
    l.Wo = (Wc + 2 * l.pw - l.kw) / l.s + 1;
    l.K = l.kh * l.kw * l.Cin;
    l.rows = (int64_t)h->B * l.Ho * l.Wo;
    l.n_in = (int64_t)h->B * l.Hin * l.Win * l.Cin;
    l.n_out = l.rows * l.Cout;
    l.dW_off = off;
    off += (size_t)l.K * l.Cout;
    l.db_off = off;
    off += (size_t)l.Cout;
    const size_t per_img = (size_t)l.Ho * l.Wo * l.K;
    size_t ci = patch_cap_floats / per_img;
    // one fill must stay below the 2 GiB operand limit of the GEMMs whatever the caller asked for
    while (ci > 1 && ci * per_img * 4 >= (size_t)limit) --ci;
    if (ci < 1) ci = 1;
    if (ci > (size_t)h->B) ci = (size_t)h->B;
    if (per_img * 4 >= (size_t)limit) {
      delete h;
      return MW_ERR_INVALID_ARG;  // a single image's patches do not fit a GEMM operand
    }
    l.chunk_images = (int)ci;
    const ConvGeom g = l.geom();
    int64_t gmax = conv_gather_max_images(g, l.Cout);
    if (gmax < 1) {
      delete h;
      return MW_ERR_INVALID_ARG;  // a single image does not fit a GEMM operand
    }
    if (cfg->max_images_per_launch > 0 && cfg->max_images_per_launch < gmax) gmax = cfg->max_images_per_launch;
    {
      // as few launches as the 2 GiB operand limit allows, of equal size
      const int64_t n_chunks = (h->B + gmax - 1) / gmax;
      l.gchunk = (int)((h->B + n_chunks - 1) / n_chunks);
    }
    l.gather = cfg->kernels == MW_CONV_KERNELS_AUTO && conv_gather_ok(g, l.Cout, nullptr, l.w);
    l.gather_rev = l.gather && conv_rev_ok(g, l.Cout);
    if (l.gather) {
      const size_t part = conv_dw_part_floats(g, l.gchunk, l.Cout);
      if (part > max_part) max_part = part;
    } else {
      any_patch_layer = true;
    }
    if (!l.gather || !l.gather_rev) need_patches = true;
    if (l.reach > 0 && !l.gather) {  // the general vijp exists for the gathered kernels only
      delete h;
      return MW_ERR_INVALID_ARG;
    }
    if (frag1d) {
      if (!l.gather || !l.gather_rev) {  // setup's checks should have made this impossible
        delete h;
        return MW_ERR_INVALID_ARG;
      }
    }
    if ((size_t)l.Cout > max_cout) max_cout = (size_t)l.Cout;
    if (ci * per_img > max_patch) max_patch = ci * per_img;
    if ((size_t)l.n_out > max_out) max_out = (size_t)l.n_out;
    if ((i & 1) && (size_t)l.n_out > max_odd) max_odd = (size_t)l.n_out;
    Hc = l.Ho;
    Wc = l.Wo;
  }
  h->total_floats = off;

  auto fail = [&](int code) {
    h->release_all();
    delete h;
    return code;
  };
  mw_conv_memstats_t& st = h->st;
  bool ok = cv_alloc(h, &h->status, 4, &st.bytes_scratch);
  ok = ok && cv_alloc(h, &h->loss_scratch, (size_t)LOSS_BLOCKS, &st.bytes_scratch);
  if (need_patches) ok = ok && cv_alloc(h, &h->patches, max_patch, &st.bytes_patches);
  ok = ok && cv_alloc(h, &h->dw_part, max_part, &st.bytes_scratch);
  ok = ok && cv_alloc(h, &h->colsum_part, (size_t)COLSUM_MAX_SLICES * max_cout, &st.bytes_scratch);
  if (!ok) return fail(MW_ERR_OOM);
  hipError_t e = ew_fill_u32(h->status, 0u, 4, stream);
  if (e != hipSuccess) return fail(record_hip_failure(e, "status init"));
  const size_t B = (size_t)h->B;
  if (h->plan & MW_PLAN_MOONWALK) {
    for (auto& l : h->layers) {
      ok = ok && cv_alloc(h, &l.Tinv, (size_t)l.Cout * l.Cout, &st.bytes_tap_inverses);
      if (l.reach > 0) {
        const size_t n1 = (size_t)l.reach + 1;
        ok = ok && cv_alloc(h, &l.Asweep, (n1 * n1 - 1) * l.Cout * l.Cout, &st.bytes_tap_inverses);
      }
      if (l.kind == MW_CONV_FRAGMENTAL_1D && l.k > 1) {
        ok = ok && cv_alloc(h, &l.Arec, (size_t)(l.k - 1) * l.Cout * l.Cout, &st.bytes_tap_inverses);
        ok = ok && cv_alloc(h, &l.frag, (size_t)(l.rows / l.block) * (l.k - 1) * l.Cout, &st.bytes_fragments);
      }
      l.mask_words = ((size_t)l.n_out + 63) / 64;
      ok = ok && cv_alloc(h, &l.mask, l.mask_words, &st.bytes_masks);
      if (ok) {
        e = ew_fill_u32(reinterpret_cast<uint32_t*>(l.mask), 0u, (int64_t)l.mask_words * 2, stream);
        if (e != hipSuccess) return fail(record_hip_failure(e, "mask init"));
      }
    }
    if (!ok) return fail(MW_ERR_OOM);
    if (h->Kre > 0)
      for (int j = 1; j < n_layers; ++j)
        if (j % h->Kre == 0)  // as the next layer reads it: whole where its vijp couples positions
          ok = ok && cv_alloc(h, &h->layers[j - 1].ckpt,
                              h->layers[j].whole_h() ? (size_t)h->layers[j].n_in
                                                                         : (size_t)h->layers[j].rows * h->layers[j].Cout,
                              &st.bytes_checkpoints);
    // activations and cotangents alternate between an "even layer" and an "odd layer" buffer; the odd
    // ones never hold the first layer's output, the largest by far when the resolution shrinks
    ok = ok && cv_alloc(h, &h->xa, max_out, &st.bytes_scratch) && cv_alloc(h, &h->xb, max_odd, &st.bytes_scratch) &&
         cv_alloc(h, &h->ha, max_out, &st.bytes_scratch) && cv_alloc(h, &h->hb, max_odd, &st.bytes_scratch) &&
         cv_alloc(h, &h->ctz, max_out, &st.bytes_scratch) &&
         cv_alloc(h, &h->h0, h->h0_full ? (size_t)h->layers[0].n_in : (size_t)h->layers[0].rows * h->layers[0].Cout,
                  &st.bytes_input_cotangent);
    if (any_patch_layer)  // pre-activations and right-hand sides exist in memory only on the patch-matrix path
      ok = ok && cv_alloc(h, &h->zbuf, max_out, &st.bytes_scratch) && cv_alloc(h, &h->hsub, max_out, &st.bytes_scratch);
    if (!ok) return fail(MW_ERR_OOM);
  }
  if (h->plan & MW_PLAN_BACKPROP) {
    for (auto& l : h->layers) ok = ok && cv_alloc(h, &l.act, (size_t)l.n_out, &st.bytes_bp_activations);
    if (!(h->plan & MW_PLAN_MOONWALK) && h->h0_full)
      ok = ok && cv_alloc(h, &h->h0, (size_t)h->layers[0].n_in, &st.bytes_input_cotangent);
    if (!(h->plan & MW_PLAN_MOONWALK))
      ok = ok && cv_alloc(h, &h->ha, max_out, &st.bytes_bp_scratch) && cv_alloc(h, &h->hb, max_odd, &st.bytes_bp_scratch) &&
           cv_alloc(h, &h->ctz, max_out, &st.bytes_bp_scratch);
    if (!ok) return fail(MW_ERR_OOM);
  }
  (void)B;
  for (auto& l : h->layers)
    if (l.gather_rev) ok = ok && cv_alloc(h, &l.wrev, (size_t)l.K * l.Cout, &st.bytes_packed_weights);
  if (!ok) return fail(MW_ERR_OOM);
  {
    int rc = build_from_weights(h, stream);
    if (rc != MW_OK) return fail(rc);
  }
  e = hipStreamSynchronize(stream);
  if (e != hipSuccess) return fail(record_hip_failure(e, "setup sync"));
  *out = h;
  return MW_OK;
}

int moonwalk_conv_refresh(mw_conv_handle_t* h, void* hip_stream) {
  if (!h) return MW_ERR_INVALID_ARG;
  return build_from_weights(h, static_cast<hipStream_t>(hip_stream));
}

int moonwalk_conv_grad(mw_conv_handle_t* h, const float* x, const float* target, float* grads_out, float* loss_out,
                       void* hip_stream) {
  if (!h || !x || !target || !grads_out) return MW_ERR_INVALID_ARG;
  if (!(h->plan & MW_PLAN_MOONWALK)) return MW_ERR_NOT_PLANNED;
  if (h->layers[0].gather && (reinterpret_cast<uintptr_t>(x) & 15)) return MW_ERR_INVALID_ARG;
  return run_conv_moonwalk(h, x, target, grads_out, loss_out, false, 0.f, static_cast<hipStream_t>(hip_stream));
}

int moonwalk_conv_sgd_step(mw_conv_handle_t* h, const float* x, const float* target, float lr, float* loss_out,
                           void* hip_stream) {
  if (!h || !x || !target || !std::isfinite(lr)) return MW_ERR_INVALID_ARG;
  if (!(h->plan & MW_PLAN_MOONWALK)) return MW_ERR_NOT_PLANNED;
  // in the patch-buffer path a layer's forward and weight-gradient products alternate chunk by chunk, so its
  // weights cannot change under it: the step needs every layer on the gathered kernels
  for (const auto& l : h->layers)
    if (!l.gather) return MW_ERR_NOT_PLANNED;
  if (reinterpret_cast<uintptr_t>(x) & 15) return MW_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int rc = run_conv_moonwalk(h, x, target, nullptr, loss_out, true, lr, s);
  if (rc != MW_OK) return rc;
  return build_from_weights(h, s);
}

}  // extern "C"

namespace {

int run_conv_moonwalk(mw_conv_handle* h, const float* x, const float* target, float* grads_out, float* loss_out, bool apply,
                      float lr, hipStream_t s) {
  const int L = h->L;
  unsigned long long* mismatches = reinterpret_cast<unsigned long long*>(h->status);
  CV_HIP(ew_fill_u32(h->status, 0u, 2, s));

  // ---------------- Phase I: forward, keep the sign masks only
  const float* xin = x;
  float* xbuf[2] = {h->xa, h->xb};
  for (int i = 0; i < L; ++i) {
    ConvLayer& l = h->layers[i];
    float* xout = xbuf[i & 1];
    int rc = conv_forward_layer(h, l, xin, xout, l.mask, s);
    if (rc != MW_OK) return rc;
    xin = xout;
  }
  // ---------------- loss and output cotangent
  {
    const ConvLayer& last = h->layers[L - 1];
    CV_HIP(ew_loss_grad(xin, target, h->B, (int)(last.n_out / h->B), h->loss_scale, h->ha, loss_out, h->loss_scratch, s, h->status + 3));
  }
  // ---------------- Phase II: reverse, input cotangent only. ct_z of layer i lives in ctbuf[i % 2]; the
  // cotangent h itself is kept only where Phase III starts from it (h_0 and the re-seed points), and
  // there in the form the vijp reads it.
  {
    float* ctbuf[2] = {h->ctz, h->hb};
    const ConvLayer& top = h->layers[L - 1];
    CV_HIP(ew_rev_scale(h->ha, top.mask, top.n_out, top.alpha, ctbuf[(L - 1) & 1], s));
    for (int i = L - 1; i >= 0; --i) {
      ConvLayer& l = h->layers[i];
      const ConvLayer* prev = i > 0 ? &h->layers[i - 1] : nullptr;
      const float* ct = ctbuf[i & 1];
      const bool frag1d = l.kind == MW_CONV_FRAGMENTAL_1D;
      if (frag1d) {
        int rc = frag_store(h, l, ct, s);
        if (rc != MW_OK) return rc;
      }
      const bool whole = l.whole_h();
      float* kept = prev ? prev->ckpt : (h->h0_full ? nullptr : h->h0);
      if (kept && !whole) {
        int rc = conv_kept_cotangent(h, l, ct, kept, s);
        if (rc != MW_OK) return rc;
      }
      if (!prev && !h->h0_full) break;  // nothing else reads h_0
      float* ct_next = prev ? ctbuf[(i - 1) & 1] : nullptr;
      bool fused = false;
      // a layer that cannot scale in its epilogue leaves h in ha (free since the line above the loop)
      const bool can_fuse = l.gather_rev && prev && l.Cin % 32 == 0;
      float* raw = prev ? (can_fuse ? nullptr : h->ha) : h->h0;
      if (whole && kept) raw = kept;  // such a layer reads every position of its input cotangent
      int rc = conv_input_grad(h, l, ct, raw, ct_next, prev, &fused, s);
      if (rc != MW_OK) return rc;
      if (prev && !fused) CV_HIP(ew_rev_scale(raw, prev->mask, prev->n_out, prev->alpha, ct_next, s));
    }
  }
  // ---------------- Phase III: forward vijp sweep
  const float inv_scale = 1.0f / h->loss_scale;
  // Where the layer's gradient goes: into grads_out, or (training step) straight onto the layer's own
  // weights as -lr * gradient, after which the entries the method constrains to zero are put back.
  const float g_scale = apply ? -lr * inv_scale : inv_scale;
  const float g_beta = apply ? 1.f : 0.f;
  float* hbuf[2] = {h->ha, h->hb};
  xin = x;
  const float* hin = h->h0;
  bool hin_as_read = !h->h0_full;  // hin holds [rows][Cout] = what this layer's vijp reads, not a whole activation
  for (int i = 0; i < L; ++i) {
    ConvLayer& l = h->layers[i];
    const bool frag1d = l.kind == MW_CONV_FRAGMENTAL_1D;
    if (i > 0 && h->layers[i - 1].ckpt) {  // re-seed
      hin = h->layers[i - 1].ckpt;
      hin_as_read = !l.whole_h();
    }
    float* xout = xbuf[i & 1];
    float* hout = hbuf[i & 1];
    if (l.gather) {
      // ct_z and the layer's outputs, image chunk by image chunk. Where the vijp couples positions, ct_z comes
      // first (fragmental layers: rebuilt block-wise from the incoming cotangent and the fragments; wide kernels:
      // solved for the (p, p) tap at all positions, then swept over the anti-diagonals of the output grid) and
      // one kernel follows: the pre-activation again, the sign check, the vijp of the activation. In the fully
      // parallel case one kernel does it all: recomputed forward, channel solve at the strided positions, epilogue.
      if (frag1d) {
        int rc = frag_rebuild(h, l, hin, h->ctz, s);
        if (rc != MW_OK) return rc;
      }
      for (int64_t img0 = 0; img0 < h->B; img0 += l.gchunk) {
        const int n_img = (int)((img0 + l.gchunk <= h->B) ? l.gchunk : h->B - img0);
        const int64_t o = img0 * l.out_img();
        const uint32_t* mask32 = reinterpret_cast<const uint32_t*>(l.mask) + o / 32;
        const float* xc = xin + img0 * l.in_img();
        if (l.whole_h()) {
          if (!frag1d) {
            CV_HIP(conv_sub_solve(l.geom(), n_img, l.Cout, hin + img0 * l.in_img(), l.Tinv, h->ctz + o, s));
            CV_HIP(conv_vijp_sweep(l.Ho, l.Wo, l.Cout, n_img, l.reach, h->ctz + o, l.Asweep, s));
          }
          CV_HIP(conv_vijp_given(l.geom(), n_img, xc, l.w, l.b, l.alpha, l.Cout, h->ctz + o, mask32, xout + o, hout + o,
                                 mismatches, s));
        } else {
          CV_HIP(conv_vijp_layer(l.geom(), n_img, xc, l.w, l.b, l.alpha, l.Cout,
                                 hin + img0 * (hin_as_read ? l.out_img() : l.in_img()), hin_as_read ? 1 : 0, l.Tinv, mask32,
                                 xout + o, hout + o, h->ctz + o, mismatches, s));
        }
      }
      int rc = conv_weight_grad(h, l, xin, h->ctz, g_scale, apply ? const_cast<float*>(l.w) : grads_out + l.dW_off,
                                apply ? const_cast<float*>(l.b) : grads_out + l.db_off, s, g_beta);
      if (rc != MW_OK) return rc;
    } else {
      if (apply) return MW_ERR_NOT_PLANNED;
      // vijp of the convolution: right-hand sides at the strided positions, then the channel solve as a product
      const float* rhs = hin;
      if (!hin_as_read) {
        CV_HIP(cv_strided_gather(hin, l.Hin, l.Win, l.Cin, l.Ho, l.Wo, l.Cout, l.s, l.rows, h->hsub, s));
        rhs = h->hsub;
      }
      const int64_t per_img = (int64_t)l.Ho * l.Wo;
      bool first = true;
      for (int64_t img0 = 0; img0 < h->B; img0 += l.chunk_images) {
        const int64_t n_img = (img0 + l.chunk_images <= h->B) ? l.chunk_images : h->B - img0;
        const int64_t r0 = img0 * per_img, R = n_img * per_img;
        CV_HIP(gemm_plain(OP_NT, TILE_AUTO, (int)R, l.Cout, l.Cout, 1.f, rhs + r0 * l.Cout, l.Cout, l.Tinv, l.Cout, 0.f,
                          h->ctz + r0 * l.Cout, l.Cout, nullptr, s));
        int rc = conv_rows(h, l, xin, r0, R, h->zbuf, s);  // recompute z; the patches stay in the buffer
        if (rc != MW_OK) return rc;
        // dW[K][Cout] (+)= patches^T ct_z over the rows of this chunk
        CV_HIP(gemm_plain(OP_TN, TILE_AUTO, l.K, l.Cout, (int)R, inv_scale, h->patches, l.K, h->ctz + r0 * l.Cout, l.Cout,
                          first ? 0.f : 1.f, grads_out + l.dW_off, l.Cout, nullptr, s));
        first = false;
      }
      CV_HIP(ew_colsum_wide(h->ctz, l.rows, l.Cout, inv_scale, 0.f, grads_out + l.db_off, h->colsum_part, s));
      CV_HIP(ew_vijp_epilogue(h->zbuf, h->ctz, l.rows, l.Cout, l.alpha, l.mask, nullptr, nullptr, nullptr, 0, xout, hout,
                              mismatches, s));
    }
    if (apply)  // the projected step: above the diagonal of the triangular tap the weights stay zero
      CV_HIP(cv_zero_above_diagonal(const_cast<float*>(l.tri_tap()), l.Cout, l.Cout, s));
    xin = xout;
    hin = hout;
    hin_as_read = false;
  }
  return MW_OK;
}

}  // namespace

extern "C" {

int backprop_conv_grad(mw_conv_handle_t* h, const float* x, const float* target, float* grads_out, float* loss_out,
                       void* hip_stream) {
  if (!h || !x || !target || !grads_out) return MW_ERR_INVALID_ARG;
  if (!(h->plan & MW_PLAN_BACKPROP)) return MW_ERR_NOT_PLANNED;
  if (h->layers[0].gather && (reinterpret_cast<uintptr_t>(x) & 15)) return MW_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int L = h->L;
  // forward, every activation stored (the sign is read back from it: x > 0 <=> z > 0)
  const float* xin = x;
  for (int i = 0; i < L; ++i) {
    ConvLayer& l = h->layers[i];
    int rc = conv_forward_layer(h, l, xin, l.act, nullptr, s);
    if (rc != MW_OK) return rc;
    xin = l.act;
  }
  {
    const ConvLayer& last = h->layers[L - 1];
    CV_HIP(ew_loss_grad(xin, target, h->B, (int)(last.n_out / h->B), h->loss_scale, h->ha, loss_out, h->loss_scratch, s, h->status + 3));
  }
  const float inv_scale = 1.0f / h->loss_scale;
  float* hbuf[2] = {h->ha, h->hb};
  const float* hcur = h->ha;
  for (int i = L - 1; i >= 0; --i) {
    ConvLayer& l = h->layers[i];
    const float* xprev = (i == 0) ? x : h->layers[i - 1].act;
    CV_HIP(ew_scale_by_act_slope(hcur, l.act, l.n_out, l.alpha, h->ctz, s));
    {
      int rc = conv_weight_grad(h, l, xprev, h->ctz, inv_scale, grads_out + l.dW_off, grads_out + l.db_off, s);
      if (rc != MW_OK) return rc;
    }
    if (i > 0 || h->h0_full) {
      // the cotangent at the output of layer j < L - 1 lives in hbuf[j % 2] (hb is sized for the odd layers
      // only); h_L was in ha and has gone into ct_z by now, so ha may be written even when it held h_L
      float* hout = i > 0 ? hbuf[(i - 1) & 1] : h->h0;
      int rc = conv_input_grad(h, l, h->ctz, hout, nullptr, nullptr, nullptr, s);
      if (rc != MW_OK) return rc;
      hcur = hout;
    }
  }
  return MW_OK;
}

int moonwalk_conv_grad_layout(const mw_conv_handle_t* h, size_t* total_floats, size_t* dW_off, size_t* db_off) {
  if (!h) return MW_ERR_INVALID_ARG;
  if (total_floats) *total_floats = h->total_floats;
  for (int i = 0; i < h->L; ++i) {
    if (dW_off) dW_off[i] = h->layers[i].dW_off;
    if (db_off) db_off[i] = h->layers[i].db_off;
  }
  return MW_OK;
}

int moonwalk_conv_memory_stats(mw_conv_handle_t* h, mw_conv_memstats_t* out) {
  if (!h || !out) return MW_ERR_INVALID_ARG;
  CV_HIP(hipDeviceSynchronize());
  *out = h->st;
  out->bytes_live = h->live;
  out->bytes_peak = h->peak;
  uint32_t status[4] = {0, 0, 0, 0};
  CV_HIP(hipMemcpy(status, h->status, sizeof(status), hipMemcpyDeviceToHost));
  const unsigned long long mm = (unsigned long long)status[0] | ((unsigned long long)status[1] << 32);
  out->sign_mismatches = mm;
  out->nonfinite_loss = status[3] ? 1 : 0;
  if (out->nonfinite_loss) return MW_ERR_NONFINITE;
  return mm ? MW_ERR_SIGN_MISMATCH : MW_OK;
}

int moonwalk_conv_fetch(mw_conv_handle_t* h, int32_t layer, int32_t what, void* host_dst, size_t cap, size_t* n_bytes) {
  if (!h) return MW_ERR_INVALID_ARG;
  if (what != MW_FETCH_H0 && (layer < 0 || layer >= h->L)) return MW_ERR_INVALID_ARG;
  CV_HIP(hipDeviceSynchronize());
  const void* src = nullptr;
  size_t bytes = 0;
  switch (what) {
    case MW_FETCH_MASK: src = h->layers[layer].mask; bytes = h->layers[layer].mask_words * 8; break;
    case MW_FETCH_H0:
      src = h->h0;
      bytes = (h->h0_full ? (size_t)h->layers[0].n_in : (size_t)h->layers[0].rows * h->layers[0].Cout) * 4;
      break;
    case MW_FETCH_P: src = h->layers[layer].Tinv; bytes = (size_t)h->layers[layer].Cout * h->layers[layer].Cout * 4; break;
    case MW_FETCH_CHECKPOINT:
      if (layer + 1 >= h->L) return MW_ERR_INVALID_ARG;
      src = h->layers[layer].ckpt;
      bytes = (h->layers[layer + 1].whole_h() ? (size_t)h->layers[layer + 1].n_in
                                                                  : (size_t)h->layers[layer + 1].rows * h->layers[layer + 1].Cout) * 4;
      break;
    case MW_FETCH_FRAG:
      src = h->layers[layer].frag;
      bytes = h->layers[layer].frag ? (size_t)(h->layers[layer].rows / h->layers[layer].block) * (h->layers[layer].k - 1) *
                                          h->layers[layer].Cout * 4
                                    : 0;
      break;
    default: return MW_ERR_INVALID_ARG;
  }
  if (!src) return MW_ERR_INVALID_ARG;
  if (n_bytes) *n_bytes = bytes;
  if (!host_dst && cap == 0) return MW_OK;
  if (!host_dst || cap < bytes) return MW_ERR_INVALID_ARG;
  if (bytes) CV_HIP(hipMemcpy(host_dst, src, bytes, hipMemcpyDeviceToHost));
  return MW_OK;
}

void moonwalk_conv_destroy(mw_conv_handle_t* h) {
  if (!h) return;
  (void)hipDeviceSynchronize();
  h->release_all();
  delete h;
}

// ---- kernel-level entries (unit parity tests)
int mw_conv_im2col(const float* x, int32_t H, int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad, int64_t row0,
                   int64_t n_rows, float* patches, void* hip_stream) {
  if (!x || !patches || H <= 0 || W <= 0 || C <= 0 || k <= 0 || stride <= 0 || pad < 0 || row0 < 0 || n_rows < 0)
    return MW_ERR_INVALID_ARG;
  if (H + 2 * pad < k || W + 2 * pad < k) return MW_ERR_INVALID_ARG;
  const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
  CV_HIP(cv_im2col(x, H, W, C, Ho, Wo, k, stride, pad, row0, n_rows, patches, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

namespace {

// geometry of a kernel-level call, or false if the gathered kernels cannot take it
bool shape_geom(const mw_conv_shape_t* sh, ConvGeom* g) {
  if (!sh || sh->batch <= 0 || sh->height <= 0 || sh->width <= 0 || sh->channels_in <= 0 || sh->channels_out <= 0) return false;
  if (sh->kh <= 0 || sh->kw <= 0 || sh->stride <= 0 || sh->pad_h < 0 || sh->pad_w < 0) return false;
  if (sh->height + 2 * sh->pad_h < sh->kh || sh->width + 2 * sh->pad_w < sh->kw) return false;
  if (sh->channels_in % 32 || sh->channels_out % 32) return false;
  const int Ho = (sh->height + 2 * sh->pad_h - sh->kh) / sh->stride + 1, Wo = (sh->width + 2 * sh->pad_w - sh->kw) / sh->stride + 1;
  *g = ConvGeom{sh->height, sh->width, sh->channels_in, Ho, Wo, sh->kh, sh->kw, sh->stride, sh->pad_h, sh->pad_w};
  if ((int64_t)g->taps() * g->C >= (1 << 24)) return false;
  return conv_gather_max_images(*g, sh->channels_out) >= sh->batch;  // one launch: everything below 2 GiB
}
bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

int mw_conv_forward(const mw_conv_shape_t* shape, const float* x, const float* w, const float* b, float alpha, float* xout,
                    uint64_t* mask, void* hip_stream) {
  ConvGeom g;
  if (!shape_geom(shape, &g) || !x || !w || !xout || !al16(x) || !al16(w) || !(alpha > 0.f)) return MW_ERR_INVALID_ARG;
  CV_HIP(conv_fwd_act(g, shape->batch, x, w, b, alpha, shape->channels_out, xout, reinterpret_cast<uint32_t*>(mask),
                      static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

int mw_conv_input_cotangent(const mw_conv_shape_t* shape, const float* ctz, const float* w, float* h, float* work,
                            void* hip_stream) {
  ConvGeom g;
  if (!shape_geom(shape, &g) || !ctz || !w || !h || !work || !al16(ctz) || !al16(work)) return MW_ERR_INVALID_ARG;
  if (!conv_rev_ok(g, shape->channels_out)) return MW_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CV_HIP(cv_pack_rev_weights(w, g.kh, g.kw, g.s, g.C, shape->channels_out, work, s));
  CV_HIP(conv_input_cotangent(g, shape->batch, shape->channels_out, ctz, work, h, nullptr, nullptr, 1.f, s));
  return MW_OK;
}

size_t mw_conv_weight_grad_work_floats(const mw_conv_shape_t* shape) {
  ConvGeom g;
  if (!shape_geom(shape, &g)) return 0;
  return conv_dw_part_floats(g, shape->batch, shape->channels_out) + (size_t)COLSUM_MAX_SLICES * shape->channels_out;
}

int mw_conv_weight_grad(const mw_conv_shape_t* shape, const float* x, const float* ctz, float scale, float* dw, float* db,
                        float* work, void* hip_stream) {
  ConvGeom g;
  if (!shape_geom(shape, &g) || !x || !ctz || !dw || !db || !work || !al16(x) || !al16(ctz) || !al16(work) || !al16(dw))
    return MW_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const size_t part = conv_dw_part_floats(g, shape->batch, shape->channels_out);
  CV_HIP(conv_dw(g, shape->batch, x, ctz, shape->channels_out, scale, 0.f, dw, work, s));
  CV_HIP(ew_colsum_wide(ctz, (int64_t)shape->batch * g.Ho * g.Wo, shape->channels_out, scale, 0.f, db, work + part, s));
  return MW_OK;
}

int mw_conv_col2im(const float* dpatches, int32_t H, int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad,
                   int64_t img0, int64_t n_img, float* h, void* hip_stream) {
  if (!dpatches || !h || H <= 0 || W <= 0 || C <= 0 || k <= 0 || stride <= 0 || pad < 0 || img0 < 0 || n_img < 0)
    return MW_ERR_INVALID_ARG;
  if (H + 2 * pad < k || W + 2 * pad < k) return MW_ERR_INVALID_ARG;
  const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
  CV_HIP(cv_col2im(dpatches, H, W, C, Ho, Wo, k, stride, pad, img0, n_img, h, static_cast<hipStream_t>(hip_stream)));
  return MW_OK;
}

}  // extern "C"
