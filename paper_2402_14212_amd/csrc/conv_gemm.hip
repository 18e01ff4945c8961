// Launchers of the gathered-operand convolution kernels (conv_gemm.h).
#include <type_traits>

#include "conv_gemm.h"
#include "mw_internal.h"

namespace mw {

namespace {

AConvPatch make_gather(const ConvGeom& g, int n_img, int k, int s, int p, int c0, int csel) {
  AConvPatch a;
  a.H = g.H; a.W = g.W; a.C = g.C; a.Ho = g.Ho; a.Wo = g.Wo;
  a.k = k; a.s = s; a.p = p; a.c0 = c0; a.Csel = csel;
  a.row_off = 0;
  a.bytes = (uint32_t)((int64_t)n_img * g.H * g.W * g.C * 4);
  a.d_howo = FastDiv((uint32_t)(g.Ho * g.Wo));
  a.d_wo = FastDiv((uint32_t)g.Wo);
  a.d_csel = FastDiv((uint32_t)csel);
  a.d_k = FastDiv((uint32_t)k);
  return a;
}

template <class Cfg, bool MASK>
hipError_t fwd_t(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                 float* xout, uint32_t* mask32, hipStream_t stream) {
  const int M = n_img * g.Ho * g.Wo, K1 = g.k * g.k * g.C;
  const AConvPatch xf = make_gather(g, n_img, g.k, g.s, g.p, 0, g.C);
  EpiFwdAct<MASK> epi{xout, b, alpha, mask32};
  auto t = make_gemm_task<Cfg, KCONTIG, RCONTIG, true, AConvPatch, EpiFwdAct<MASK>, false>(M, Cout, K1, x, 0, w, Cout, xf, epi,
                                                                                         nullptr, 0.f);
  return launch_task<Cfg::NT>(t, stream);
}

template <class Cfg>
hipError_t fwd_m(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                 float* xout, uint32_t* mask32, hipStream_t stream) {
  if (mask32) return fwd_t<Cfg, true>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
  return fwd_t<Cfg, false>(g, n_img, x, w, b, alpha, Cout, xout, nullptr, stream);
}

template <class Cfg>
hipError_t vijp_t(const ConvGeom& g, int n_img, const float* x, const float* w, int Cout, const float* hin,
                  const float* Tinv, const EpiVijp<false>& epi, hipStream_t stream) {
  const int M = n_img * g.Ho * g.Wo, K1 = g.k * g.k * g.C;
  ConvVijpTask<Cfg> t{M, Cout, K1, x, w, hin, Tinv,
                      make_gather(g, n_img, g.k, g.s, g.p, 0, g.C),   // patches of x
                      make_gather(g, n_img, 1, g.s, 0, 0, Cout),      // h_in at (s i', s j'), first Cout channels
                      epi, ceil_div(M, Cfg::BM), ceil_div(Cout, Cfg::BN)};
  return launch_task<Cfg::NT>(t, stream);
}

struct DwPlan {
  int tile, slices, k_per;
};

DwPlan plan_dw(int K1, int Cout, int64_t rows) {
  DwPlan p;
  int bm, bn;
  if (K1 >= 128 && Cout >= 128) { p.tile = TILE_128W8; bm = 128; bn = 128; }
  else if (Cout >= 128) { p.tile = TILE_64X128; bm = 64; bn = 128; }
  else { p.tile = TILE_64; bm = 64; bn = 64; }
  const int64_t tiles = (int64_t)ceil_div(K1, bm) * ceil_div(Cout, bn);
  // about four workgroups per CU when the rows allow it, at least eight K tiles per slice
  int64_t want = (1024 + tiles - 1) / tiles;
  if (want > CONV_DW_MAX_SLICES) want = CONV_DW_MAX_SLICES;
  int64_t k_per = (rows + want - 1) / want;
  if (k_per < 256) k_per = 256;
  k_per = (k_per + 31) / 32 * 32;
  p.k_per = (int)k_per;
  p.slices = (int)((rows + k_per - 1) / k_per);
  if (p.slices < 1) p.slices = 1;
  return p;
}

template <class Cfg>
hipError_t dw_t(const ConvGeom& g, int n_img, const float* x, const float* ctz, int Cout, const DwPlan& p, float* part,
                hipStream_t stream) {
  const int rows = n_img * g.Ho * g.Wo, K1 = g.k * g.k * g.C;
  SplitKTnTask<Cfg, AConvPatch> t{K1, Cout, rows, x, 0, ctz, Cout, make_gather(g, n_img, g.k, g.s, g.p, 0, g.C), part,
                                  p.slices, p.k_per, ceil_div(K1, Cfg::BM), ceil_div(Cout, Cfg::BN)};
  return launch_task<Cfg::NT>(t, stream);
}

}  // namespace

bool conv_gather_ok(const ConvGeom& g, int Cout, const float* x, const float* w) {
  return g.C % 4 == 0 && Cout % 32 == 0 && aligned16(x) && aligned16(w) && (int64_t)g.k * g.k * g.C < (1 << 24);
}

int64_t conv_gather_max_images(const ConvGeom& g, int Cout) {
  // every operand of a launch (image chunk, its output rows) must stay below 2 GiB
  const int64_t limit = 0x7FFFFFFF;
  const int64_t in_img = (int64_t)g.H * g.W * g.C * 4, out_img = (int64_t)g.Ho * g.Wo * (Cout > g.C ? Cout : g.C) * 4;
  const int64_t per = in_img > out_img ? in_img : out_img;
  return per >= limit ? 0 : (limit - 1) / per;
}

hipError_t conv_fwd_act(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                        float* xout, uint32_t* mask32, hipStream_t stream) {
  if (n_img <= 0) return hipSuccess;
  const int M = n_img * g.Ho * g.Wo, K1 = g.k * g.k * g.C;
  switch (pick_tile(M, Cout, K1)) {
    case TILE_128W8: return fwd_m<Tile128W8>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
    case TILE_64X128: return fwd_m<Tile64x128>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
    case TILE_64K2: return fwd_m<Tile64K2>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
    case TILE_32K4: return fwd_m<Tile32K4>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
    default: return fwd_m<Tile64>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
  }
}

hipError_t conv_vijp_layer(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                           const float* hin, const float* Tinv, const uint32_t* mask32, float* xout, float* hout, float* ctz,
                           unsigned long long* mismatches, hipStream_t stream) {
  if (n_img <= 0) return hipSuccess;
  const int M = n_img * g.Ho * g.Wo, K1 = g.k * g.k * g.C;
  // the leaky path of the epilogue reads the mask as 32-bit words, so a 4-byte aligned start is enough
  EpiVijp<false> epi{b, alpha, 1.0f / alpha, reinterpret_cast<const uint64_t*>(mask32), nullptr, nullptr, nullptr, 0,
                     xout, hout, ctz, mismatches};
  switch (pick_tile(M, Cout, K1)) {  // the tile of conv_fwd_act: the recomputed signs must match bit for bit
    case TILE_128W8: return vijp_t<Tile128W8>(g, n_img, x, w, Cout, hin, Tinv, epi, stream);
    case TILE_64X128: return vijp_t<Tile64x128>(g, n_img, x, w, Cout, hin, Tinv, epi, stream);
    case TILE_64K2: return vijp_t<Tile64K2>(g, n_img, x, w, Cout, hin, Tinv, epi, stream);
    case TILE_32K4: return vijp_t<Tile32K4>(g, n_img, x, w, Cout, hin, Tinv, epi, stream);
    default: return vijp_t<Tile64>(g, n_img, x, w, Cout, hin, Tinv, epi, stream);
  }
}

size_t conv_dw_part_floats(const ConvGeom& g, int n_img, int Cout) {
  // the most slices any chunk of at most n_img images is split into
  const int K1 = g.k * g.k * g.C;
  int most = 1;
  for (int n = 1; n <= n_img; ++n) {
    const int sl = plan_dw(K1, Cout, (int64_t)n * g.Ho * g.Wo).slices;
    if (sl > most) most = sl;
  }
  return (size_t)most * K1 * Cout;
}

hipError_t conv_dw(const ConvGeom& g, int n_img, const float* x, const float* ctz, int Cout, float scale, float beta,
                   float* dW, float* part, hipStream_t stream) {
  if (n_img <= 0) return hipSuccess;
  const int K1 = g.k * g.k * g.C;
  const DwPlan p = plan_dw(K1, Cout, (int64_t)n_img * g.Ho * g.Wo);
  hipError_t e;
  switch (p.tile) {
    case TILE_128W8: e = dw_t<Tile128W8>(g, n_img, x, ctz, Cout, p, part, stream); break;
    case TILE_64X128: e = dw_t<Tile64x128>(g, n_img, x, ctz, Cout, p, part, stream); break;
    default: e = dw_t<Tile64>(g, n_img, x, ctz, Cout, p, part, stream); break;
  }
  if (e != hipSuccess) return e;
  return ew_reduce_slices(part, p.slices, (int64_t)K1 * Cout, scale, beta, dW, stream);
}

}  // namespace mw
