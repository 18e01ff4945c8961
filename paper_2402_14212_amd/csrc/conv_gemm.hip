// Launchers of the gathered-operand convolution kernels (conv_gemm.h).
#include <type_traits>

#include "conv_gemm.h"
#include "mw_internal.h"

namespace mw {

namespace {

AConvPatch make_gather(const ConvGeom& g, int n_img, int kh, int kw, int s, int ph, int pw, int c0, int csel) {
  AConvPatch a;
  a.H = g.H; a.W = g.W; a.C = g.C; a.Ho = g.Ho; a.Wo = g.Wo;
  a.kh = kh; a.kw = kw; a.s = s; a.py = ph; a.px = pw; a.c0 = c0; a.Csel = csel;
  a.row_off = 0;
  a.xdiag = 0;
  a.bytes = (uint32_t)((int64_t)n_img * g.H * g.W * g.C * 4);
  a.d_howo = FastDiv((uint32_t)(g.Ho * g.Wo));
  a.d_wo = FastDiv((uint32_t)g.Wo);
  a.d_csel = FastDiv((uint32_t)csel);
  a.d_kw = FastDiv((uint32_t)kw);
  a.d1 = (uint32_t)(g.W - g.Wo) * (uint32_t)(s * g.C);
  a.d2 = (uint32_t)(g.H - g.Ho * s) * (uint32_t)(g.W * g.C);
  return a;
}

// taps ky < k with ky mod s == r
int class_taps(int k, int s, int r) { return r < k ? (k - r + s - 1) / s : 0; }

template <class Cfg>
hipError_t rev_t(const ConvGeom& g, int n_img, int Cout, const float* ctz, const float* wrev, const EpiConvRev& epi,
                 hipStream_t stream) {
  ConvRevTask<Cfg> t;
  t.N = g.C;
  t.CT = ctz;
  t.Wrev = wrev;
  t.epi = epi;
  t.tiles_n = ceil_div(g.C, Cfg::BN);
  int n = 0, first = 0;
  int64_t w_off = 0;
  for (int ry = 0; ry < g.s; ++ry)
    for (int rx = 0; rx < g.s; ++rx) {
      const int nty = class_taps(g.kh, g.s, ry), ntx = class_taps(g.kw, g.s, rx);
      // pixels iy with (iy + p) mod s == ry: iy + p = s q + ry for q in [q_lo, q_hi]
      auto lo = [&](int p, int r) { return (p - r + g.s - 1) / g.s; };        // ceil((p - r) / s), p >= 0 > r - s
      auto hi = [&](int extent, int p, int r) { return (extent + p - 1 - r) >= 0 ? (extent + p - 1 - r) / g.s : -1; };
      const int qy_lo = lo(g.ph, ry), qx_lo = lo(g.pw, rx);
      const int nqy = hi(g.H, g.ph, ry) - qy_lo + 1, nqx = hi(g.W, g.pw, rx) - qx_lo + 1;
      const int64_t w_here = w_off;
      w_off += (int64_t)nty * ntx * Cout * g.C;
      if (nqy <= 0 || nqx <= 0) continue;
      RevClass& rc = t.cls[n++];
      AConvPatch& a = rc.g;
      a.H = g.Ho; a.W = g.Wo; a.C = Cout; a.Ho = nqy; a.Wo = nqx;
      a.kh = nty; a.kw = ntx; a.s = 1;
      // tap slot ky' holds ky = ry + s (nty - 1 - ky'): its source row is q - (nty - 1 - ky')
      a.py = nty - 1 - qy_lo; a.px = ntx - 1 - qx_lo;
      a.c0 = 0; a.Csel = Cout; a.row_off = 0; a.xdiag = 0;
      a.bytes = (uint32_t)((int64_t)n_img * g.Ho * g.Wo * Cout * 4);
      a.d_howo = FastDiv((uint32_t)(nqy * nqx));
      a.d_wo = FastDiv((uint32_t)nqx);
      a.d_csel = FastDiv((uint32_t)Cout);
      a.d_kw = FastDiv((uint32_t)(ntx > 0 ? ntx : 1));
      a.d1 = 0; a.d2 = 0;  // rows never run along K in this product
      rc.oy = g.s * qy_lo + ry - g.ph;
      rc.ox = g.s * qx_lo + rx - g.pw;
      rc.K = nty * ntx * Cout;
      rc.M = n_img * nqy * nqx;
      rc.tiles_m = ceil_div(rc.M, Cfg::BM);
      rc.first = first;
      rc.w_off = w_here;
      first += (rc.tiles_m * t.tiles_n + 7) / 8 * 8;
    }
  t.n_cls = n;
  t.total_blocks = first;
  if (n == 0) return hipSuccess;
  return launch_task<Cfg::NT>(t, stream);
}

template <class Cfg, bool MASK>
hipError_t fwd_t(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                 float* xout, uint32_t* mask32, hipStream_t stream) {
  const int M = n_img * g.Ho * g.Wo, K1 = g.taps() * g.C;
  const AConvPatch xf = make_gather(g, n_img, g.kh, g.kw, g.s, g.ph, g.pw, 0, g.C);
  EpiFwdAct<MASK> epi{xout, b, alpha, mask32};
  auto t = make_gemm_task<Cfg, KCONTIG, RCONTIG, true, AConvPatch, EpiFwdAct<MASK>, false>(M, Cout, K1, x, 0, w, Cout, xf, epi,
                                                                                         nullptr, 0.f);
  return launch_task<Cfg::NT>(t, stream);
}

template <class Cfg>
hipError_t fwd_given_t(const ConvGeom& g, int n_img, const float* x, const float* w, int Cout, const EpiVijpGiven& epi,
                       hipStream_t stream) {
  const int M = n_img * g.Ho * g.Wo, K1 = g.taps() * g.C;
  const AConvPatch xf = make_gather(g, n_img, g.kh, g.kw, g.s, g.ph, g.pw, 0, g.C);
  auto t = make_gemm_task<Cfg, KCONTIG, RCONTIG, true, AConvPatch, EpiVijpGiven, false>(M, Cout, K1, x, 0, w, Cout, xf, epi, nullptr,
                                                                                      0.f);
  return launch_task<Cfg::NT>(t, stream);
}

template <class Cfg>
hipError_t fwd_m(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                 float* xout, uint32_t* mask32, hipStream_t stream) {
  if (mask32) return fwd_t<Cfg, true>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
  return fwd_t<Cfg, false>(g, n_img, x, w, b, alpha, Cout, xout, nullptr, stream);
}

template <class Cfg>
hipError_t vijp_t(const ConvGeom& g, int n_img, const float* x, const float* w, int Cout, const float* hin, int hin_as_read,
                  const float* Tinv, const EpiVijp<false>& epi, hipStream_t stream) {
  const int M = n_img * g.Ho * g.Wo, K1 = g.taps() * g.C;
  // the right-hand sides: h_in at (s i', s j'), first Cout channels, or already laid out that way
  const ConvGeom rows_only{g.Ho, g.Wo, Cout, g.Ho, g.Wo, 1, 1, 1, 0, 0};
  const AConvPatch gh =
      hin_as_read ? make_gather(rows_only, n_img, 1, 1, 1, 0, 0, 0, Cout) : make_gather(g, n_img, 1, 1, g.s, 0, 0, 0, Cout);
  ConvVijpTask<Cfg> t{M, Cout, K1, x, w, hin, Tinv,
                      make_gather(g, n_img, g.kh, g.kw, g.s, g.ph, g.pw, 0, g.C),   // patches of x
                      gh,
                      epi, ceil_div(M, Cfg::BM), ceil_div(Cout, Cfg::BN)};
  // two workgroups per CU wherever the LDS allows it: the epilogue (three stores and a mask word per
  // element) is long, and a second workgroup's products fill it
  constexpr int RESIDENT = (2 * ConvVijpTask<Cfg>::LDS_BYTES <= 160 * 1024 && Cfg::NT == 512) ? 2 : 1;
  return launch_task_resident<Cfg::NT, RESIDENT>(t, stream);
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
  // four workgroups per CU when the rows allow it, never a few more than that (they would run on
  // their own after all the others), and at least eight K tiles per slice
  int64_t want = tiles >= 1024 ? 1 : 1024 / tiles;
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
  const int rows = n_img * g.Ho * g.Wo, K1 = g.taps() * g.C;
  SplitKTnTask<Cfg, AConvPatch> t{K1, Cout, rows, x, 0, ctz, Cout, make_gather(g, n_img, g.kh, g.kw, g.s, g.ph, g.pw, 0, g.C), part,
                                  p.slices, p.k_per, ceil_div(K1, Cfg::BM), ceil_div(Cout, Cfg::BN)};
  return launch_task<Cfg::NT>(t, stream);
}

// The tile for a product whose K runs over (tap, channel) with csel channels per tap: what pick_tile
// says, unless that tile's K step would straddle taps; then the 64 x 64 tile, whose K step is 32.
int gather_tile(int M, int N, int K, int csel_a, int csel_b) {
  const int t = pick_tile(M, N, K);
  const int bk = t == TILE_64K2 ? 64 : (t == TILE_32K4 ? 128 : 32);
  return (csel_a % bk == 0 && csel_b % bk == 0) ? t : TILE_64;
}

}  // namespace

bool conv_gather_ok(const ConvGeom& g, int Cout, const float* x, const float* w) {
  return g.C % 32 == 0 && Cout % 32 == 0 && aligned16(x) && aligned16(w) && (int64_t)g.taps() * g.C < (1 << 24);
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
  const int M = n_img * g.Ho * g.Wo, K1 = g.taps() * g.C;
  switch (gather_tile(M, Cout, K1, g.C, Cout)) {
    case TILE_128W8: return fwd_m<Tile128W8>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
    case TILE_64X128: return fwd_m<Tile64x128>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
    case TILE_64K2: return fwd_m<Tile64K2>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
    case TILE_32K4: return fwd_m<Tile32K4>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
    default: return fwd_m<Tile64>(g, n_img, x, w, b, alpha, Cout, xout, mask32, stream);
  }
}

hipError_t conv_vijp_given(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                           const float* ctz, const uint32_t* mask32, float* xout, float* hout, unsigned long long* mismatches,
                           hipStream_t stream) {
  if (n_img <= 0) return hipSuccess;
  const int M = n_img * g.Ho * g.Wo, K1 = g.taps() * g.C;
  EpiVijpGiven epi{EpiVijp<false>{b, alpha, 1.0f / alpha, reinterpret_cast<const uint64_t*>(mask32), nullptr, nullptr, nullptr, 0,
                                  xout, hout, nullptr, mismatches},
                   ctz};
  switch (gather_tile(M, Cout, K1, g.C, Cout)) {  // the tile of conv_fwd_act: the recomputed signs must match bit for bit
    case TILE_128W8: return fwd_given_t<Tile128W8>(g, n_img, x, w, Cout, epi, stream);
    case TILE_64X128: return fwd_given_t<Tile64x128>(g, n_img, x, w, Cout, epi, stream);
    case TILE_64K2: return fwd_given_t<Tile64K2>(g, n_img, x, w, Cout, epi, stream);
    case TILE_32K4: return fwd_given_t<Tile32K4>(g, n_img, x, w, Cout, epi, stream);
    default: return fwd_given_t<Tile64>(g, n_img, x, w, Cout, epi, stream);
  }
}

hipError_t conv_vijp_layer(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                           const float* hin, int hin_as_read, const float* Tinv, const uint32_t* mask32, float* xout, float* hout, float* ctz,
                           unsigned long long* mismatches, hipStream_t stream) {
  if (n_img <= 0) return hipSuccess;
  const int M = n_img * g.Ho * g.Wo, K1 = g.taps() * g.C;
  // the leaky path of the epilogue reads the mask as 32-bit words, so a 4-byte aligned start is enough
  EpiVijp<false> epi{b, alpha, 1.0f / alpha, reinterpret_cast<const uint64_t*>(mask32), nullptr, nullptr, nullptr, 0,
                     xout, hout, ctz, mismatches};
  switch (gather_tile(M, Cout, K1, g.C, Cout)) {  // the tile of conv_fwd_act: the recomputed signs must match bit for bit
    case TILE_128W8: return vijp_t<Tile128W8>(g, n_img, x, w, Cout, hin, hin_as_read, Tinv, epi, stream);
    case TILE_64X128: return vijp_t<Tile64x128>(g, n_img, x, w, Cout, hin, hin_as_read, Tinv, epi, stream);
    case TILE_64K2: return vijp_t<Tile64K2>(g, n_img, x, w, Cout, hin, hin_as_read, Tinv, epi, stream);
    case TILE_32K4: return vijp_t<Tile32K4>(g, n_img, x, w, Cout, hin, hin_as_read, Tinv, epi, stream);
    default: return vijp_t<Tile64>(g, n_img, x, w, Cout, hin, hin_as_read, Tinv, epi, stream);
  }
}

// ct = sub(h) Tinv^T for all positions at once: the right-hand sides of the vijp, solved for the (p, p) tap alone
template <class Cfg>
hipError_t sub_solve_t(const ConvGeom& g, int n_img, int Cout, const float* hin, const float* Tinv, float* ct, hipStream_t stream) {
  const int M = n_img * g.Ho * g.Wo;
  const AConvPatch gh = make_gather(g, n_img, 1, 1, g.s, 0, 0, 0, Cout);
  EpiStore epi{ct, Cout, 1.f, 0.f, nullptr};
  auto t = make_gemm_task<Cfg, KCONTIG, KCONTIG, true, AConvPatch, EpiStore, false>(M, Cout, Cout, hin, 0, Tinv, Cout, gh, epi, nullptr,
                                                                                  0.f);
  return launch_task<Cfg::NT>(t, stream);
}

hipError_t conv_sub_solve(const ConvGeom& g, int n_img, int Cout, const float* hin, const float* Tinv, float* ct, hipStream_t stream) {
  if (n_img <= 0) return hipSuccess;
  const int M = n_img * g.Ho * g.Wo;
  switch (gather_tile(M, Cout, Cout, Cout, Cout)) {
    case TILE_128W8: return sub_solve_t<Tile128W8>(g, n_img, Cout, hin, Tinv, ct, stream);
    case TILE_64X128: return sub_solve_t<Tile64x128>(g, n_img, Cout, hin, Tinv, ct, stream);
    case TILE_64K2: return sub_solve_t<Tile64K2>(g, n_img, Cout, hin, Tinv, ct, stream);
    case TILE_32K4: return sub_solve_t<Tile32K4>(g, n_img, Cout, hin, Tinv, ct, stream);
    default: return sub_solve_t<Tile64>(g, n_img, Cout, hin, Tinv, ct, stream);
  }
}

// One anti-diagonal d of the general vijp (see EpiDiagAccum). ct: the h' image chunk [n_img][Ho][Wo][Cout], G on the
// diagonals not yet swept; Asweep: [Cout][K] with K = ((reach + 1)^2 - 1) Cout, tap slots in the gather's order.
template <class Cfg>
hipError_t sweep_t(int Ho, int Wo, int Cout, int n_img, int d, int reach, float* ct, const float* Asweep, hipStream_t stream) {
  const int i0 = d - (Wo - 1) > 0 ? d - (Wo - 1) : 0;
  const int i1 = d < Ho - 1 ? d : Ho - 1;
  const int n_d = i1 - i0 + 1;
  if (n_d <= 0) return hipSuccess;
  const int taps = (reach + 1) * (reach + 1);
  const int K = (taps - 1) * Cout, M = n_img * n_d;
  AConvPatch a;
  a.H = Ho; a.W = Wo; a.C = Cout; a.Ho = n_d; a.Wo = 1;
  a.kh = reach + 1; a.kw = reach + 1; a.s = 1;
  // slot (ky, kx) reads (i' - reach + ky, j' - reach + kx); the last slot is the position itself and is left out of K
  a.py = reach - i0; a.px = reach + i0 - d; a.xdiag = 1;
  a.c0 = 0; a.Csel = Cout; a.row_off = 0;
  a.bytes = (uint32_t)((int64_t)n_img * Ho * Wo * Cout * 4);
  a.d1 = 0; a.d2 = 0;
  a.d_howo = FastDiv((uint32_t)n_d);
  a.d_wo = FastDiv(1u);
  a.d_csel = FastDiv((uint32_t)Cout);
  a.d_kw = FastDiv((uint32_t)(reach + 1));
  EpiDiagAccum epi{ct, n_d, Ho * Wo, i0 * Wo + d - i0, Wo - 1, a.bytes, FastDiv((uint32_t)n_d)};
  auto t = make_gemm_task<Cfg, KCONTIG, KCONTIG, true, AConvPatch, EpiDiagAccum, false>(M, Cout, K, ct, 0, Asweep, K, a, epi, nullptr,
                                                                                      0.f);
  return launch_task<Cfg::NT>(t, stream);
}

hipError_t conv_vijp_sweep(int Ho, int Wo, int Cout, int n_img, int reach, float* ct, const float* Asweep, hipStream_t stream) {
  if (n_img <= 0 || reach <= 0) return hipSuccess;
  const int K = ((reach + 1) * (reach + 1) - 1) * Cout;
  for (int d = 1; d <= Ho + Wo - 2; ++d) {  // diagonal 0 has no earlier position
    const int i0 = d - (Wo - 1) > 0 ? d - (Wo - 1) : 0, i1 = d < Ho - 1 ? d : Ho - 1;
    const int M = n_img * (i1 - i0 + 1);
    hipError_t e;
    switch (gather_tile(M, Cout, K, Cout, Cout)) {
      case TILE_128W8: e = sweep_t<Tile128W8>(Ho, Wo, Cout, n_img, d, reach, ct, Asweep, stream); break;
      case TILE_64X128: e = sweep_t<Tile64x128>(Ho, Wo, Cout, n_img, d, reach, ct, Asweep, stream); break;
      case TILE_64K2: e = sweep_t<Tile64K2>(Ho, Wo, Cout, n_img, d, reach, ct, Asweep, stream); break;
      case TILE_32K4: e = sweep_t<Tile32K4>(Ho, Wo, Cout, n_img, d, reach, ct, Asweep, stream); break;
      default: e = sweep_t<Tile64>(Ho, Wo, Cout, n_img, d, reach, ct, Asweep, stream); break;
    }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

bool conv_rev_ok(const ConvGeom& g, int Cout) {
  return g.s * g.s <= CONV_REV_MAX_CLASSES && Cout % 32 == 0 && g.C % 4 == 0;
}

hipError_t conv_input_cotangent(const ConvGeom& g, int n_img, int Cout, const float* ctz, const float* wrev, float* raw,
                                float* ct, const uint32_t* mask32, float alpha, hipStream_t stream) {
  if (n_img <= 0) return hipSuccess;
  EpiConvRev epi{raw, ct, mask32, alpha, g.H, g.W, g.s, (uint32_t)((int64_t)n_img * g.H * g.W * g.C * 4)};
  // the tile for the largest class: about a quarter of the input pixels, all taps of that class
  const int M = n_img * ((g.H + g.s - 1) / g.s) * ((g.W + g.s - 1) / g.s);
  const int K = class_taps(g.kh, g.s, 0) * class_taps(g.kw, g.s, 0) * Cout;
  switch (gather_tile(M, g.C, K, Cout, Cout)) {
    case TILE_128W8: return rev_t<Tile128W8>(g, n_img, Cout, ctz, wrev, epi, stream);
    case TILE_64X128: return rev_t<Tile64x128>(g, n_img, Cout, ctz, wrev, epi, stream);
    case TILE_64K2: return rev_t<Tile64K2>(g, n_img, Cout, ctz, wrev, epi, stream);
    case TILE_32K4: return rev_t<Tile32K4>(g, n_img, Cout, ctz, wrev, epi, stream);
    default: return rev_t<Tile64>(g, n_img, Cout, ctz, wrev, epi, stream);
  }
}

size_t conv_dw_part_floats(const ConvGeom& g, int n_img, int Cout) {
  // the most slices any chunk of at most n_img images is split into
  const int K1 = g.taps() * g.C;
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
  const int K1 = g.taps() * g.C;
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
