// Phase-III layer kernel: recompute z = x W^T + b and ct_z = h P^T for the same output tile and
// finish the layer (activation, cotangent of the layer output, fragment restore) in registers.
#include "gemm_dispatch.h"

namespace mw {

template <bool RELU>
static hipError_t vijp_dual_t(int tile, int M, int N, int K, const VijpArgs& a, hipStream_t stream) {
  EpiVijp<RELU> epi{a.bias, a.alpha, a.alpha > 0.f ? 1.0f / a.alpha : 0.f, a.mask, a.offsets, a.frag,
                    a.frag_base, a.frag_capacity, a.Xout, a.Hout, a.CTZ, a.mismatches};
  if (tile == TILE_AUTO) tile = pick_tile(M, N, K);
  switch (tile) {
    case TILE_128: return launch_vijp_dual<Tile128, RELU>(M, N, K, a.X, a.W, a.Hin, a.P, epi, stream);
    case TILE_64: return launch_vijp_dual<Tile64, RELU>(M, N, K, a.X, a.W, a.Hin, a.P, epi, stream);
    case TILE_32K4: return launch_vijp_dual<Tile32K4, RELU>(M, N, K, a.X, a.W, a.Hin, a.P, epi, stream);
    case TILE_32K8: return launch_vijp_dual<Tile32K8, RELU>(M, N, K, a.X, a.W, a.Hin, a.P, epi, stream);
    case TILE_64K2: return launch_vijp_dual<Tile64K2, RELU>(M, N, K, a.X, a.W, a.Hin, a.P, epi, stream);
    case TILE_128W8: return launch_vijp_dual<Tile128W8, RELU>(M, N, K, a.X, a.W, a.Hin, a.P, epi, stream);
    case TILE_64X128: return launch_vijp_dual<Tile64x128, RELU>(M, N, K, a.X, a.W, a.Hin, a.P, epi, stream);
    default: return hipErrorInvalidValue;
  }
}

template <class CfgV, bool RELU, class CfgD>
static hipError_t pair_t(int M, int N, int K, const VijpArgs& a, const DwArgs& d, hipStream_t stream) {
  static_assert(CfgV::NT == CfgD::NT, "both tasks run in workgroups of the same size");
  EpiVijp<RELU> epi{a.bias, a.alpha, a.alpha > 0.f ? 1.0f / a.alpha : 0.f, a.mask, a.offsets, a.frag,
                    a.frag_base, a.frag_capacity, a.Xout, a.Hout, a.CTZ, a.mismatches};
  EpiStore es{d.dW, d.N, d.scale, d.beta, nullptr};
  auto tv = make_vijp_task<CfgV, true, RELU>(M, N, K, a.X, a.W, a.Hin, a.P, epi);
  auto td = make_gemm_task<CfgD, RCONTIG, RCONTIG, true, ANone, EpiStore, true>(d.M, d.N, d.K, d.CTZ, d.M, d.X, d.N,
                                                                               ANone{}, es, d.db, d.scale);
  td.colsum_beta = d.beta;
  return launch_task_pair<CfgV::NT>(tv, td, stream);
}

// tile_d comes from pick_tile_dw: among the four-wavefront tiles next to a four-wavefront layer
// kernel, the eight-wavefront 128x128 tile otherwise
template <class CfgV, bool RELU>
static hipError_t pair_d(int tile_d, int M, int N, int K, const VijpArgs& a, const DwArgs& d, hipStream_t stream) {
  if constexpr (CfgV::NT == 512) {
    return pair_t<CfgV, RELU, Tile128W8>(M, N, K, a, d, stream);
  } else {
    if (tile_d == TILE_128) return pair_t<CfgV, RELU, Tile128>(M, N, K, a, d, stream);
    return pair_t<CfgV, RELU, Tile64>(M, N, K, a, d, stream);
  }
}

template <bool RELU>
static hipError_t pair_v(int tile_v, int tile_d, int M, int N, int K, const VijpArgs& a, const DwArgs& d,
                         hipStream_t stream) {
  switch (tile_v) {
    case TILE_128W8: return pair_d<Tile128W8, RELU>(tile_d, M, N, K, a, d, stream);
    case TILE_64X128: return pair_d<Tile64x128, RELU>(tile_d, M, N, K, a, d, stream);
    case TILE_64K2: return pair_d<Tile64K2, RELU>(tile_d, M, N, K, a, d, stream);
    case TILE_128: return pair_d<Tile128, RELU>(tile_d, M, N, K, a, d, stream);
    case TILE_64: return pair_d<Tile64, RELU>(tile_d, M, N, K, a, d, stream);
    default: return pair_d<Tile32K4, RELU>(tile_d, M, N, K, a, d, stream);
  }
}

hipError_t gemm_phase3_pair(const VijpArgs* v, int M, int N, int K, const DwArgs* d, hipStream_t stream) {
  const int tile_v = v ? pick_tile(M, N, K) : TILE_AUTO;
  const int tile_d = d ? pick_tile_dw(d->M, d->N, d->K, tile_v, true) : TILE_AUTO;
  if (v && d && M > 0 && N > 0 && d->M > 0 && d->N > 0 && d->db) {
    const bool shapes_ok = extent_ok(M, K, K) && extent_ok(N, K, K) && extent_ok(M, N, N) &&
                           extent_ok(d->K, d->M, d->M) && extent_ok(d->K, d->N, d->N) && extent_ok(d->M, d->N, d->N);
    const bool vec = vijp_vec_ok(K, v->X, v->W, v->Hin, v->P) && operand_vec_ok(d->CTZ, d->M, d->M) &&
                     operand_vec_ok(d->X, d->N, d->N);
    if (shapes_ok && vec && tile_v != TILE_32K8)
      return v->alpha == 0.f ? pair_v<true>(tile_v, tile_d, M, N, K, *v, *d, stream)
                             : pair_v<false>(tile_v, tile_d, M, N, K, *v, *d, stream);
  }
  if (v) {
    hipError_t e = gemm_vijp_dual(tile_v, M, N, K, *v, stream);
    if (e != hipSuccess) return e;
  }
  if (d) return gemm_dw(tile_d, d->M, d->N, d->K, d->CTZ, d->X, d->scale, d->dW, d->db, stream, d->beta);
  return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// Phase III of several stretches side by side (GroupedVijpTask / GroupedDwTask).

static_assert(MAX_GROUP == MAX_PHASE3_GROUP, "the task's set table and the driver's argument arrays");

bool phase3_group_ok(int M, int N, int K) {
  // layers whose Phase-I product takes the 32 x 32 tile with K split over four wavefronts (outputs too small to
  // fill the chip with larger tiles); pairs of whole 128-wide K tiles, so that the split falls on the same
  // boundaries and every set has an even number of 32-wide slices
  return M > 0 && N > 0 && K > 0 && K % 256 == 0 && N % 32 == 0 && pick_tile(M, N, K) == TILE_32K4 && extent_ok(M, K, K) &&
         extent_ok(N, K, K) && extent_ok(M, N, N);
}

template <bool RELU>
static GroupedVijpTask<Tile64, RELU, 4> make_grouped_vijp(int n, const VijpArgs* v, int M, int N, int K) {
  GroupedVijpTask<Tile64, RELU, 4> t{};
  t.n_sets = n;
  if (n <= 0) return t;  // no workgroups
  t.M = M; t.N = N; t.K = K;
  t.alpha = v[0].alpha;
  t.inv_alpha = v[0].alpha > 0.f ? 1.0f / v[0].alpha : 0.f;
  t.frag = v[0].frag;
  t.frag_capacity = v[0].frag_capacity;
  t.mismatches = v[0].mismatches;
  t.tiles_m = ceil_div(M, Tile64::BM);
  t.tiles_n = ceil_div(N, Tile64::BN);
  for (int g = 0; g < n; ++g)
    t.set[g] = VijpSet{v[g].X, v[g].W, v[g].Hin, v[g].P, v[g].bias, v[g].mask, v[g].offsets, v[g].frag_base,
                       v[g].Xout, v[g].Hout, v[g].CTZ};
  return t;
}

template <class CfgD>
static GroupedDwTask<CfgD> make_grouped_dw(int n, const DwArgs* d) {
  GroupedDwTask<CfgD> t{};
  t.n_sets = n;
  if (n <= 0) return t;  // no workgroups
  t.M = d[0].M; t.N = d[0].N; t.K = d[0].K;
  t.scale = d[0].scale;
  t.beta = d[0].beta;
  t.tiles_m = ceil_div(t.M, CfgD::BM);
  t.tiles_n = ceil_div(t.N, CfgD::BN);
  for (int g = 0; g < n; ++g) t.set[g] = DwSet{d[g].CTZ, d[g].X, d[g].dW, d[g].db};
  return t;
}

template <bool RELU, class CfgD, int MIN_WG>
static hipError_t group_t(int n_v, const VijpArgs* v, int M, int N, int K, int n_d, const DwArgs* d, hipStream_t stream) {
  static_assert(CfgD::NT == Tile64::NT, "both tasks run in workgroups of the same size");
  // MIN_WG workgroups of the layer task must fit a CU side by side (one's loads under the others' matrix
  // work): the register count is held to that share of a SIMD's file. Two is what measures best: the layer task
  // takes 182 registers by itself; squeezed into a third of the file (168) it spills inside its main loop
  // one kernel for every launch of the sweep: a group's first launch has no weight gradients yet, the last one
  // of the step no layer kernels left (an empty task takes no workgroups)
  return launch_task_pair_resident<Tile64::NT, MIN_WG>(make_grouped_vijp<RELU>(n_v, v, M, N, K),
                                                       make_grouped_dw<CfgD>(n_d, d), stream);
}

hipError_t gemm_phase3_group(int n_v, const VijpArgs* v, int M, int N, int K, int n_d, const DwArgs* d, hipStream_t stream) {
  if (n_v < 0 || n_d < 0 || n_v > MAX_GROUP || n_d > MAX_GROUP || (n_v == 0 && n_d == 0)) return hipErrorInvalidValue;
  if (n_v > 0) {
    if (!phase3_group_ok(M, N, K)) return hipErrorInvalidValue;
    for (int g = 0; g < n_v; ++g)
      if (!vijp_vec_ok(K, v[g].X, v[g].W, v[g].Hin, v[g].P) || v[g].alpha != v[0].alpha) return hipErrorInvalidValue;
  }
  int tile_d = TILE_64;
  if (n_d > 0) {
    // the tile the weight gradient takes next to a layer kernel of the 32 x 32 K-split tile (the same product
    // launched with one layer gets the same tile, hence the same bits)
    tile_d = pick_tile_dw(d[0].M, d[0].N, d[0].K, TILE_32K4, true);
    if (!extent_ok(d[0].K, d[0].M, d[0].M) || !extent_ok(d[0].K, d[0].N, d[0].N) || !extent_ok(d[0].M, d[0].N, d[0].N))
      return hipErrorInvalidValue;
    for (int g = 0; g < n_d; ++g) {
      if (d[g].M != d[0].M || d[g].N != d[0].N || d[g].K != d[0].K || d[g].scale != d[0].scale || d[g].beta != d[0].beta)
        return hipErrorInvalidValue;
      if (!operand_vec_ok(d[g].CTZ, d[g].M, d[g].M) || !operand_vec_ok(d[g].X, d[g].N, d[g].N)) return hipErrorInvalidValue;
    }
  }
  const bool relu = n_v > 0 && v[0].alpha == 0.f;
  if (tile_d == TILE_128)
    return relu ? group_t<true, Tile128, 2>(n_v, v, M, N, K, n_d, d, stream)
                : group_t<false, Tile128, 2>(n_v, v, M, N, K, n_d, d, stream);
  return relu ? group_t<true, Tile64, 2>(n_v, v, M, N, K, n_d, d, stream) : group_t<false, Tile64, 2>(n_v, v, M, N, K, n_d, d, stream);
}

template <class CfgD, class CfgR>
static hipError_t bp_pair_t(const BpLayerArgs& a, hipStream_t stream) {
  static_assert(CfgD::NT == CfgR::NT, "both tasks run in workgroups of the same size");
  ASlopeFromAct xf{a.act, a.alpha};
  EpiStore ed{a.dW, a.d_in, a.scale, 0.f, nullptr};
  EpiStore er{a.Hout, a.d_in, 1.f, 0.f, nullptr};
  auto td = make_gemm_task<CfgD, RCONTIG, RCONTIG, true, ASlopeFromAct, EpiStore, true>(
      a.d_out, a.d_in, a.batch, a.Hy, a.d_out, a.Xprev, a.d_in, xf, ed, a.db, a.scale);
  auto tr = make_gemm_task<CfgR, KCONTIG, RCONTIG, true, ASlopeFromAct, EpiStore, false>(
      a.batch, a.d_in, a.d_out, a.Hy, a.d_out, a.W, a.d_in, xf, er, nullptr, 0.f);
  return launch_task_pair<CfgD::NT>(tr, td, stream);
}

template <class CfgR>
static hipError_t bp_pair_d(int tile_d, const BpLayerArgs& a, hipStream_t stream) {
  if constexpr (CfgR::NT == 512) {
    return bp_pair_t<Tile64x128, CfgR>(a, stream);
  } else {
    if (tile_d == TILE_128) return bp_pair_t<Tile128, CfgR>(a, stream);
    return bp_pair_t<Tile64, CfgR>(a, stream);
  }
}

static hipError_t bp_pair_r(int tile_r, int tile_d, const BpLayerArgs& a, hipStream_t stream) {
  switch (tile_r) {
    case TILE_128W8: return bp_pair_d<Tile128W8>(tile_d, a, stream);
    case TILE_64X128: return bp_pair_d<Tile64x128>(tile_d, a, stream);
    case TILE_64K2: return bp_pair_d<Tile64K2>(tile_d, a, stream);
    case TILE_128: return bp_pair_d<Tile128>(tile_d, a, stream);
    case TILE_64: return bp_pair_d<Tile64>(tile_d, a, stream);
    default: return bp_pair_d<Tile32K4>(tile_d, a, stream);
  }
}

hipError_t gemm_bp_layer(const BpLayerArgs& a, hipStream_t stream) {
  const int tile_r = a.Hout ? pick_tile(a.batch, a.d_in, a.d_out) : TILE_AUTO;
  const int tile_d = pick_tile_dw(a.d_out, a.d_in, a.batch, tile_r, false);
  if (a.Hout && a.batch > 0 && a.d_in > 0 && a.d_out > 0) {
    const bool shapes_ok = extent_ok(a.batch, a.d_out, a.d_out) && extent_ok(a.batch, a.d_in, a.d_in) &&
                           extent_ok(a.d_out, a.d_in, a.d_in);
    const bool vec = operand_vec_ok(a.Hy, a.d_out, a.d_out) && aligned16(a.act) && operand_vec_ok(a.Xprev, a.d_in, a.d_in) &&
                     operand_vec_ok(a.W, a.d_in, a.d_in);
    if (shapes_ok && vec && tile_r != TILE_32K8)
      return bp_pair_r(tile_r, tile_d, a, stream);
  }
  hipError_t e = gemm_dw_act(tile_d, a.d_out, a.d_in, a.batch, a.Hy, a.act, a.alpha, a.Xprev, a.scale, a.dW, a.db, stream);
  if (e != hipSuccess || !a.Hout) return e;
  return gemm_rev_act(tile_r, a.batch, a.d_in, a.d_out, a.Hy, a.act, a.alpha, a.W, a.Hout, stream);
}

hipError_t gemm_vijp_dual(int tile, int M, int N, int K, const VijpArgs& a, hipStream_t stream) {
  return a.alpha == 0.f ? vijp_dual_t<true>(tile, M, N, K, a, stream) : vijp_dual_t<false>(tile, M, N, K, a, stream);
}

}  // namespace mw
