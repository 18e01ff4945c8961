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
    default: return hipErrorInvalidValue;
  }
}

hipError_t gemm_vijp_dual(int tile, int M, int N, int K, const VijpArgs& a, hipStream_t stream) {
  return a.alpha == 0.f ? vijp_dual_t<true>(tile, M, N, K, a, stream) : vijp_dual_t<false>(tile, M, N, K, a, stream);
}

}  // namespace mw
