// Tile dispatch shared by the gemm_*.hip translation units.
#pragma once
#include "gemm_kernels.h"
#include "mw_internal.h"

namespace mw {

template <int LA, int LB, bool COLSUM, class Xf, class Epi>
inline hipError_t dispatch_gemm(int tile, int M, int N, int K, const float* A, int64_t lda, const float* B,
                                int64_t ldb, const Xf& xf, const Epi& epi, bool xf_vec_ok, float* colsum_out,
                                float colsum_scale, hipStream_t stream, float colsum_beta = 0.f) {
  if (tile == TILE_AUTO) tile = pick_tile(M, N, K);
  switch (tile) {
    case TILE_128:
      return launch_gemm<Tile128, LA, LB, Xf, Epi, COLSUM>(M, N, K, A, lda, B, ldb, xf, epi, xf_vec_ok, colsum_out,
                                                          colsum_scale, stream, colsum_beta);
    case TILE_64:
      return launch_gemm<Tile64, LA, LB, Xf, Epi, COLSUM>(M, N, K, A, lda, B, ldb, xf, epi, xf_vec_ok, colsum_out,
                                                         colsum_scale, stream, colsum_beta);
    case TILE_32K4:
      return launch_gemm<Tile32K4, LA, LB, Xf, Epi, COLSUM>(M, N, K, A, lda, B, ldb, xf, epi, xf_vec_ok, colsum_out,
                                                           colsum_scale, stream, colsum_beta);
    case TILE_32K8:
      return launch_gemm<Tile32K8, LA, LB, Xf, Epi, COLSUM>(M, N, K, A, lda, B, ldb, xf, epi, xf_vec_ok, colsum_out,
                                                           colsum_scale, stream, colsum_beta);
    case TILE_64K2:
      return launch_gemm<Tile64K2, LA, LB, Xf, Epi, COLSUM>(M, N, K, A, lda, B, ldb, xf, epi, xf_vec_ok, colsum_out,
                                                           colsum_scale, stream, colsum_beta);
    case TILE_128W8:
      return launch_gemm<Tile128W8, LA, LB, Xf, Epi, COLSUM>(M, N, K, A, lda, B, ldb, xf, epi, xf_vec_ok, colsum_out,
                                                           colsum_scale, stream, colsum_beta);
    case TILE_64X128:
      return launch_gemm<Tile64x128, LA, LB, Xf, Epi, COLSUM>(M, N, K, A, lda, B, ldb, xf, epi, xf_vec_ok, colsum_out,
                                                           colsum_scale, stream, colsum_beta);
    default:
      return hipErrorInvalidValue;
  }
}

}  // namespace mw
