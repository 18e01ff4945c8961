// TN products: C[M][N] = A[K][M]^T B[K][N] (weight gradient; K is the batch), with the column
// sums of A (the bias gradient) as a by-product of the operand fetch.
#include "gemm_dispatch.h"

namespace mw {

hipError_t gemm_plain_tn(int tile, int M, int N, int K, float alpha, const float* A, int64_t lda, const float* B,
                         int64_t ldb, float beta, float* C, int64_t ldc, const float* bias, hipStream_t stream) {
  EpiStore epi{C, ldc, alpha, beta, bias};
  return dispatch_gemm<RCONTIG, RCONTIG, false>(tile, M, N, K, A, lda, B, ldb, ANone{}, epi, true, nullptr, 0.f, stream);
}

hipError_t gemm_dw(int tile, int M, int N, int K, const float* CTZ, const float* X, float scale, float* dW,
                   float* db, hipStream_t stream, float beta) {
  EpiStore epi{dW, N, scale, beta, nullptr};
  if (db)
    return dispatch_gemm<RCONTIG, RCONTIG, true>(tile, M, N, K, CTZ, M, X, N, ANone{}, epi, true, db, scale, stream, beta);
  return dispatch_gemm<RCONTIG, RCONTIG, false>(tile, M, N, K, CTZ, M, X, N, ANone{}, epi, true, nullptr, 0.f, stream);
}

hipError_t gemm_dw_act(int tile, int M, int N, int K, const float* Hy, const float* act, float alpha,
                       const float* X, float scale, float* dW, float* db, hipStream_t stream) {
  EpiStore epi{dW, N, scale, 0.f, nullptr};
  ASlopeFromAct xf{act, alpha};
  const bool xf_ok = aligned16(act);
  return dispatch_gemm<RCONTIG, RCONTIG, true>(tile, M, N, K, Hy, M, X, N, xf, epi, xf_ok, db, scale, stream);
}

}  // namespace mw
