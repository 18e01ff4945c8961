// NT products: C[M][N] = A[M][K] B[N][K]^T (forward pre-activations, affine vijp, Gram matrix).
#include "gemm_dispatch.h"

namespace mw {

hipError_t gemm_plain_nt(int tile, int M, int N, int K, float alpha, const float* A, int64_t lda, const float* B,
                         int64_t ldb, float beta, float* C, int64_t ldc, const float* bias, hipStream_t stream) {
  EpiStore epi{C, ldc, alpha, beta, bias};
  return dispatch_gemm<KCONTIG, KCONTIG, false>(tile, M, N, K, A, lda, B, ldb, ANone{}, epi, true, nullptr, 0.f, stream);
}

hipError_t gemm_fwd_act(int tile, int M, int N, int K, const float* X, const float* W, const float* bias,
                        float alpha, float* Xout, uint64_t* mask, hipStream_t stream, float* Zkeep) {
  if (mask) {
    if (N % 32 != 0) return hipErrorInvalidValue;
    EpiFwdAct<true> epi{Xout, bias, alpha, reinterpret_cast<uint32_t*>(mask), Zkeep};
    return dispatch_gemm<KCONTIG, KCONTIG, false>(tile, M, N, K, X, K, W, K, ANone{}, epi, true, nullptr, 0.f, stream);
  }
  EpiFwdAct<false> epi{Xout, bias, alpha, nullptr, Zkeep};
  return dispatch_gemm<KCONTIG, KCONTIG, false>(tile, M, N, K, X, K, W, K, ANone{}, epi, true, nullptr, 0.f, stream);
}

}  // namespace mw
