// NN products: C[M][N] = A[M][K] B[K][N] (reverse vjp w.r.t. the layer input).
#include "gemm_dispatch.h"

namespace mw {

hipError_t gemm_plain_nn(int tile, int M, int N, int K, float alpha, const float* A, int64_t lda, const float* B,
                         int64_t ldb, float beta, float* C, int64_t ldc, const float* bias, hipStream_t stream) {
  EpiStore epi{C, ldc, alpha, beta, bias};
  return dispatch_gemm<KCONTIG, RCONTIG, false>(tile, M, N, K, A, lda, B, ldb, ANone{}, epi, true, nullptr, 0.f, stream);
}

hipError_t gemm_rev_fused(int tile, int M, int N, int K, const float* CTin, const float* W, const RevArgs& r,
                          hipStream_t stream) {
  if (r.alpha == 0.f) {
    EpiRevSlope<true> epi{r.CT, r.RAW, r.mask, r.alpha, r.offsets, r.frag, r.frag_base, r.frag_capacity, r.overflow};
    return dispatch_gemm<KCONTIG, RCONTIG, false>(tile, M, N, K, CTin, K, W, N, ANone{}, epi, true, nullptr, 0.f,
                                                  stream);
  }
  EpiRevSlope<false> epi{r.CT, r.RAW, r.mask, r.alpha, nullptr, nullptr, nullptr, 0, nullptr};
  return dispatch_gemm<KCONTIG, RCONTIG, false>(tile, M, N, K, CTin, K, W, N, ANone{}, epi, true, nullptr, 0.f, stream);
}

hipError_t gemm_rev_act(int tile, int M, int N, int K, const float* H, const float* act, float alpha,
                        const float* W, float* Hout, hipStream_t stream) {
  EpiStore epi{Hout, N, 1.f, 0.f, nullptr};
  ASlopeFromAct xf{act, alpha};
  const bool xf_ok = aligned16(act);
  return dispatch_gemm<KCONTIG, RCONTIG, false>(tile, M, N, K, H, K, W, N, xf, epi, xf_ok, nullptr, 0.f, stream);
}

}  // namespace mw
