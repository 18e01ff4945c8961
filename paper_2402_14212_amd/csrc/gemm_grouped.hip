// Grouped products: one launch for the same NT or NN product on several operand sets of one shape.
#include "gemm_dispatch.h"

namespace mw {

namespace {

template <class Cfg, int LA, int LB>
hipError_t grouped_t(int n_sets, int M, int N, int K, float alpha, const float* const* A, int64_t lda,
                     const float* const* B, int64_t ldb, float beta, const float* const* D, float* const* C, int64_t ldc,
                     hipStream_t stream, float eye) {
  GroupedGemmTask<Cfg, LA, LB> t{n_sets, M, N, K, A, lda, B, ldb, C, D, ldc, alpha, beta, ceil_div(M, Cfg::BM), ceil_div(N, Cfg::BN)};
  t.eye = eye;
  return launch_task<Cfg::NT>(t, stream);
}

template <int LA, int LB>
hipError_t grouped_l(int n_sets, int M, int N, int K, float alpha, const float* const* A, int64_t lda,
                     const float* const* B, int64_t ldb, float beta, const float* const* D, float* const* C, int64_t ldc,
                     hipStream_t stream, float eye, bool bf16) {
  // the tile one product of n_sets times the rows would take, among the tiles without a K split
  auto tiles = [&](int tm, int tn) { return (int64_t)n_sets * ceil_div(M, tm) * ceil_div(N, tn); };
  if (bf16) {
    if (tiles(128, 128) >= 512) return grouped_t<Tile128W8B, LA, LB>(n_sets, M, N, K, alpha, A, lda, B, ldb, beta, D, C, ldc, stream, eye);
    if (tiles(64, 128) >= 512) return grouped_t<Tile64x128B, LA, LB>(n_sets, M, N, K, alpha, A, lda, B, ldb, beta, D, C, ldc, stream, eye);
    return grouped_t<Tile64B, LA, LB>(n_sets, M, N, K, alpha, A, lda, B, ldb, beta, D, C, ldc, stream, eye);
  }
  if (tiles(128, 128) >= 512) return grouped_t<Tile128W8, LA, LB>(n_sets, M, N, K, alpha, A, lda, B, ldb, beta, D, C, ldc, stream, eye);
  if (tiles(64, 128) >= 512) return grouped_t<Tile64x128, LA, LB>(n_sets, M, N, K, alpha, A, lda, B, ldb, beta, D, C, ldc, stream, eye);
  return grouped_t<Tile64, LA, LB>(n_sets, M, N, K, alpha, A, lda, B, ldb, beta, D, C, ldc, stream, eye);
}

}  // namespace

// C[g] = alpha * op(A[g], B[g]) + beta * D[g] + eye * I for g < n_sets; op NT: A [M][K], B [N][K]; op NN: A [M][K], B [K][N].
// The tables hold device pointers and live in device memory. Every operand must be 16-byte aligned with a
// row stride that is a multiple of 4 floats (the caller checks; the kernels use 128-bit loads). bf16: the NN
// product's operands are rounded to bf16 in front of the matrix unit (sums and everything else in fp32).
hipError_t gemm_grouped(int op, int n_sets, int M, int N, int K, float alpha, const float* const* A, int64_t lda,
                        const float* const* B, int64_t ldb, float beta, const float* const* D, float* const* C, int64_t ldc,
                        hipStream_t stream, float eye, bool bf16) {
  if (n_sets <= 0 || M <= 0 || N <= 0) return hipSuccess;
  const bool b_k = op == OP_NT;
  if (!extent_ok(M, K, lda) || !extent_ok(b_k ? N : K, b_k ? K : N, ldb) || !extent_ok(M, N, ldc)) return hipErrorInvalidValue;
  if (eye != 0.f && M != N) return hipErrorInvalidValue;
  if (lda % 4 || ldb % 4 || ldc % 4 || (int64_t)n_sets * ceil_div(M, 64) * ceil_div(N, 64) > 0x7FFFFFFF) return hipErrorInvalidValue;
  switch (op) {
    case OP_NT:
      if (bf16) return hipErrorInvalidValue;
      return grouped_l<KCONTIG, KCONTIG>(n_sets, M, N, K, alpha, A, lda, B, ldb, beta, D, C, ldc, stream, eye, false);
    case OP_NN: return grouped_l<KCONTIG, RCONTIG>(n_sets, M, N, K, alpha, A, lda, B, ldb, beta, D, C, ldc, stream, eye, bf16);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mw
