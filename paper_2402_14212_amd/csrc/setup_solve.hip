// Right inverse of a dense layer, P = (W W^T)^{-1} W, on the device.
//
// G = W W^T is factored by a blocked right-looking Cholesky (block size 64): the 64x64
// diagonal block is factored and inverted by one workgroup in LDS, the panel below it and the
// trailing update are GEMMs. P then comes from two blocked right-looking triangular solves,
// L Y = W and L^T P = Y, whose diagonal steps multiply by the stored inverses of the diagonal
// blocks and whose updates are GEMMs as well.
//
// A non-positive pivot means W W^T is not positive definite, i.e. W has no full row rank and
// the layer is not a submersion; the flag is raised and the factorisation continues with a
// unit pivot so that nothing non-finite is produced.
#include "mw_internal.h"

namespace mw {

// from gemm_nt.hip / gemm_nn.hip / gemm_tn.hip
hipError_t gemm_plain_nt(int tile, int M, int N, int K, float alpha, const float* A, int64_t lda, const float* B,
                         int64_t ldb, float beta, float* C, int64_t ldc, const float* bias, hipStream_t stream);
hipError_t gemm_plain_nn(int tile, int M, int N, int K, float alpha, const float* A, int64_t lda, const float* B,
                         int64_t ldb, float beta, float* C, int64_t ldc, const float* bias, hipStream_t stream);
hipError_t gemm_plain_tn(int tile, int M, int N, int K, float alpha, const float* A, int64_t lda, const float* B,
                         int64_t ldb, float beta, float* C, int64_t ldc, const float* bias, hipStream_t stream);

namespace {

constexpr int NB = 64;

// Factor the bs x bs diagonal block at G (row stride ldg) in place (lower triangle) and write
// the inverse of its Cholesky factor to Linv (64 x 64, row stride 64, zero outside the triangle).
// One workgroup per matrix: workgroup j takes the block `stride` floats after workgroup j - 1's.
__global__ void __launch_bounds__(256)
k_chol_diag(float* __restrict__ G0, int64_t ldg, int bs, float* __restrict__ Linv0, int64_t stride,
            int32_t* __restrict__ bad_pivot) {
  __shared__ float a[NB][NB + 1];
  __shared__ float x[NB][NB + 1];
  float* __restrict__ G = G0 + (int64_t)blockIdx.x * stride;
  float* __restrict__ Linv = Linv0 + (int64_t)blockIdx.x * stride;
  const int tid = threadIdx.x;
  for (int i = tid; i < NB * NB; i += 256) {
    int r = i / NB, c = i % NB;
    a[r][c] = (r < bs && c <= r) ? G[(int64_t)r * ldg + c] : 0.f;
    x[r][c] = 0.f;
  }
  __syncthreads();
  for (int j = 0; j < bs; ++j) {
    if (tid == 0) {
      float p = a[j][j];
      if (!(p > 0.f)) {
        *bad_pivot = 1;
        p = 1.f;
      }
      a[j][j] = sqrtf(p);
    }
    __syncthreads();
    const float d = a[j][j];
    for (int i = j + 1 + tid; i < bs; i += 256) a[i][j] /= d;
    __syncthreads();
    // trailing update of the lower triangle: a[i][c] -= a[i][j] * a[c][j], j < c <= i
    const int rem = bs - j - 1;
    for (int t = tid; t < rem * rem; t += 256) {
      int i = j + 1 + t / rem, c = j + 1 + t % rem;
      if (c <= i) a[i][c] -= a[i][j] * a[c][j];
    }
    __syncthreads();
  }
  // inverse of the lower-triangular factor, one column per thread (forward substitution)
  if (tid < bs) {
    const int c = tid;
    x[c][c] = 1.f / a[c][c];
    for (int i = c + 1; i < bs; ++i) {
      float s = 0.f;
      for (int t = c; t < i; ++t) s += a[i][t] * x[t][c];
      x[i][c] = -s / a[i][i];
    }
  }
  __syncthreads();
  for (int i = tid; i < NB * NB; i += 256) {
    int r = i / NB, c = i % NB;
    Linv[i] = x[r][c];
    if (r < bs && c <= r) G[(int64_t)r * ldg + c] = a[r][c];
  }
}

}  // namespace

size_t setup_work_floats(int d_out, int d_in) {
  size_t n = (size_t)d_out, m = (size_t)d_in;
  size_t nblk = (n + NB - 1) / NB;
  return n * n + n * m + nblk * NB * NB;
}

#define MW_TRY(expr)                  \
  do {                                \
    hipError_t e__ = (expr);          \
    if (e__ != hipSuccess) return e__; \
  } while (0)

// `count` layers of one shape side by side (layer j works in work + j * setup_work_floats(d_out, d_in)):
// the steps of one layer depend on each other, those of different layers do not, so the 64 x 64
// diagonal factorisations (one workgroup each, about 110 us) of all layers are one launch per block
// step instead of one per layer and step; the products are issued layer by layer.
hipError_t setup_right_inverse_group(int count, const float* const* W, int d_out, int d_in, float* const* P, float* work,
                                     int32_t* bad_pivot, hipStream_t stream) {
  const int n = d_out, m = d_in;
  const int nblk = (n + NB - 1) / NB;
  const size_t ws = setup_work_floats(d_out, d_in);
  auto Gof = [&](int j) { return work + (size_t)j * ws; };
  auto Yof = [&](int j) { return Gof(j) + (size_t)n * n; };
  auto Dof = [&](int j) { return Yof(j) + (size_t)n * m; };

  for (int j = 0; j < count; ++j) {
    // G = W W^T
    MW_TRY(gemm_plain_nt(TILE_AUTO, n, n, m, 1.f, W[j], m, W[j], m, 0.f, Gof(j), n, nullptr, stream));
    // Y = W (right-hand side of the first solve, overwritten block row by block row)
    MW_TRY(ew_copy(W[j], Yof(j), (int64_t)n * m, stream));
  }

  // blocked Cholesky: G = L L^T, L stored in the lower triangle of G
  for (int k = 0; k < nblk; ++k) {
    const int k0 = k * NB, bs = (n - k0 < NB) ? n - k0 : NB, k1 = k0 + bs, below = n - k1;
    hipLaunchKernelGGL(k_chol_diag, dim3(count), dim3(256), 0, stream, Gof(0) + (size_t)k0 * n + k0, (int64_t)n, bs,
                       Dof(0) + (size_t)k * NB * NB, (int64_t)ws, bad_pivot);
    MW_TRY(hipGetLastError());
    for (int j = 0; below > 0 && j < count; ++j) {
      float* G = Gof(j);
      const float* Lk_inv = Dof(j) + (size_t)k * NB * NB;
      float* panel = G + (size_t)k1 * n + k0;  // [below][bs]
      // panel <- panel * Lkk^{-T}. In place is safe: with the 64-wide tile there is a single
      // column tile, so each workgroup reads only the rows it later writes.
      MW_TRY(gemm_plain_nt(TILE_64, below, bs, bs, 1.f, panel, n, Lk_inv, NB, 0.f, panel, n, nullptr, stream));
      // trailing block -= panel * panel^T
      MW_TRY(gemm_plain_nt(TILE_AUTO, below, below, bs, -1.f, panel, n, panel, n, 1.f,
                           G + (size_t)k1 * n + k1, n, nullptr, stream));
    }
  }

  for (int j = 0; j < count; ++j) {
    float* G = Gof(j);
    float* Y = Yof(j);
    const float* Dinv = Dof(j);
    // L Y = W, right-looking
    for (int k = 0; k < nblk; ++k) {
      const int k0 = k * NB, bs = (n - k0 < NB) ? n - k0 : NB, k1 = k0 + bs, below = n - k1;
      float* Yk = Y + (size_t)k0 * m;
      const float* Lk_inv = Dinv + (size_t)k * NB * NB;
      // Yk <- Lkk^{-1} Yk  (single row tile: in place is safe for the same reason as above)
      MW_TRY(gemm_plain_nn(TILE_64, bs, m, bs, 1.f, Lk_inv, NB, Yk, m, 0.f, Yk, m, nullptr, stream));
      if (below > 0)
        MW_TRY(gemm_plain_nn(TILE_AUTO, below, m, bs, -1.f, G + (size_t)k1 * n + k0, n, Yk, m, 1.f,
                             Y + (size_t)k1 * m, m, nullptr, stream));
    }
    // L^T P = Y, right-looking from the last block row upwards
    for (int k = nblk - 1; k >= 0; --k) {
      const int k0 = k * NB, bs = (n - k0 < NB) ? n - k0 : NB;
      const float* Yk = Y + (size_t)k0 * m;
      float* Pk = P[j] + (size_t)k0 * m;
      const float* Lk_inv = Dinv + (size_t)k * NB * NB;
      // Pk = Lkk^{-T} Yk
      MW_TRY(gemm_plain_tn(TILE_64, bs, m, bs, 1.f, Lk_inv, NB, Yk, m, 0.f, Pk, m, nullptr, stream));
      // rows above: Y[0:k0] -= L[k0:k1, 0:k0]^T Pk
      if (k0 > 0)
        MW_TRY(gemm_plain_tn(TILE_AUTO, k0, m, bs, -1.f, G + (size_t)k0 * n, n, Pk, m, 1.f, Y, m, nullptr, stream));
    }
  }
  return hipSuccess;
}

hipError_t setup_right_inverse(const float* W, int d_out, int d_in, float* P, float* work, int32_t* bad_pivot,
                               hipStream_t stream) {
  return setup_right_inverse_group(1, &W, d_out, d_in, &P, work, bad_pivot, stream);
}

}  // namespace mw
