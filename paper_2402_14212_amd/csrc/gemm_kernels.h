// Kernels and epilogues built on gemm_f32.h, and their host-side launch helpers.
#pragma once

#include "gemm_f32.h"

namespace mw {

// ------------------------------------------------------------------------------------ epilogues

// C = alpha * acc (+ bias[col]) (+ beta * C)
struct EpiStore {
  float* C;
  int64_t ldc;
  float alpha, beta;
  const float* bias;
  __device__ __forceinline__ void operator()(int row, int col, bool valid, const float (&v)[1]) const {
    if (!valid) return;
    float r = alpha * v[0];
    if (bias) r += bias[col];
    float* c = C + (int64_t)row * ldc + col;
    if (beta != 0.f) r += beta * *c;
    *c = r;
  }
};

// Phase-I forward epilogue: z = acc + b, m = (z > 0), x = m ? z : alpha z. With MASK the 32
// sign bits each half-wavefront holds for one output row go out as one 32-bit half of a packed
// mask word (requires N % 32 == 0; the launcher checks).
template <bool MASK>
struct EpiFwdAct {
  float* X;
  int64_t ldx;
  const float* bias;
  float alpha;
  uint32_t* mask32;
  int64_t n_cols;
  __device__ __forceinline__ void operator()(int row, int col, bool valid, const float (&v)[1]) const {
    float z = 0.f;
    if (valid) {
      z = v[0];
      if (bias) z += bias[col];
    }
    bool bit = valid && (z > 0.f);
    if (valid) X[(int64_t)row * ldx + col] = bit ? z : alpha * z;
    if (MASK) {
      unsigned long long bal = __ballot(bit);
      int lane = threadIdx.x & 63;
      if ((lane & 31) == 0 && valid)
        mask32[((int64_t)row * n_cols + col) >> 5] = lane ? (uint32_t)(bal >> 32) : (uint32_t)bal;
    }
  }
};

// Phase-III epilogue for one layer. v[0] = x_{i-1} W^T (pre-bias), v[1] = h_{i-1} P^T.
//   leaky: m = (z > 0) recomputed; h_y = m ? ct_z : ct_z * (1/alpha).
//   ReLU : m = stored bit; ct_z zeroed where erased; h_y restored from the fragment store at
//          rank = offsets[word] + popcount(erased bits below e in the word).
// Every recomputed sign is compared with the stored phase-I bit; differences are counted.
template <bool RELU>
struct EpiVijp {
  const float* bias;
  float alpha, inv_alpha;
  const uint64_t* mask;
  const uint32_t* offsets;     // ReLU only
  const float* frag;           // ReLU only: start of the whole store
  const uint64_t* frag_base;   // ReLU only: device scalar, start of this layer in the store
  uint64_t frag_capacity;
  float* X;
  float* H;
  float* CTZ;
  int64_t n_cols;
  unsigned long long* mismatches;
  __device__ __forceinline__ void operator()(int row, int col, bool valid, const float (&v)[2]) const {
    if (!valid) return;
    int64_t e = (int64_t)row * n_cols + col;
    float z = v[0];
    if (bias) z += bias[col];
    uint64_t w = mask[e >> 6];
    int sh = (int)(e & 63);
    bool stored = (w >> sh) & 1ull;
    bool fresh = z > 0.f;
    if (fresh != stored) atomicAdd(mismatches, 1ull);
    bool bit;
    float c, h;
    if (RELU) {
      bit = stored;
      c = bit ? v[1] : 0.f;
      h = c;
      if (!bit) {
        uint64_t idx = *frag_base + offsets[e >> 6] + (uint64_t)__popcll(~w & ((1ull << sh) - 1ull));
        h = idx < frag_capacity ? frag[idx] : 0.f;
      }
    } else {
      bit = fresh;
      c = v[1];
      h = bit ? c : c * inv_alpha;
    }
    X[e] = bit ? z : alpha * z;
    H[e] = h;
    CTZ[e] = c;
  }
};

// ------------------------------------------------------------------------------------ kernels

template <class Cfg, int LA, int LB, class Xf, class Epi, bool COLSUM>
__global__ void __launch_bounds__(Cfg::NT)
gemm_kernel(int M, int N, int K, const float* __restrict__ A, int64_t lda, const float* __restrict__ B,
            int64_t ldb, Xf xf, Epi epi, float* __restrict__ colsum_out, float colsum_scale, int tiles_m,
            int tiles_n) {
  extern __shared__ __align__(16) float lds[];
  int tm_i, tn_i;
  tile_coords(tiles_m, tiles_n, tm_i, tn_i);
  const int m0 = tm_i * Cfg::BM, n0 = tn_i * Cfg::BN;

  f32x16 acc[1][Cfg::NACC];
  float asum[Cfg::WTM];
#pragma unroll
  for (int a = 0; a < Cfg::NACC; ++a)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[0][a][i] = 0.f;
#pragma unroll
  for (int t = 0; t < Cfg::WTM; ++t) asum[t] = 0.f;

  gemm_mainloop<Cfg, LA, LB, COLSUM>(A, lda, B, ldb, M, N, K, m0, n0, lds, xf, acc[0], asum);

  if (COLSUM) {
#pragma unroll
    for (int t = 0; t < Cfg::WTM; ++t) asum[t] += __shfl_xor(asum[t], 32);
  }
  if (!reduce_k_slices<Cfg, 1>(lds, acc, asum)) return;
  for_each_output<Cfg, 1>(M, N, m0, n0, acc, epi);

  if (COLSUM && n0 == 0) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wn = (wave / Cfg::WK) % Cfg::WN, wm = wave / (Cfg::WK * Cfg::WN);
    if (wn == 0 && lane < 32) {
#pragma unroll
      for (int t = 0; t < Cfg::WTM; ++t) {
        int row = m0 + (wm * Cfg::WTM + t) * 32 + lane;
        if (row < M) colsum_out[row] = colsum_scale * asum[t];
      }
    }
  }
}

// One layer of the phase-III sweep: both NT products for the same output tile, then EpiVijp.
//   acc0 = X[Bt][K] W[N][K]^T ,  acc1 = Hin[Bt][K] P[N][K]^T
template <class Cfg, bool RELU>
__global__ void __launch_bounds__(Cfg::NT)
vijp_dual_kernel(int M, int N, int K, const float* __restrict__ X, const float* __restrict__ W,
                 const float* __restrict__ Hin, const float* __restrict__ P, EpiVijp<RELU> epi, int tiles_m,
                 int tiles_n) {
  extern __shared__ __align__(16) float lds[];
  int tm_i, tn_i;
  tile_coords(tiles_m, tiles_n, tm_i, tn_i);
  const int m0 = tm_i * Cfg::BM, n0 = tn_i * Cfg::BN;

  f32x16 acc[2][Cfg::NACC];
  float asum[Cfg::WTM];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int a = 0; a < Cfg::NACC; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[s][a][i] = 0.f;
#pragma unroll
  for (int t = 0; t < Cfg::WTM; ++t) asum[t] = 0.f;

  const ANone none{};
  gemm_mainloop<Cfg, KCONTIG, KCONTIG, false>(X, K, W, K, M, N, K, m0, n0, lds, none, acc[0], asum);
  gemm_mainloop<Cfg, KCONTIG, KCONTIG, false>(Hin, K, P, K, M, N, K, m0, n0, lds, none, acc[1], asum);
  if (!reduce_k_slices<Cfg, 2>(lds, acc, asum)) return;
  for_each_output<Cfg, 2>(M, N, m0, n0, acc, epi);
}

// ------------------------------------------------------------------------------------ launch helpers

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Kernels here use up to ~72 KiB of dynamic LDS (the CU has 160 KiB); anything above the 64 KiB
// default needs the limit raised once per kernel.
template <class KernelT>
inline hipError_t ensure_lds(KernelT kernel, int bytes) {
  if (bytes <= 48 * 1024) return hipSuccess;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             bytes);
}

template <class Cfg, int LA, int LB, class Xf, class Epi, bool COLSUM>
inline hipError_t launch_gemm(int M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb,
                              const Xf& xf, const Epi& epi, float* colsum_out, float colsum_scale,
                              hipStream_t stream) {
  if (M <= 0 || N <= 0) return hipSuccess;
  auto kernel = gemm_kernel<Cfg, LA, LB, Xf, Epi, COLSUM>;
  constexpr int bytes = lds_bytes<Cfg, LA, LB, 1>();
  static hipError_t attr = ensure_lds(kernel, bytes);
  if (attr != hipSuccess) return attr;
  int tiles_m = ceil_div(M, Cfg::BM), tiles_n = ceil_div(N, Cfg::BN);
  hipLaunchKernelGGL(kernel, dim3(tiles_m * tiles_n), dim3(Cfg::NT), bytes, stream, M, N, K, A, lda, B, ldb, xf,
                     epi, colsum_out, colsum_scale, tiles_m, tiles_n);
  return hipGetLastError();
}

template <class Cfg, bool RELU>
inline hipError_t launch_vijp_dual(int M, int N, int K, const float* X, const float* W, const float* Hin,
                                   const float* P, const EpiVijp<RELU>& epi, hipStream_t stream) {
  if (M <= 0 || N <= 0) return hipSuccess;
  auto kernel = vijp_dual_kernel<Cfg, RELU>;
  constexpr int bytes = lds_bytes<Cfg, KCONTIG, KCONTIG, 2>();
  static hipError_t attr = ensure_lds(kernel, bytes);
  if (attr != hipSuccess) return attr;
  int tiles_m = ceil_div(M, Cfg::BM), tiles_n = ceil_div(N, Cfg::BN);
  hipLaunchKernelGGL(kernel, dim3(tiles_m * tiles_n), dim3(Cfg::NT), bytes, stream, M, N, K, X, W, Hin, P, epi,
                     tiles_m, tiles_n);
  return hipGetLastError();
}

}  // namespace mw
