// Convolution as a GEMM whose operand A is gathered from the image on the fly (no patch matrix in
// memory), and the three kernels the convolutional Moonwalk pass builds from it:
//   forward + activation + sign mask                       (Phase I, and backprop's forward)
//   recomputed forward + channel solve + vijp epilogue      (Phase III, one launch per layer chunk)
//   weight gradient, split over the patch rows               (Phase III, and backprop)
// Images are NHWC. Patch row r = (image, oy, ox), patch column q = (ky, kx, c): the element is
// x[image][oy*s - p + ky][ox*s - p + kx][c0 + c], zero outside the image (Sec. 4.2, Lemma 1 for the
// layers this is used on).
#pragma once

#include <type_traits>

#include "gemm_kernels.h"

namespace mw {

// n / d for n < 2^31 by one multiply-high (round-up reciprocal); d >= 1.
struct FastDiv {
  uint32_t mul, shift, d;
  FastDiv() : mul(0), shift(0), d(1) {}
  explicit FastDiv(uint32_t div) : d(div) {
    uint32_t l = 0;
    while ((1ull << l) < div) ++l;  // ceil(log2 d)
    if (div <= 1) {
      mul = 0;
      shift = 0;
    } else {
      mul = (uint32_t)(((1ull << (31 + l)) + div - 1) / div);  // < 2^32 because d > 2^(l-1)
      shift = l - 1;
    }
  }
  __device__ __forceinline__ uint32_t div(uint32_t n) const { return d == 1 ? n : (__umulhi(n, mul) >> shift); }
};

// Operand-A gather for the patch matrix of a convolution (all extents in elements).
// Needs C, Csel and c0 to be multiples of 4 and a 16-byte aligned image, so that every chunk of
// four patch columns is four consecutive channels of one pixel.
struct AConvPatch {
  int H, W, C;       // image height, width, channels per pixel (the pixel stride)
  int Ho, Wo;        // output grid
  int k, s, p;       // taps per side, stride, padding
  int c0, Csel;      // channels [c0, c0 + Csel) of every tap enter the patch
  int row_off;       // patch row of the A pointer's row 0 (set per split by the split-K task)
  uint32_t bytes;    // extent of the image chunk behind the A pointer
  FastDiv d_howo, d_wo, d_csel, d_k;

  struct Dev {
    struct Aux {};
    const AConvPatch& g;
    int row_off;
    __device__ __forceinline__ Dev(const AConvPatch& p, int, int, int64_t) : g(p), row_off(p.row_off) {}
    // outer = patch row, inner = patch column, whatever the operand layout
    __device__ __forceinline__ Chunk chunk(int outer, int inner, int n_outer, int n_inner, int64_t) const {
      const uint32_t row = (uint32_t)(outer + row_off);
      const uint32_t b = g.d_howo.div(row), rem = row - b * (uint32_t)(g.Ho * g.Wo);
      const uint32_t oy = g.d_wo.div(rem), ox = rem - oy * (uint32_t)g.Wo;
      const uint32_t tap = g.d_csel.div((uint32_t)inner), c = (uint32_t)inner - tap * (uint32_t)g.Csel;
      const uint32_t ky = g.d_k.div(tap), kx = tap - ky * (uint32_t)g.k;
      const int iy = (int)oy * g.s - g.p + (int)ky, ix = (int)ox * g.s - g.p + (int)kx;
      const bool ok = outer < n_outer && inner < n_inner && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
      Chunk ch;
      ch.e = (((b * (uint32_t)g.H + (uint32_t)iy) * (uint32_t)g.W + (uint32_t)ix) * (uint32_t)g.C) + (uint32_t)g.c0 + c;
      ch.nvalid = ok ? 4 : 0;
      return ch;
    }
    __device__ __forceinline__ uint32_t extent(int, int, int64_t) const { return g.bytes; }
    template <bool VEC>
    __device__ __forceinline__ void fetch(Aux&, const Chunk&) const {}
    __device__ __forceinline__ float4 apply(float4 v, const Aux&) const { return v; }
  };
};

// Phase III for the rows of one image chunk of a convolutional layer:
//   acc0 = patches(x) w        (M x K1)(K1 x N)    the pre-activation again
//   acc1 = sub(h_in) Tinv^T    (M x N)(N x N)      the vijp: h_in at the strided positions, first N
//                                                  channels, times the inverse of the triangular tap
// then the leaky vijp epilogue (x out, h out, ct_z, sign check against the Phase-I mask).
template <class Cfg>
struct ConvVijpTask {
  int M, N, K1;
  const float* X;     // image chunk entering the layer
  const float* Wt;    // [K1][N]
  const float* Hin;   // cotangent chunk at the layer input (same geometry as X)
  const float* Tinv;  // [N][N]
  AConvPatch gx, gh;
  EpiVijp<false> epi;
  int tiles_m, tiles_n;
  static constexpr int LDS_A = lds_bytes<Cfg, KCONTIG, RCONTIG, 2>();
  static constexpr int LDS_B = lds_bytes<Cfg, KCONTIG, KCONTIG, 2>();
  static constexpr int LDS_BYTES = LDS_A > LDS_B ? LDS_A : LDS_B;
  __host__ __device__ int blocks() const { return tiles_m * tiles_n; }

  __device__ __forceinline__ void run(int bid, float* __restrict__ lds) const {
    int tm_i, tn_i;
    tile_coords(bid, tiles_m, tiles_n, tm_i, tn_i);
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
    {
      const AConvPatch::Dev dx(gx, M, K1, 0);
      gemm_mainloop<Cfg, KCONTIG, RCONTIG, true, false>(X, 0, Wt, N, M, N, K1, m0, n0, lds, dx, acc[0], asum);
    }
    {
      const AConvPatch::Dev dh(gh, M, N, 0);
      gemm_mainloop<Cfg, KCONTIG, KCONTIG, true, false>(Hin, 0, Tinv, N, M, N, N, m0, n0, lds, dh, acc[1], asum);
    }
    typename EpiVijp<false>::Dev ed(epi, M, N);
    reduce_and_finish<Cfg, 2>(lds, M, N, m0, n0, acc, asum, ed);
    ed.finish();
  }
};

// One slice of a TN product split over K: part[slice][M][N] = A[k_lo .. k_hi)^T B[k_lo .. k_hi).
// A is either a plain [K][M] matrix or gathered (Xf = AConvPatch: K runs over patch rows, M over
// patch columns). The slices are summed afterwards in slice order by ew_reduce_slices, so the
// result does not depend on which workgroup finishes first.
template <class Cfg, class Xf>
struct SplitKTnTask {
  int M, N, K;
  const float* A;
  int64_t lda;
  const float* B;  // [K][N]
  int64_t ldb;
  Xf xf;
  float* part;
  int slices, k_per;  // k_per is a multiple of Cfg::BK
  int tiles_m, tiles_n;
  static constexpr bool GATHER = !std::is_same<Xf, ANone>::value;
  static constexpr int LDS_BYTES = lds_bytes<Cfg, RCONTIG, RCONTIG, 1>();
  __host__ __device__ int blocks() const { return tiles_m * tiles_n * slices; }

  __device__ __forceinline__ void run(int bid, float* __restrict__ lds) const {
    // the tiles of one slice read the same rows of both operands: keep them together on one XCD
    const int tiles = tiles_m * tiles_n;
    const int id = xcd_remap(bid, tiles * slices);
    const int slice = id / tiles, tile = id - slice * tiles;
    const int m0 = (tile % tiles_m) * Cfg::BM, n0 = (tile / tiles_m) * Cfg::BN;
    const int k_lo = slice * k_per;
    const int k_n = (K - k_lo) < k_per ? (K - k_lo) : k_per;

    f32x16 acc[1][Cfg::NACC];
    float asum[Cfg::WTM];
#pragma unroll
    for (int a = 0; a < Cfg::NACC; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[0][a][i] = 0.f;
#pragma unroll
    for (int t = 0; t < Cfg::WTM; ++t) asum[t] = 0.f;
    {
      typename Xf::Dev xd(xf, k_n, M, lda);
      const float* a = A;
      if constexpr (GATHER) xd.row_off += k_lo;
      else a += (int64_t)k_lo * lda;
      gemm_mainloop<Cfg, RCONTIG, RCONTIG, true, false>(a, lda, B + (int64_t)k_lo * ldb, ldb, M, N, k_n, m0, n0, lds, xd,
                                                        acc[0], asum);
    }
    EpiStore es{part + (int64_t)slice * M * N, N, 1.f, 0.f, nullptr};
    EpiStore::Dev ed(es, M, N);
    reduce_and_finish<Cfg, 1>(lds, M, N, m0, n0, acc, asum, ed);
  }
};

}  // namespace mw
