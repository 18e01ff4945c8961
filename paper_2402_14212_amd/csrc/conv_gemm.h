// Convolution as a GEMM whose operand A is gathered from the image on the fly (no patch matrix in
// memory), and the three kernels the convolutional Moonwalk pass builds from it:
//   forward + activation + sign mask                       (Phase I, and backprop's forward)
//   recomputed forward + channel solve + vijp epilogue      (Phase III, one launch per layer chunk)
//   weight gradient, split over the patch rows               (Phase III, and backprop)
//   input cotangent (the transposed convolution)            (Phase II, and backprop)
// Images are NHWC. Patch row r = (image, oy, ox), patch column q = (ky, kx, c): the element is
// x[image][oy*s - py + ky][ox*s - px + kx][c0 + c], zero outside the image (Sec. 4.2, Lemma 1 for the
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
// four patch columns is four consecutive channels of one pixel; with the patch columns along K
// (forward, input cotangent) Csel must be a multiple of the K tile, so that a tile lies inside one
// tap (the launchers choose the tile accordingly).
//
// The element offset splits into a part that depends on the patch row only and one that depends on
// the patch column only, e = rowterm(b, oy, ox) + colterm(ky, kx, c). In each operand layout one of
// the two is fixed per thread for the whole K loop and is worked out once (prepare); the other
// belongs to the K tile and is carried from tile to tile in workgroup-wide (scalar) state
// (advance), so the loop itself has neither divisions nor full multiplies:
//   columns along K: (ky, kx, first channel) of the tile; the thread adds its fixed row part.
//   rows along K:    (b, oy, ox) of the tile's first row; the thread's row is a fixed number of
//                    rows further on, which is at most one carry in ox and one in oy after its
//                    fixed (image, row, column) displacement has been added.
struct AConvPatch {
  int H, W, C;       // image height, width, channels per pixel (the pixel stride)
  int Ho, Wo;        // output grid
  int kh, kw;        // taps in y and x
  int s, py, px;     // stride, offsets (the padding) in y and x
  int c0, Csel;      // channels [c0, c0 + Csel) of every tap enter the patch
  int row_off;       // patch row of the A pointer's row 0 (set per split by the split-K task)
  int xdiag;         // 1: rows run along an anti-diagonal of the image, x = ox*s - px - oy (columns along K only;
                     // the grid is then Ho x 1 and oy counts the positions of the diagonal)
  uint32_t bytes;    // extent of the image chunk behind the A pointer
  uint32_t d1, d2;   // change of the row part of the offset (mod 2^32) when ox wraps to the next output
                     // row: (W - Wo) s C, and when oy wraps to the next image: (H - Ho s) W C
  FastDiv d_howo, d_wo, d_csel, d_kw;

  static constexpr int MAX_CHUNKS = 4;   // chunks of one operand tile per thread, over all tile shapes
  static constexpr int FAR = 1 << 28;    // a coordinate no image reaches: marks rows / columns outside the matrix

  struct Dev {
    struct Aux {};
    const AConvPatch& g;
    int row_off;
    // per-thread, fixed for the K loop
    uint32_t fterm[MAX_CHUNKS];
    int fy[MAX_CHUNKS], fx[MAX_CHUNKS];   // columns along K: iy0, ix0 of the row; rows along K: ky, kx of the column
    uint32_t dx[MAX_CHUNKS], dy[MAX_CHUNKS];  // rows along K: the thread's row displacement inside a tile
    int rr[MAX_CHUNKS];                   // rows along K: the thread's row offset inside a tile
    // workgroup-wide, per K tile
    uint32_t tterm;                       // colterm of the tile (columns along K) / rowterm of its first row
    int ky, kx, cb;                       // columns along K
    uint32_t b0, oy0, ox0;                // rows along K
    int k_left;                           // k still inside the matrix from this tile's start on

    __device__ __forceinline__ Dev(const AConvPatch& p, int, int, int64_t) : g(p), row_off(p.row_off) {}

    __device__ __forceinline__ uint32_t row_term(uint32_t b, uint32_t oy, uint32_t ox) const {  // mod 2^32
      const uint32_t iy0 = oy * (uint32_t)g.s - (uint32_t)g.py;
      const uint32_t ix0 = ox * (uint32_t)g.s - (uint32_t)g.px - (uint32_t)g.xdiag * oy;
      return ((b * (uint32_t)g.H + iy0) * (uint32_t)g.W + ix0) * (uint32_t)g.C;
    }
    __device__ __forceinline__ void split_row(uint32_t row, uint32_t& b, uint32_t& oy, uint32_t& ox) const {
      b = g.d_howo.div(row);
      const uint32_t rem = row - b * (uint32_t)(g.Ho * g.Wo);
      oy = g.d_wo.div(rem);
      ox = rem - oy * (uint32_t)g.Wo;
    }

    template <int LAYOUT, int R, int BK, int NT>
    __device__ __forceinline__ void prepare(int row0, int n_rows, int n_k) {
      constexpr int NV = R * BK / 4 / NT;
      static_assert(NV <= MAX_CHUNKS, "tile shape has more chunks per thread than the gather keeps state for");
      k_left = n_k;
      if (LAYOUT == KCONTIG) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const int f = (int)threadIdx.x + i * NT;
          const int row = row0 + f / (BK / 4), kk = 4 * (f % (BK / 4));
          uint32_t b, oy, ox;
          split_row((uint32_t)(row + row_off), b, oy, ox);
          fterm[i] = row_term(b, oy, ox) + (uint32_t)kk;
          fy[i] = row < n_rows ? (int)oy * g.s - g.py : FAR;
          fx[i] = (int)ox * g.s - g.px - g.xdiag * (int)oy;
        }
        ky = 0; kx = 0; cb = 0;
        tterm = (uint32_t)g.c0;
      } else {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const int f = (int)threadIdx.x + i * NT;
          const int col = row0 + 4 * (f % (R / 4));
          const uint32_t tap = g.d_csel.div((uint32_t)col), c = (uint32_t)col - tap * (uint32_t)g.Csel;
          const uint32_t ty = g.d_kw.div(tap), tx = tap - ty * (uint32_t)g.kw;
          rr[i] = f / (R / 4);
          // the displacement of rr rows: whole images, whole output rows, columns
          uint32_t db, dyy, dxx;
          split_row((uint32_t)rr[i], db, dyy, dxx);
          dy[i] = dyy;
          dx[i] = dxx;
          fterm[i] = (ty * (uint32_t)g.W + tx) * (uint32_t)g.C + (uint32_t)g.c0 + c    // colterm
                     + row_term(db, dyy, dxx) - row_term(0, 0, 0);                    // + displacement of the row
          fy[i] = col < n_rows ? (int)ty : FAR;
          fx[i] = (int)tx;
        }
        split_row((uint32_t)row_off, b0, oy0, ox0);
        tterm = row_term(b0, oy0, ox0);
      }
    }

    template <int LAYOUT, int BK>
    __device__ __forceinline__ void advance() {
      k_left -= BK;
      if (LAYOUT == KCONTIG) {
        cb += BK;
        tterm += (uint32_t)BK;
        if (cb >= g.Csel) {  // next tap
          cb = 0;
          tterm += (uint32_t)(g.C - g.Csel);
          if (++kx == g.kw) {
            kx = 0;
            ++ky;
            tterm += (uint32_t)((g.W - g.kw) * g.C);
          }
        }
      } else {
        ox0 += (uint32_t)BK;
        while (ox0 >= (uint32_t)g.Wo) {
          ox0 -= (uint32_t)g.Wo;
          if (++oy0 == (uint32_t)g.Ho) {
            oy0 = 0;
            ++b0;
          }
        }
        tterm = row_term(b0, oy0, ox0);
      }
    }

    // outer = patch row and inner = patch column in either layout
    template <int LAYOUT>
    __device__ __forceinline__ Chunk chunk(int i, int, int, int, int, int64_t) const {
      Chunk ch;
      int iy, ix;
      if (LAYOUT == KCONTIG) {
        const int kyv = k_left > 0 ? ky : FAR;   // tiles requested beyond K read nothing
        ch.e = fterm[i] + tterm;
        iy = fy[i] + kyv;
        ix = fx[i] + kx;
      } else {
        // the thread's row: first row of the tile displaced by (db, dy, dx); one carry at most in ox
        // and in oy, because every summand is below its modulus
        uint32_t ox = ox0 + dx[i];
        const bool c1 = ox >= (uint32_t)g.Wo;
        ox -= c1 ? (uint32_t)g.Wo : 0u;
        uint32_t oy = oy0 + dy[i] + (c1 ? 1u : 0u);
        const bool c2 = oy >= (uint32_t)g.Ho;
        oy -= c2 ? (uint32_t)g.Ho : 0u;
        ch.e = fterm[i] + tterm + (c1 ? g.d1 : 0u) + (c2 ? g.d2 : 0u);
        const int kyv = rr[i] < k_left ? fy[i] : FAR;  // rows beyond this product's K range read nothing
        iy = __mul24((int)oy, g.s) - g.py + kyv;
        ix = __mul24((int)ox, g.s) - g.px + fx[i];
      }
      ch.nvalid = ((unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W) ? 4 : 0;
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
      AConvPatch::Dev dx(gx, M, K1, 0);
      gemm_mainloop<Cfg, KCONTIG, RCONTIG, true, false>(X, 0, Wt, N, M, N, K1, m0, n0, lds, dx, acc[0], asum);
    }
    {
      AConvPatch::Dev dh(gh, M, N, 0);
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

// ---------------------------------------------------------------------------------------------
// Input cotangent of a convolution, h[b, iy, ix, :] = sum over taps (ky, kx) with (iy + p - ky) and
// (ix + p - kx) divisible by s of ct_z[b, (iy + p - ky) / s, (ix + p - kx) / s, :] w[ky, kx, :, :]^T.
// The input pixels fall into s x s classes by ((iy + p) mod s, (ix + p) mod s); within a class every
// pixel sees the same taps, so each class is one product
//   (pixels of the class) x (its taps x C_out)  times  (its taps x C_out) x C_in
// whose operand A is gathered from ct_z (stride 1) and whose rows are scattered to the class's
// pixels. The per-class weight matrices are packed once per weight update (cv_pack_rev_weights).
constexpr int CONV_REV_MAX_CLASSES = 9;

struct RevClass {
  AConvPatch g;    // gather from ct_z: Ho, Wo = the class's pixel grid per image, s = 1
  int oy, ox;      // image position of grid point (0, 0); grid point (qy, qx) is pixel (oy + s qy, ox + s qx)
  int K, M;        // taps * C_out; n_img * grid points
  int tiles_m;
  int first;       // first block of the class in the launch (a multiple of 8)
  int64_t w_off;   // start of the class's [K][C_in] weights in the packed array
};

// h (RAW, may be NULL) and/or its product with the previous layer's activation slope (CT with
// mask32 and alpha, may be NULL) at the scattered pixel.
struct EpiConvRev {
  float* RAW;
  float* CT;
  const uint32_t* mask32;  // sign bits of the layer input's flat index, 32 per word
  float alpha;
  int H, W, s;             // input image and stride
  uint32_t bytes;          // extent of the image chunk behind RAW / CT
  struct Dev {
    __amdgpu_buffer_rsrc_t rraw, rct, rmask;
    const EpiConvRev& p;
    const RevClass& rc;
    __device__ __forceinline__ Dev(const EpiConvRev& e, const RevClass& c) : p(e), rc(c) {
      rraw = make_rsrc(e.RAW, e.RAW ? e.bytes : 0u);
      rct = make_rsrc(e.CT, e.CT ? e.bytes : 0u);
      rmask = make_rsrc(e.mask32, e.CT ? (e.bytes / 128u + 1u) * 4u : 0u);
    }
    template <int CNT>
    __device__ __forceinline__ void part(int M, int N, int row_base, int col, int g, int i0,
                                         const float (&v)[1][CNT]) const {
      const bool cv = col < N;
      const bool raw = p.RAW != nullptr, ct = p.CT != nullptr;
      uint32_t off[CNT], word[CNT];
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        const int row = row_base + acc_row(i0 + j, g);
        const uint32_t b = rc.g.d_howo.div((uint32_t)row), rem = (uint32_t)row - b * (uint32_t)(rc.g.Ho * rc.g.Wo);
        const uint32_t qy = rc.g.d_wo.div(rem), qx = rem - qy * (uint32_t)rc.g.Wo;
        const uint32_t pix = (b * (uint32_t)p.H + (uint32_t)rc.oy + (uint32_t)p.s * qy) * (uint32_t)p.W + (uint32_t)rc.ox +
                             (uint32_t)p.s * qx;
        const uint32_t e = pix * (uint32_t)N + (uint32_t)col;
        const bool valid = cv && row < M;
        off[j] = valid ? e * 4u : OOB;
        word[j] = buf_load_u32(rmask, (ct && valid) ? (e >> 5) * 4u : OOB);
      }
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        const float h = v[0][j];
        if (raw) buf_store_f32(rraw, off[j], h);
        if (ct) {
          // bit index e & 31 = col & 31 because N is a multiple of 32
          const bool bit = (word[j] >> ((uint32_t)col & 31u)) & 1u;
          buf_store_f32(rct, off[j], h * (bit ? 1.f : p.alpha));
        }
      }
    }
  };
};

// ---------------------------------------------------------------------------------------------
// The general vijp of a submersive convolution (kernels wider than padding + stride): the equation of
// h[s i', s j', :C_out] then also holds earlier output positions (i' - a, j' - b), 0 <= a, b <= reach,
// through the taps (p + a s, p + b s) (constructive proof of the lemma on submersive convolutional
// layers). With G = sub(h) T^{-T} computed for all positions at once,
//     h'[i', j'] = G[i', j'] - sum_{(a, b) != (0, 0)} h'[i' - a, j' - b] (T^{-1} w[p + a s][p + b s][:C_out])^T,
// and every position of an anti-diagonal i' + j' = d depends on earlier diagonals only: one launch per
// diagonal, rows = (image, position on the diagonal), operand A gathered from the h' image itself.
struct EpiDiagAccum {
  float* OUT;          // the h' image chunk, [n_img][Ho][Wo][N]; the diagonal's entries hold G and get the sum subtracted
  int n_d;             // positions on the diagonal
  int img_pixels;      // Ho * Wo
  int f0, step;        // flat pixel index of the diagonal's first position, and the step to the next (Wo - 1)
  uint32_t bytes;
  FastDiv d_nd;
  struct Dev {
    __amdgpu_buffer_rsrc_t ro;
    const EpiDiagAccum& p;
    __device__ __forceinline__ Dev(const EpiDiagAccum& e, int, int) : p(e) { ro = make_rsrc(e.OUT, e.bytes); }
    template <int CNT>
    __device__ __forceinline__ void part(int M, int N, int row_base, int col, int g, int i0, const float (&v)[1][CNT]) const {
      uint32_t off[CNT];
      float old[CNT];
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        const int row = row_base + acc_row(i0 + j, g);
        const uint32_t b = p.d_nd.div((uint32_t)row), m = (uint32_t)row - b * (uint32_t)p.n_d;
        const uint32_t pix = b * (uint32_t)p.img_pixels + (uint32_t)p.f0 + m * (uint32_t)p.step;
        off[j] = (col < N && row < M) ? (pix * (uint32_t)N + (uint32_t)col) * 4u : OOB;
        old[j] = buf_load_f32(ro, off[j]);
      }
#pragma unroll
      for (int j = 0; j < CNT; ++j) buf_store_f32(ro, off[j], old[j] - v[0][j]);
    }
    __device__ __forceinline__ void finish() const {}
  };
};

template <class Cfg>
struct ConvRevTask {
  int n_cls, N;        // classes; N = C_in
  const float* CT;     // ct_z chunk [n_img][Ho][Wo][C_out]
  const float* Wrev;   // packed per-class weights
  EpiConvRev epi;
  int tiles_n, total_blocks;
  RevClass cls[CONV_REV_MAX_CLASSES];
  static constexpr int LDS_BYTES = lds_bytes<Cfg, KCONTIG, RCONTIG, 1>();
  __host__ __device__ int blocks() const { return total_blocks; }

  __device__ __forceinline__ void run(int bid, float* __restrict__ lds) const {
    int c = n_cls - 1;
    while (c > 0 && bid < cls[c].first) --c;
    const RevClass& rc = cls[c];
    const int b = bid - rc.first;
    if (b >= rc.tiles_m * tiles_n) return;  // padding up to the next class (whole workgroup)
    int tm_i, tn_i;
    tile_coords(b, rc.tiles_m, tiles_n, tm_i, tn_i);
    const int m0 = tm_i * Cfg::BM, n0 = tn_i * Cfg::BN;
    f32x16 acc[1][Cfg::NACC];
    float asum[Cfg::WTM];
#pragma unroll
    for (int a = 0; a < Cfg::NACC; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[0][a][i] = 0.f;
#pragma unroll
    for (int t = 0; t < Cfg::WTM; ++t) asum[t] = 0.f;
    {
      AConvPatch::Dev dg(rc.g, rc.M, rc.K, 0);
      gemm_mainloop<Cfg, KCONTIG, RCONTIG, true, false>(CT, 0, Wrev + rc.w_off, N, rc.M, N, rc.K, m0, n0, lds, dg, acc[0],
                                                        asum);
    }
    const EpiConvRev::Dev ed(epi, rc);
    reduce_and_finish<Cfg, 1>(lds, rc.M, N, m0, n0, acc, asum, ed);
  }
};

}  // namespace mw
