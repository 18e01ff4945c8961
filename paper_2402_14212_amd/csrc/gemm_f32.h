// fp32 MFMA GEMM building blocks for gfx950 (CDNA4), wave64.
//
// One workgroup = WM x WN x WK wavefronts. Each wavefront owns WTM x WTN output tiles of 32x32
// (v_mfma_f32_32x32x2_f32) and, when WK > 1, one 32-wide slice of every K tile; the K slices
// are summed through LDS in a fixed order, so results are bit-identical run to run.
//
// Operand tiles travel global -> registers -> LDS. Global access is through buffer
// instructions: an out-of-range element is given an offset beyond the buffer, for which the
// hardware returns 0 (loads) or drops the access (stores), so the main loop and the epilogues
// contain no bounds branches. Two K tiles are in flight in registers while a third is being
// multiplied out of double-buffered LDS (one barrier per K tile).
//
// Operand layouts (ld = row stride in floats):
//   KCONTIG  element (row, k) at p[row * ld + k]     (k is the fast index in memory)
//   RCONTIG  element (row, k) at p[k * ld + row]     (row is the fast index in memory)
// "row" is the m index for operand A and the n index for operand B.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mw {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int KCONTIG = 0;
constexpr int RCONTIG = 1;
constexpr int NUM_XCD = 8;

// PREC_: 0 = fp32 matrix instructions (v_mfma_f32_32x32x2_f32); 1 = the operands are rounded to bf16 (to nearest
// even) on their way from LDS to the matrix unit and multiplied by v_mfma_f32_32x32x16_bf16, sums in fp32: for
// products whose result is a small correction to something held in fp32 (2^-8 relative error per operand).
template <int WTM_, int WTN_, int WM_, int WN_, int WK_, int ST_ = 2, int PREC_ = 0>
struct TileCfg {
  static constexpr int WTM = WTM_, WTN = WTN_, WM = WM_, WN = WN_, WK = WK_;
  static constexpr int PREC = PREC_;
  // operand tiles in flight in registers (even). Two is what measures best on every tile here:
  // with four, the extra registers cost more than the longer lead time gains.
  static constexpr int ST = ST_;
  static_assert(ST_ >= 2 && ST_ % 2 == 0, "the register pipeline alternates over two LDS stages");
  static constexpr int BM = 32 * WTM * WM;
  static constexpr int BN = 32 * WTN * WN;
  static constexpr int BK = 32 * WK;            // every wavefront consumes 32 k per K tile
  static constexpr int NT = 64 * WM * WN * WK;  // threads per workgroup
  static constexpr int NACC = WTM * WTN;        // 32x32 accumulator tiles per wavefront
};
using Tile128 = TileCfg<2, 2, 2, 2, 1>;   // 128 x 128, K tile 32, 4 wavefronts
using Tile64 = TileCfg<1, 1, 2, 2, 1>;    //  64 x  64, K tile 32, 4 wavefronts
using Tile32K4 = TileCfg<1, 1, 1, 1, 4>;  //  32 x  32, K tile 128 split over 4 wavefronts
using Tile32K8 = TileCfg<1, 1, 1, 1, 8>;  //  32 x  32, K tile 256 split over 8 wavefronts
using Tile64K2 = TileCfg<1, 1, 2, 2, 2>;  //  64 x  64, K tile 64 split over 2 groups of 4 wavefronts
using Tile128W8 = TileCfg<1, 2, 4, 2, 1>;  // 128 x 128, K tile 32, 8 wavefronts of 32 x 64
using Tile64x128 = TileCfg<1, 1, 2, 4, 1>;  //  64 x 128, K tile 32, 8 wavefronts of 32 x 32
using Tile128W8B = TileCfg<1, 2, 4, 2, 1, 2, 1>;   // the same three with bf16 matrix instructions
using Tile64x128B = TileCfg<1, 1, 2, 4, 1, 2, 1>;
using Tile64B = TileCfg<1, 1, 2, 2, 1, 2, 1>;

// LDS footprint (floats) of one operand tile of R rows.
template <int LAYOUT, int R, int BK>
__host__ __device__ constexpr int lds_tile_floats() {
  return LAYOUT == KCONTIG ? R * (BK + 4) : BK * (R + 4);
}

template <class Cfg, int LA, int LB>
__host__ __device__ constexpr int lds_stage_floats() {
  return lds_tile_floats<LA, Cfg::BM, Cfg::BK>() + lds_tile_floats<LB, Cfg::BN, Cfg::BK>();
}

// Bytes of dynamic LDS a kernel built from these pieces needs: two pipeline stages, and room
// for the split-K reduction (which reuses the same memory after the main loop).
template <class Cfg, int LA, int LB, int NSETS>
__host__ __device__ constexpr int lds_bytes() {
  int pipe = 2 * lds_stage_floats<Cfg, LA, LB>();
  int red = Cfg::WK > 1 ? Cfg::WK * Cfg::WM * Cfg::WN * (Cfg::NACC * 16 * NSETS + Cfg::WTM) * 64 : 0;
  return 4 * (pipe > red ? pipe : red);
}

// Workgroups are handed to the 8 XCDs round-robin by their linear id. Remap so that every XCD
// (one L2 each) works on a contiguous range of logical tile ids.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks) {
  int xcd = bid % NUM_XCD, local = bid / NUM_XCD;
  int base = nblocks / NUM_XCD, rem = nblocks % NUM_XCD;
  return xcd * base + (xcd < rem ? xcd : rem) + local;
}

// ---------------------------------------------------------------------------------------------
// Buffer resources. A raw buffer (stride 0) of `bytes` bytes starting at p: an access at byte
// offset >= bytes reads 0 / is dropped. OOB is the offset handed to every masked-off lane.
constexpr uint32_t OOB = 0x80000000u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
// extent in bytes of an [n_outer][n_inner] matrix with row stride ld (floats)
__device__ __forceinline__ uint32_t extent_bytes(int n_outer, int n_inner, int64_t ld) {
  if (n_outer <= 0 || n_inner <= 0) return 0u;
  return (uint32_t)((((int64_t)n_outer - 1) * ld + n_inner) * 4);
}
__device__ __forceinline__ float buf_load_f32(__amdgpu_buffer_rsrc_t r, uint32_t off) {
  return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0));
}
__device__ __forceinline__ uint32_t buf_load_u32(__amdgpu_buffer_rsrc_t r, uint32_t off) {
  return __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0);
}
__device__ __forceinline__ float4 buf_load_f32x4(__amdgpu_buffer_rsrc_t r, uint32_t off) {
  u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
  return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
__device__ __forceinline__ void buf_store_f32(__amdgpu_buffer_rsrc_t r, uint32_t off, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, (int)off, 0, 0);
}
__device__ __forceinline__ void buf_store_u32(__amdgpu_buffer_rsrc_t r, uint32_t off, uint32_t v) {
  __builtin_amdgcn_raw_buffer_store_b32(v, r, (int)off, 0, 0);
}

// One 4-element chunk of an operand tile: element offset of its first element and how many of
// its elements lie inside the matrix (VEC: 0 or 4).
struct Chunk {
  uint32_t e;   // outer * ld + inner
  int nvalid;   // 0..4
};

// ---------------------------------------------------------------------------------------------
// Operand-A transforms. A transform has two halves so that the global loads of a tile stay in
// flight while earlier tiles are multiplied: fetch() issues whatever extra loads it needs next
// to the operand's own load, apply() runs just before the values are written to LDS.

// Where operand A's chunks live. The default is a plain matrix: chunk (outer, inner) of an
// [n_outer][n_inner] array with row stride ld. A transform that gathers A from somewhere else
// (an image, for the patch matrix of a convolution) replaces these two functions.
struct ALinearDev {
  // Called once by the main loop before the first tile is requested (row0: the tile's first row of
  // the operand; n_rows, n_k: its extents), and once after every tile request, in tile order.
  template <int LAYOUT, int R, int BK, int NT>
  __device__ __forceinline__ void prepare(int /*row0*/, int /*n_rows*/, int /*n_k*/) {}
  template <int LAYOUT, int BK>
  __device__ __forceinline__ void advance() {}
  // i: which of the thread's chunks of the tile this is
  template <int LAYOUT>
  __device__ __forceinline__ Chunk chunk(int /*i*/, int outer, int inner, int n_outer, int n_inner, int64_t ld) const {
    Chunk c;
    c.e = (uint32_t)outer * (uint32_t)ld + (uint32_t)inner;
    const int left = n_inner - inner;
    c.nvalid = (outer < n_outer && left > 0) ? (left < 4 ? left : 4) : 0;
    return c;
  }
  __device__ __forceinline__ uint32_t extent(int n_outer, int n_inner, int64_t ld) const {
    return extent_bytes(n_outer, n_inner, ld);
  }
};

struct ANone {
  struct Dev : ALinearDev {
    struct Aux {};
    __device__ __forceinline__ Dev() {}
    __device__ __forceinline__ Dev(const ANone&, int, int, int64_t) {}
    template <bool VEC>
    __device__ __forceinline__ void fetch(Aux&, const Chunk&) const {}
    __device__ __forceinline__ float4 apply(float4 v, const Aux&) const { return v; }
  };
};

// Multiply by the activation slope taken from the stored activation itself: x > 0 <=> z > 0.
struct ASlopeFromAct {
  const float* act;  // same shape and row stride as A
  float alpha;
  struct Dev : ALinearDev {
    struct Aux { float4 a; };
    __amdgpu_buffer_rsrc_t rs;
    float alpha;
    __device__ __forceinline__ Dev(const ASlopeFromAct& p, int n_outer, int n_inner, int64_t ld) : alpha(p.alpha) {
      rs = make_rsrc(p.act, extent_bytes(n_outer, n_inner, ld));
    }
    template <bool VEC>
    __device__ __forceinline__ void fetch(Aux& aux, const Chunk& c) const {
      if (VEC) {
        aux.a = buf_load_f32x4(rs, c.nvalid ? c.e * 4u : OOB);
      } else {
        aux.a.x = buf_load_f32(rs, c.nvalid > 0 ? c.e * 4u : OOB);
        aux.a.y = buf_load_f32(rs, c.nvalid > 1 ? c.e * 4u + 4u : OOB);
        aux.a.z = buf_load_f32(rs, c.nvalid > 2 ? c.e * 4u + 8u : OOB);
        aux.a.w = buf_load_f32(rs, c.nvalid > 3 ? c.e * 4u + 12u : OOB);
      }
    }
    __device__ __forceinline__ float4 apply(float4 v, const Aux& aux) const {
      v.x *= (aux.a.x > 0.f) ? 1.f : alpha;
      v.y *= (aux.a.y > 0.f) ? 1.f : alpha;
      v.z *= (aux.a.z > 0.f) ? 1.f : alpha;
      v.w *= (aux.a.w > 0.f) ? 1.f : alpha;
      return v;
    }
  };
};

// ---------------------------------------------------------------------------------------------
// Global -> register -> LDS staging of one operand tile (R rows x BK k).
// VEC: the operand is 16-byte aligned with ld % 4 == 0 and a fast extent that is a multiple of
// 4, so every chunk is entirely inside or entirely outside and moves as one dwordx4.

// XfDev is the device-side state of an operand transform (ANone::Dev etc.).
template <int LAYOUT, int R, int BK, int NT, bool VEC, class XfDev>
struct TileLoader {
  static constexpr int NV = R * BK / 4 / NT;  // chunks per thread
  static_assert(R * BK % (4 * NT) == 0, "tile must divide evenly over the workgroup");
  float4 v[NV];
  typename XfDev::Aux aux[NV];

  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rs, int64_t ld, int row0, int k0, int n_rows, int n_k,
                                       const XfDev& xf) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int f = (int)threadIdx.x + i * NT;
      int outer, inner, n_outer, n_inner;
      if (LAYOUT == KCONTIG) {
        outer = row0 + f / (BK / 4); inner = k0 + 4 * (f % (BK / 4)); n_outer = n_rows; n_inner = n_k;
      } else {
        outer = k0 + f / (R / 4); inner = row0 + 4 * (f % (R / 4)); n_outer = n_k; n_inner = n_rows;
      }
      const Chunk c = xf.template chunk<LAYOUT>(i, outer, inner, n_outer, n_inner, ld);
      if (VEC) {
        v[i] = buf_load_f32x4(rs, c.nvalid ? c.e * 4u : OOB);
      } else {
        v[i].x = buf_load_f32(rs, c.nvalid > 0 ? c.e * 4u : OOB);
        v[i].y = buf_load_f32(rs, c.nvalid > 1 ? c.e * 4u + 4u : OOB);
        v[i].z = buf_load_f32(rs, c.nvalid > 2 ? c.e * 4u + 8u : OOB);
        v[i].w = buf_load_f32(rs, c.nvalid > 3 ? c.e * 4u + 12u : OOB);
      }
      xf.template fetch<VEC>(aux[i], c);
    }
  }

  __device__ __forceinline__ void store(float* __restrict__ lds, const XfDev& xf) const {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int f = (int)threadIdx.x + i * NT;
      float4 w = xf.apply(v[i], aux[i]);
      if (LAYOUT == KCONTIG) {
        int r = f / (BK / 4), c4 = f % (BK / 4);
        *reinterpret_cast<float4*>(lds + r * (BK + 4) + 4 * c4) = w;
      } else {
        int k = f / (R / 4), r4 = f % (R / 4);
        *reinterpret_cast<float4*>(lds + k * (R + 4) + 4 * r4) = w;
      }
    }
  }
};

// Fragment fetch for the 32x32x2 MFMA: lane l supplies row (l & 31) and, in MFMA step j of a
// half, k = 32 * wk + 16 * (l >> 5) + 8 * half + j. Both operands use the same k assignment.
template <int LAYOUT, int R, int BK>
__device__ __forceinline__ void read_frag8(const float* __restrict__ lds, int row, int kbase, float (&f)[8]) {
  if (LAYOUT == KCONTIG) {
    const float4* q = reinterpret_cast<const float4*>(lds + row * (BK + 4) + kbase);
    float4 a = q[0], b = q[1];
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
    f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] = lds[(kbase + j) * (R + 4) + row];
  }
}

// Multiply one staged K tile into the accumulators.
template <class Cfg, int LA, int LB, bool COLSUM>
__device__ __forceinline__ void mma_stage(const float* __restrict__ sa, const float* __restrict__ sb, int wm, int wn,
                                          int wk, int r, int g, f32x16 (&acc)[Cfg::NACC], float (&asum)[Cfg::WTM]) {
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int kbase = 32 * wk + 16 * g + 8 * half;
    float fa[Cfg::WTM][8], fb[Cfg::WTN][8];
#pragma unroll
    for (int tm = 0; tm < Cfg::WTM; ++tm)
      read_frag8<LA, Cfg::BM, Cfg::BK>(sa, (wm * Cfg::WTM + tm) * 32 + r, kbase, fa[tm]);
#pragma unroll
    for (int tn = 0; tn < Cfg::WTN; ++tn)
      read_frag8<LB, Cfg::BN, Cfg::BK>(sb, (wn * Cfg::WTN + tn) * 32 + r, kbase, fb[tn]);
    if (Cfg::PREC == 1) {
      // one 32x32x16 instruction per half: lane group g supplies the eight k values 16 g + 8 half + 0..7 of its
      // row for both operands (which k a slot stands for does not matter as long as A and B agree)
      static_assert(!(COLSUM && Cfg::PREC == 1), "column sums are taken from the fp32 operands");
      bf16x8 va[Cfg::WTM], vb[Cfg::WTN];
#pragma unroll
      for (int tm = 0; tm < Cfg::WTM; ++tm)
#pragma unroll
        for (int j = 0; j < 8; ++j) va[tm][j] = (__bf16)fa[tm][j];
#pragma unroll
      for (int tn = 0; tn < Cfg::WTN; ++tn)
#pragma unroll
        for (int j = 0; j < 8; ++j) vb[tn][j] = (__bf16)fb[tn][j];
#pragma unroll
      for (int tm = 0; tm < Cfg::WTM; ++tm)
#pragma unroll
        for (int tn = 0; tn < Cfg::WTN; ++tn)
          acc[tm * Cfg::WTN + tn] =
              __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[tm], vb[tn], acc[tm * Cfg::WTN + tn], 0, 0, 0);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int tm = 0; tm < Cfg::WTM; ++tm) {
          if (COLSUM) asum[tm] += fa[tm][j];
#pragma unroll
          for (int tn = 0; tn < Cfg::WTN; ++tn)
            acc[tm * Cfg::WTN + tn] =
                __builtin_amdgcn_mfma_f32_32x32x2f32(fa[tm][j], fb[tn][j], acc[tm * Cfg::WTN + tn], 0, 0, 0);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Main loop: acc += A_tile(m0.., :) * B_tile(n0.., :)^T over the whole K range.
// Must be entered by the whole workgroup; ends with a barrier, so LDS may be reused afterwards.
// If COLSUM, asum[tm] accumulates, per lane, the sum of the A values that lane fed to the MFMA
// (after the A transform); combined over lanes/waves by the caller into column sums of A.
// The accumulation order over K is fixed (tile by tile, the same for every launch with the same
// Cfg), which is what makes two kernels that call this with the same operands agree bit for bit.

// The register half of the pipeline: Cfg::ST tiles of each operand in flight.
template <class Cfg, int LA, int LB, bool VEC, class XfDev>
struct TilePipe {
  TileLoader<LA, Cfg::BM, Cfg::BK, Cfg::NT, VEC, XfDev> a[Cfg::ST];
  TileLoader<LB, Cfg::BN, Cfg::BK, Cfg::NT, VEC, ANone::Dev> b[Cfg::ST];
};

// CHAIN selects how the loop starts and ends:
//   CHAIN_NONE   a product on its own;
//   CHAIN_FIRST  another product of the same shape and layouts follows (operands A2, B2): its
//                first tiles are fetched where this one would fetch beyond K, so the second
//                product starts without waiting for memory. Needs a tile count that is a non-zero
//                multiple of Cfg::ST.
//   CHAIN_SECOND that following product: tile 0 is already in LDS stage 0 and tiles 1 .. ST-1 in
//                registers.
enum { CHAIN_NONE = 0, CHAIN_FIRST = 1, CHAIN_SECOND = 2 };

// Main loop: acc += A_tile(m0.., :) * B_tile(n0.., :)^T over the whole K range.
// Tile t is multiplied out of LDS stage t % 2 while tiles t+1 .. t+ST-1 are on their way in
// registers and tile t+ST is being requested: a tile has ST-1 multiply phases to arrive before
// it is written to LDS. One barrier per tile.
template <class Cfg, int LA, int LB, bool VEC, bool COLSUM, int CHAIN, class XfDev>
__device__ __forceinline__ void gemm_mainloop_chain(const float* __restrict__ A, int64_t lda,
                                                    const float* __restrict__ B, int64_t ldb, int M, int N, int K,
                                                    int m0, int n0, float* __restrict__ lds, XfDev& xf,
                                                    f32x16 (&acc)[Cfg::NACC], float (&asum)[Cfg::WTM],
                                                    TilePipe<Cfg, LA, LB, VEC, XfDev>& p,
                                                    const float* __restrict__ A2, const float* __restrict__ B2) {
  constexpr int BM = Cfg::BM, BK = Cfg::BK, ST = Cfg::ST;
  constexpr int A_FLOATS = lds_tile_floats<LA, BM, BK>();
  constexpr int STAGE = lds_stage_floats<Cfg, LA, LB>();

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wk = wave % Cfg::WK;
  const int wn = (wave / Cfg::WK) % Cfg::WN;
  const int wm = wave / (Cfg::WK * Cfg::WN);
  const int r = lane & 31, g = lane >> 5;

  const uint32_t bytes_a = LA == KCONTIG ? xf.extent(M, K, lda) : xf.extent(K, M, lda);
  const uint32_t bytes_b = LB == KCONTIG ? extent_bytes(N, K, ldb) : extent_bytes(K, N, ldb);
  const __amdgpu_buffer_rsrc_t ra = make_rsrc(A, bytes_a);
  const __amdgpu_buffer_rsrc_t rb = make_rsrc(B, bytes_b);
  const __amdgpu_buffer_rsrc_t ra2 = make_rsrc(CHAIN == CHAIN_FIRST ? A2 : A, bytes_a);
  const __amdgpu_buffer_rsrc_t rb2 = make_rsrc(CHAIN == CHAIN_FIRST ? B2 : B, bytes_b);
  const ANone::Dev none;

  const int nkt = (K + BK - 1) / BK;
  // Request tile `idx` into register slot `slot`. Tiles beyond K load as zeros without touching
  // memory, so no request needs a test; for the first product of a chain they are the next
  // product's tiles instead.
#define MW_REQUEST(slot, idx)                                                        \
  do {                                                                               \
    const int idx_ = (idx);                                                          \
    if (CHAIN == CHAIN_FIRST && idx_ >= nkt) {                                       \
      p.a[slot].load(ra2, lda, m0, (idx_ - nkt) * BK, M, K, xf);                     \
      p.b[slot].load(rb2, ldb, n0, (idx_ - nkt) * BK, N, K, none);                   \
    } else {                                                                         \
      p.a[slot].load(ra, lda, m0, idx_ * BK, M, K, xf);                              \
      p.b[slot].load(rb, ldb, n0, idx_ * BK, N, K, none);                            \
    }                                                                                \
    xf.template advance<LA, BK>();                                                   \
  } while (0)
#define MW_TO_LDS(slot, stage)                                  \
  do {                                                          \
    p.a[slot].store(lds + (stage) * STAGE, xf);                 \
    p.b[slot].store(lds + (stage) * STAGE + A_FLOATS, none);    \
  } while (0)
#define MW_MULTIPLY(stage) \
  mma_stage<Cfg, LA, LB, COLSUM>(lds + (stage) * STAGE, lds + (stage) * STAGE + A_FLOATS, wm, wn, wk, r, g, acc, asum)

  if (CHAIN != CHAIN_SECOND) {
    xf.template prepare<LA, BM, BK, Cfg::NT>(m0, M, K);
#pragma unroll
    for (int j = 0; j < ST; ++j) MW_REQUEST(j, j);
    MW_TO_LDS(0, 0);
    __syncthreads();
  }

  // ST tiles per trip with no exit between them; what is left of an uneven tile count is peeled
  // off after the loop. (An exit in the middle of the body makes the compiler assume, at the loop
  // head, that any of the requests may still be pending, and it then waits for all of them.)
  int t = 0;
  for (; t + ST <= nkt; t += ST) {
#pragma unroll
    for (int u = 0; u < ST; ++u) {
      // tile t+u is in LDS stage u % 2; slot u is free, slots u+1 .. hold the tiles after it
      MW_REQUEST(u, t + u + ST);
      MW_MULTIPLY(u % 2);
      MW_TO_LDS((u + 1) % ST, (u + 1) % 2);
      __syncthreads();
    }
  }
  const int rem = nkt - t;  // 0 .. ST-1 tiles left: tile t in stage 0, the others in slots 1 ..
#pragma unroll
  for (int u = 0; u < ST - 1; ++u) {
    if (u < rem) {
      MW_MULTIPLY(u % 2);
      if (u + 1 < rem) MW_TO_LDS(u + 1, (u + 1) % 2);
      __syncthreads();
    }
  }
#undef MW_REQUEST
#undef MW_TO_LDS
#undef MW_MULTIPLY
}

template <class Cfg, int LA, int LB, bool VEC, bool COLSUM, class XfDev>
__device__ __forceinline__ void gemm_mainloop(const float* __restrict__ A, int64_t lda, const float* __restrict__ B,
                                              int64_t ldb, int M, int N, int K, int m0, int n0,
                                              float* __restrict__ lds, XfDev& xf, f32x16 (&acc)[Cfg::NACC],
                                              float (&asum)[Cfg::WTM]) {
  TilePipe<Cfg, LA, LB, VEC, XfDev> p;
  gemm_mainloop_chain<Cfg, LA, LB, VEC, COLSUM, CHAIN_NONE>(A, lda, B, ldb, M, N, K, m0, n0, lds, xf, acc, asum, p,
                                                           nullptr, nullptr);
}

// The same product with the summation order of a tile whose K tile is KSETS times as wide and split over
// KSETS wavefronts (WK = KSETS): there wavefront w adds up the K slices w, w + KSETS, w + 2 KSETS, ... (32 wide
// each) and the KSETS sums are then added in the order 0, 1, 2, ... Here one wavefront owns the whole K range
// (Cfg::WK == 1) and walks it in that order: first every slice of set 0 into `acc`, then every slice of set 1,
// ...; a finished set is added to the running total `sum` (set 0 starts it). Every accumulator therefore sees the
// same sequence of matrix instructions on the same operand values as the split tile's, and the sums are added in
// the same order: the result has the same bits. (A larger tile with that property lets a product that must
// reproduce the split tile's bits -- the pre-activations of Phase III against Phase I -- run with more operand
// reuse. Walking the sets one after the other instead of keeping KSETS accumulators costs 16 registers, not
// 16 KSETS.) K must be a multiple of KSETS * ST * BK (the launcher checks); CHAIN as in gemm_mainloop_chain; the
// result is left in `sum`.
template <class Cfg, int LA, int LB, bool VEC, int KSETS, int CHAIN, class XfDev>
__device__ __forceinline__ void gemm_mainloop_sets(const float* __restrict__ A, int64_t lda, const float* __restrict__ B,
                                                   int64_t ldb, int M, int N, int K, int m0, int n0,
                                                   float* __restrict__ lds, XfDev& xf, f32x16 (&sum)[Cfg::NACC],
                                                   TilePipe<Cfg, LA, LB, VEC, XfDev>& p,
                                                   const float* __restrict__ A2, const float* __restrict__ B2) {
  static_assert(Cfg::WK == 1, "the walk over the sets stands in for the K split");
  static_assert(Cfg::ST == 2, "two tiles in flight");
  constexpr int BM = Cfg::BM, BK = Cfg::BK, ST = Cfg::ST;
  constexpr int A_FLOATS = lds_tile_floats<LA, BM, BK>();
  constexpr int STAGE = lds_stage_floats<Cfg, LA, LB>();

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wn = wave % Cfg::WN;
  const int wm = wave / Cfg::WN;
  const int r = lane & 31, g = lane >> 5;

  const uint32_t bytes_a = LA == KCONTIG ? xf.extent(M, K, lda) : xf.extent(K, M, lda);
  const uint32_t bytes_b = LB == KCONTIG ? extent_bytes(N, K, ldb) : extent_bytes(K, N, ldb);
  const __amdgpu_buffer_rsrc_t ra = make_rsrc(A, bytes_a);
  const __amdgpu_buffer_rsrc_t rb = make_rsrc(B, bytes_b);
  const __amdgpu_buffer_rsrc_t ra2 = make_rsrc(CHAIN == CHAIN_FIRST ? A2 : A, bytes_a);
  const __amdgpu_buffer_rsrc_t rb2 = make_rsrc(CHAIN == CHAIN_FIRST ? B2 : B, bytes_b);
  const ANone::Dev none;
  float unused[Cfg::WTM];

  const int per_set = K / (BK * KSETS);  // K tiles per set: a multiple of ST
  // the tile to request next: slice `rt` of set `rset` starts at k = (rt * KSETS + rset) * BK; past the last set
  // come the first tiles of the next product (CHAIN_FIRST) or nothing (loads beyond K return zeros untouched)
  int rt = 0, rset = 0;
#define MW_REQUEST(slot)                                                             \
  do {                                                                               \
    const int k0_ = (rt * KSETS + (rset < KSETS ? rset : 0)) * BK;                   \
    if (CHAIN == CHAIN_FIRST && rset >= KSETS) {                                     \
      p.a[slot].load(ra2, lda, m0, k0_, M, K, xf);                                   \
      p.b[slot].load(rb2, ldb, n0, k0_, N, K, none);                                 \
    } else {                                                                         \
      p.a[slot].load(ra, lda, m0, rset < KSETS ? k0_ : K, M, K, xf);                 \
      p.b[slot].load(rb, ldb, n0, rset < KSETS ? k0_ : K, N, K, none);               \
    }                                                                                \
    xf.template advance<LA, BK>();                                                   \
    if (++rt == per_set) {                                                           \
      rt = 0;                                                                        \
      ++rset;                                                                        \
    }                                                                                \
  } while (0)
#define MW_TO_LDS(slot, stage)                                  \
  do {                                                          \
    p.a[slot].store(lds + (stage) * STAGE, xf);                 \
    p.b[slot].store(lds + (stage) * STAGE + A_FLOATS, none);    \
  } while (0)

  if (CHAIN != CHAIN_SECOND) {
    xf.template prepare<LA, BM, BK, Cfg::NT>(m0, M, K);
#pragma unroll
    for (int j = 0; j < ST; ++j) MW_REQUEST(j);
    MW_TO_LDS(0, 0);
    __syncthreads();
  } else {
    rt = ST;  // tiles 0 .. ST-1 of this product were requested by the product before
    if (rt == per_set) {
      rt = 0;
      rset = 1;
    }
  }
  for (int set = 0; set < KSETS; ++set) {
    f32x16 acc[Cfg::NACC];
#pragma unroll
    for (int a = 0; a < Cfg::NACC; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;
    for (int t = 0; t < per_set; t += ST) {
#pragma unroll
      for (int u = 0; u < ST; ++u) {
        // the tile to multiply is in LDS stage u; register slot u is free, slot u ^ 1 holds the tile after it
        MW_REQUEST(u);
        mma_stage<Cfg, LA, LB, false>(lds + u * STAGE, lds + u * STAGE + A_FLOATS, wm, wn, 0, r, g, acc, unused);
        MW_TO_LDS(u ^ 1, u ^ 1);
        __syncthreads();
      }
    }
#pragma unroll
    for (int a = 0; a < Cfg::NACC; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) sum[a][i] = (set == 0) ? acc[a][i] : sum[a][i] + acc[a][i];
  }
#undef MW_REQUEST
#undef MW_TO_LDS
}

// Position of this lane's 16 accumulator values inside a 32x32 tile: value i sits in row
// 8*(i/4) + 4*(lane>>5) + i%4 and column lane & 31.
__device__ __forceinline__ int acc_row(int i, int g) { return 8 * (i / 4) + 4 * g + (i % 4); }

// Finish a workgroup tile: sum the K slices held by the WK wavefronts of each (wm, wn) position
// and hand the sums to the epilogue. With WK == 1 every wavefront passes its own registers.
// With WK > 1 all wavefronts park their accumulators in LDS (which must be free: main loop
// finished) and wavefront wk then owns registers [wk*16/WK, (wk+1)*16/WK) of every 32x32 tile:
// it adds the WK partial values in the fixed order wk = 0, 1, 2, ... and runs the epilogue for
// those rows, so the epilogue's stores are spread over all wavefronts.
// The epilogue is called by all 64 lanes together (it may use ballots):
//   epi.template part<CNT>(M, N, row_base, col, g, i0, v)   with v[NSETS][CNT] = values of
//   accumulator registers i0 .. i0+CNT-1 of the tile whose first row is row_base.
// asum (column sums of operand A, per lane) is reduced into the wk == 0 wavefront.
template <class Cfg, int NSETS, class Epi>
__device__ __forceinline__ void reduce_and_finish(float* __restrict__ lds, int M, int N, int m0, int n0,
                                                  const f32x16 (&acc)[NSETS][Cfg::NACC], float (&asum)[Cfg::WTM],
                                                  Epi& epi) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wk = wave % Cfg::WK;
  const int wn = (wave / Cfg::WK) % Cfg::WN;
  const int wm = wave / (Cfg::WK * Cfg::WN);
  const int g = lane >> 5;
  if (Cfg::WK == 1) {
#pragma unroll
    for (int tm = 0; tm < Cfg::WTM; ++tm)
#pragma unroll
      for (int tn = 0; tn < Cfg::WTN; ++tn) {
        float v[NSETS][16];
#pragma unroll
        for (int s = 0; s < NSETS; ++s)
#pragma unroll
          for (int i = 0; i < 16; ++i) v[s][i] = acc[s][tm * Cfg::WTN + tn][i];
        epi.template part<16>(M, N, m0 + (wm * Cfg::WTM + tm) * 32, n0 + (wn * Cfg::WTN + tn) * 32 + (lane & 31), g,
                              0, v);
      }
    return;
  }
  constexpr int CNT = 16 / Cfg::WK;                                   // registers per wavefront per tile
  static_assert(Cfg::WK == 1 || 16 % Cfg::WK == 0, "WK must divide 16");
  constexpr int PER_WAVE = (Cfg::NACC * 16 * NSETS + Cfg::WTM) * 64;  // floats parked per wavefront
  const int pos = wave / Cfg::WK;                                     // wm * WN + wn
  float* mine = lds + (pos * Cfg::WK + wk) * PER_WAVE;
#pragma unroll
  for (int s = 0; s < NSETS; ++s)
#pragma unroll
    for (int a = 0; a < Cfg::NACC; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) mine[((s * Cfg::NACC + a) * 16 + i) * 64 + lane] = acc[s][a][i];
#pragma unroll
  for (int tm = 0; tm < Cfg::WTM; ++tm) mine[(NSETS * Cfg::NACC * 16 + tm) * 64 + lane] = asum[tm];
  __syncthreads();
  const float* base = lds + pos * Cfg::WK * PER_WAVE;
  const int i0 = wk * CNT;
#pragma unroll
  for (int tm = 0; tm < Cfg::WTM; ++tm)
#pragma unroll
    for (int tn = 0; tn < Cfg::WTN; ++tn) {
      float v[NSETS][CNT];
#pragma unroll
      for (int s = 0; s < NSETS; ++s)
#pragma unroll
        for (int j = 0; j < CNT; ++j) {
          const int slot = ((s * Cfg::NACC + tm * Cfg::WTN + tn) * 16 + i0 + j) * 64 + lane;
          float t = base[slot];
          for (int w = 1; w < Cfg::WK; ++w) t += base[w * PER_WAVE + slot];
          v[s][j] = t;
        }
      epi.template part<CNT>(M, N, m0 + (wm * Cfg::WTM + tm) * 32, n0 + (wn * Cfg::WTN + tn) * 32 + (lane & 31), g,
                             i0, v);
    }
  if (wk == 0) {
#pragma unroll
    for (int tm = 0; tm < Cfg::WTM; ++tm) {
      float t = asum[tm];
      for (int w = 1; w < Cfg::WK; ++w) t += base[w * PER_WAVE + (NSETS * Cfg::NACC * 16 + tm) * 64 + lane];
      asum[tm] = t;
    }
  }
}

// Logical tile coordinates of workgroup `bid` of a grid of tiles_m * tiles_n: XCD-aware, m fastest
// (all row tiles of one column panel of B land on the same XCD, so B is fetched from HBM once).
// `bid` is the block id within the task; when a launch carries two tasks the first one's block
// count is padded to a multiple of 8 so that bid % 8 is still the XCD the block runs on.
__device__ __forceinline__ void tile_coords(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
  int id = xcd_remap(bid, tiles_m * tiles_n);
  tm = id % tiles_m;
  tn = id / tiles_m;
}

}  // namespace mw
