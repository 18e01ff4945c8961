// fp32 MFMA GEMM building blocks for gfx950 (CDNA4), wave64.
//
// One workgroup = 4 wavefronts arranged WM x WN x WK. Each wavefront owns WTM x WTN output
// tiles of 32x32 (v_mfma_f32_32x32x2_f32) and, when WK > 1, one slice of every K tile; the
// K slices are summed through LDS in a fixed order, so results are bit-identical run to run.
// Operand tiles are staged through double-buffered LDS with one barrier per K tile; the next
// tile's global loads are in flight while the current one is multiplied.
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

constexpr int KCONTIG = 0;
constexpr int RCONTIG = 1;
constexpr int NUM_XCD = 8;

template <int WTM_, int WTN_, int WM_, int WN_, int WK_>
struct TileCfg {
  static constexpr int WTM = WTM_, WTN = WTN_, WM = WM_, WN = WN_, WK = WK_;
  static constexpr int BM = 32 * WTM * WM;
  static constexpr int BN = 32 * WTN * WN;
  static constexpr int BK = 32 * WK;            // every wavefront consumes 32 k per K tile
  static constexpr int NT = 64 * WM * WN * WK;  // threads per workgroup
  static constexpr int NACC = WTM * WTN;        // 32x32 accumulator tiles per wavefront
};
using Tile128 = TileCfg<2, 2, 2, 2, 1>;   // 128 x 128, K tile 32
using Tile64 = TileCfg<1, 1, 2, 2, 1>;    //  64 x  64, K tile 32
using Tile32K4 = TileCfg<1, 1, 1, 1, 4>;  //  32 x  32, K tile 128 split over 4 wavefronts

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
  int red = (Cfg::WK - 1) * Cfg::WM * Cfg::WN * (Cfg::NACC * 16 * NSETS + Cfg::WTM) * 64;
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
// Guarded 4-wide global load. The 4 elements are (outer, inner .. inner+3) of a matrix whose
// fast index is `inner`: address p[outer * ld + inner]. Out-of-range elements read as 0.
// `vec_ok` (wave-uniform) says that p is 16-byte aligned and ld % 4 == 0, so that a chunk that
// starts at a multiple of 4 and lies inside the matrix can be fetched with one dwordx4 load.
__device__ __forceinline__ float4 load4(const float* __restrict__ p, int64_t ld, int outer, int inner,
                                        int n_outer, int n_inner, bool vec_ok) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (outer < n_outer && inner < n_inner) {
    const float* q = p + (int64_t)outer * ld + inner;
    if (vec_ok && inner + 3 < n_inner) {
      v = *reinterpret_cast<const float4*>(q);
    } else {
      v.x = q[0];
      if (inner + 1 < n_inner) v.y = q[1];
      if (inner + 2 < n_inner) v.z = q[2];
      if (inner + 3 < n_inner) v.w = q[3];
    }
  }
  return v;
}

__device__ __forceinline__ bool vec_ok_for(const void* p, int64_t ld) {
  return ((reinterpret_cast<uintptr_t>(p) & 15) == 0) && ((ld & 3) == 0);
}

// ---------------------------------------------------------------------------------------------
// Operand-A transforms. A transform has two halves so that the global loads of a tile stay in
// flight while the previous tile is multiplied: fetch() issues whatever extra loads it needs
// next to the operand's own load, apply() runs just before the values are written to LDS.
// The 4 values are (outer, inner .. inner+3) at flat offset outer * ld + inner; elements beyond
// the matrix edge hold 0 already.

struct ANone {
  struct Aux {};
  __device__ __forceinline__ void fetch(Aux&, int64_t, int, int, int, int, bool) const {}
  __device__ __forceinline__ float4 apply(float4 v, const Aux&) const { return v; }
};

// Multiply by the activation slope taken from packed sign bits: bit e of the mask (LSB-first,
// flat index e = outer * ld + inner of the full tensor) selects 1, a cleared bit selects alpha.
struct ASlopeFromMask {
  const uint32_t* mask32;  // the uint64 words seen as little-endian halves
  float alpha;
  struct Aux { uint32_t bits; };
  __device__ __forceinline__ void fetch(Aux& aux, int64_t ld, int outer, int inner, int n_outer, int n_inner,
                                        bool) const {
    aux.bits = 0;
    if (outer < n_outer && inner < n_inner) {
      int64_t e = (int64_t)outer * ld + inner;
      uint64_t lo = mask32[e >> 5];
      int sh = (int)(e & 31);
      // the 4 bits straddle two 32-bit halves only when ld is not a multiple of 4; the second
      // half is read only if an element of this row lives there (so it is inside the mask)
      if (sh > 28 && inner + (32 - sh) < n_inner) lo |= (uint64_t)mask32[(e >> 5) + 1] << 32;
      aux.bits = (uint32_t)(lo >> sh);
    }
  }
  __device__ __forceinline__ float4 apply(float4 v, const Aux& aux) const {
    v.x *= (aux.bits & 1u) ? 1.f : alpha;
    v.y *= (aux.bits & 2u) ? 1.f : alpha;
    v.z *= (aux.bits & 4u) ? 1.f : alpha;
    v.w *= (aux.bits & 8u) ? 1.f : alpha;
    return v;
  }
};

// Multiply by the activation slope taken from the stored activation itself: x > 0 <=> z > 0.
struct ASlopeFromAct {
  const float* act;  // same shape and row stride as A
  float alpha;
  struct Aux { float4 a; };
  __device__ __forceinline__ void fetch(Aux& aux, int64_t ld, int outer, int inner, int n_outer, int n_inner,
                                        bool vec_ok) const {
    aux.a = load4(act, ld, outer, inner, n_outer, n_inner, vec_ok && vec_ok_for(act, ld));
  }
  __device__ __forceinline__ float4 apply(float4 v, const Aux& aux) const {
    v.x *= (aux.a.x > 0.f) ? 1.f : alpha;
    v.y *= (aux.a.y > 0.f) ? 1.f : alpha;
    v.z *= (aux.a.z > 0.f) ? 1.f : alpha;
    v.w *= (aux.a.w > 0.f) ? 1.f : alpha;
    return v;
  }
};

// ---------------------------------------------------------------------------------------------
// Global -> register -> LDS staging of one operand tile (R rows x BK k).

template <int LAYOUT, int R, int BK, int NT, class Xf>
struct TileLoader {
  static constexpr int NV = R * BK / 4 / NT;  // float4 per thread
  static_assert(R * BK % (4 * NT) == 0, "tile must divide evenly over the workgroup");
  float4 v[NV];
  typename Xf::Aux aux[NV];

  __device__ __forceinline__ void load(const float* __restrict__ p, int64_t ld, int row0, int k0, int n_rows,
                                       int n_k, bool vec_ok, const Xf& xf) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int f = (int)threadIdx.x + i * NT;
      if (LAYOUT == KCONTIG) {
        int r = f / (BK / 4), c4 = f % (BK / 4);
        v[i] = load4(p, ld, row0 + r, k0 + 4 * c4, n_rows, n_k, vec_ok);
        xf.fetch(aux[i], ld, row0 + r, k0 + 4 * c4, n_rows, n_k, vec_ok);
      } else {
        int k = f / (R / 4), r4 = f % (R / 4);
        v[i] = load4(p, ld, k0 + k, row0 + 4 * r4, n_k, n_rows, vec_ok);
        xf.fetch(aux[i], ld, k0 + k, row0 + 4 * r4, n_k, n_rows, vec_ok);
      }
    }
  }

  __device__ __forceinline__ void store(float* __restrict__ lds, const Xf& xf) const {
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

// ---------------------------------------------------------------------------------------------
// Main loop: acc += A_tile(m0.., :) * B_tile(n0.., :)^T over the whole K range.
// Must be entered by the whole workgroup; ends with a barrier, so LDS may be reused afterwards.
// If COLSUM, asum[tm] accumulates, per lane, the sum of the A values that lane fed to the MFMA
// (after the A transform); combined over lanes/waves by the caller into column sums of A.

template <class Cfg, int LA, int LB, bool COLSUM, class Xf>
__device__ __forceinline__ void gemm_mainloop(const float* __restrict__ A, int64_t lda, const float* __restrict__ B,
                                              int64_t ldb, int M, int N, int K, int m0, int n0,
                                              float* __restrict__ lds, const Xf& xf, f32x16 (&acc)[Cfg::NACC],
                                              float (&asum)[Cfg::WTM]) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK;
  constexpr int A_FLOATS = lds_tile_floats<LA, BM, BK>();
  constexpr int STAGE = lds_stage_floats<Cfg, LA, LB>();

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wk = wave % Cfg::WK;
  const int wn = (wave / Cfg::WK) % Cfg::WN;
  const int wm = wave / (Cfg::WK * Cfg::WN);
  const int r = lane & 31, g = lane >> 5;

  const bool a_vec = vec_ok_for(A, lda), b_vec = vec_ok_for(B, ldb);

  TileLoader<LA, BM, BK, Cfg::NT, Xf> la;
  TileLoader<LB, BN, BK, Cfg::NT, ANone> lb;
  const ANone none{};

  const int nkt = (K + BK - 1) / BK;
  la.load(A, lda, m0, 0, M, K, a_vec, xf);
  lb.load(B, ldb, n0, 0, N, K, b_vec, none);
  la.store(lds, xf);
  lb.store(lds + A_FLOATS, none);
  __syncthreads();

  for (int t = 0; t < nkt; ++t) {
    const float* sa = lds + (t & 1) * STAGE;
    const float* sb = sa + A_FLOATS;
    const bool more = (t + 1 < nkt);
    if (more) {
      la.load(A, lda, m0, (t + 1) * BK, M, K, a_vec, xf);
      lb.load(B, ldb, n0, (t + 1) * BK, N, K, b_vec, none);
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int kbase = 32 * wk + 16 * g + 8 * half;
      float fa[Cfg::WTM][8], fb[Cfg::WTN][8];
#pragma unroll
      for (int tm = 0; tm < Cfg::WTM; ++tm)
        read_frag8<LA, BM, BK>(sa, (wm * Cfg::WTM + tm) * 32 + r, kbase, fa[tm]);
#pragma unroll
      for (int tn = 0; tn < Cfg::WTN; ++tn)
        read_frag8<LB, BN, BK>(sb, (wn * Cfg::WTN + tn) * 32 + r, kbase, fb[tn]);
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
    if (more) {
      float* da = lds + ((t + 1) & 1) * STAGE;
      la.store(da, xf);
      lb.store(da + A_FLOATS, none);
    }
    __syncthreads();
  }
}

// Sum the K slices held by the WK wavefronts of each (wm, wn) position into the wk == 0
// wavefront, in the fixed order wk = 1, 2, ... . LDS must be free (main loop finished).
// Returns true for the wavefronts that hold the result (wk == 0).
template <class Cfg, int NSETS>
__device__ __forceinline__ bool reduce_k_slices(float* __restrict__ lds, f32x16 (&acc)[NSETS][Cfg::NACC],
                                                float (&asum)[Cfg::WTM]) {
  if (Cfg::WK == 1) return true;
  constexpr int PER_WAVE = (Cfg::NACC * 16 * NSETS + Cfg::WTM) * 64;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wk = wave % Cfg::WK;
  const int pos = wave / Cfg::WK;  // wm * WN + wn
  if (wk > 0) {
    float* dst = lds + ((wk - 1) * Cfg::WM * Cfg::WN + pos) * PER_WAVE;
#pragma unroll
    for (int s = 0; s < NSETS; ++s)
#pragma unroll
      for (int a = 0; a < Cfg::NACC; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) dst[((s * Cfg::NACC + a) * 16 + i) * 64 + lane] = acc[s][a][i];
#pragma unroll
    for (int tm = 0; tm < Cfg::WTM; ++tm) dst[(NSETS * Cfg::NACC * 16 + tm) * 64 + lane] = asum[tm];
  }
  __syncthreads();
  if (wk > 0) return false;
  for (int w = 1; w < Cfg::WK; ++w) {
    const float* src = lds + ((w - 1) * Cfg::WM * Cfg::WN + pos) * PER_WAVE;
#pragma unroll
    for (int s = 0; s < NSETS; ++s)
#pragma unroll
      for (int a = 0; a < Cfg::NACC; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[s][a][i] += src[((s * Cfg::NACC + a) * 16 + i) * 64 + lane];
#pragma unroll
    for (int tm = 0; tm < Cfg::WTM; ++tm) asum[tm] += src[(NSETS * Cfg::NACC * 16 + tm) * 64 + lane];
  }
  return true;
}

// Walk the accumulator registers of this wavefront and hand every element to the epilogue.
// Output element of accumulator register i of a 32x32 tile: row 8*(i/4) + 4*(lane>>5) + i%4,
// column lane & 31. The epilogue is called by all 64 lanes together (it may use ballots):
//   epi(row, col, valid, v[NSETS])
template <class Cfg, int NSETS, class Epi>
__device__ __forceinline__ void for_each_output(int M, int N, int m0, int n0, const f32x16 (&acc)[NSETS][Cfg::NACC],
                                                Epi& epi) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wn = (wave / Cfg::WK) % Cfg::WN;
  const int wm = wave / (Cfg::WK * Cfg::WN);
#pragma unroll
  for (int tm = 0; tm < Cfg::WTM; ++tm)
#pragma unroll
    for (int tn = 0; tn < Cfg::WTN; ++tn)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        int row = m0 + (wm * Cfg::WTM + tm) * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i % 4);
        int col = n0 + (wn * Cfg::WTN + tn) * 32 + (lane & 31);
        float v[NSETS];
#pragma unroll
        for (int s = 0; s < NSETS; ++s) v[s] = acc[s][tm * Cfg::WTN + tn][i];
        epi(row, col, row < M && col < N, v);
      }
}

// Logical tile coordinates of this workgroup: XCD-aware, m fastest (all row tiles of one
// column panel of B land on the same XCD, so B is fetched from HBM once).
__device__ __forceinline__ void tile_coords(int tiles_m, int tiles_n, int& tm, int& tn) {
  int id = xcd_remap((int)blockIdx.x, tiles_m * tiles_n);
  tm = id % tiles_m;
  tn = id / tiles_m;
}

}  // namespace mw
