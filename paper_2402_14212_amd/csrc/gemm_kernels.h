// Kernels and epilogues built on gemm_f32.h, and their host-side launch helpers.
//
// Epilogues are branch-free: every global access is a buffer access whose offset is OOB for
// lanes that fall outside the matrix, and all loads of a 32x32 tile are issued before the first
// use, so the memory latency of an epilogue is paid once per tile, not once per element.
#pragma once

#include "gemm_f32.h"

namespace mw {

// ------------------------------------------------------------------------------------ epilogues
// Each epilogue is a plain parameter struct (a kernel argument) with a device-side state `Dev`
// built inside the kernel. Dev::part<CNT>() receives CNT consecutive accumulator registers
// i0 .. i0+CNT-1 of one 32x32 tile for this lane (see acc_row for their rows).

// C = alpha * acc (+ bias[col]) (+ beta * C)
struct EpiStore {
  float* C;
  int64_t ldc;
  float alpha, beta;
  const float* bias;
  struct Dev;
};
struct EpiStore::Dev {
  __amdgpu_buffer_rsrc_t rc, rbias;
  int64_t ldc;
  float alpha, beta;
  bool bias;
  __device__ __forceinline__ Dev(const EpiStore& p, int M, int N)
      : ldc(p.ldc), alpha(p.alpha), beta(p.beta), bias(p.bias != nullptr) {
    rc = make_rsrc(p.C, extent_bytes(M, N, p.ldc));
    rbias = make_rsrc(p.bias, p.bias ? (uint32_t)N * 4u : 0u);
  }
  __device__ __forceinline__ void finish() const {}
  template <int CNT>
  __device__ __forceinline__ void part(int M, int N, int row_base, int col, int g, int i0,
                                       const float (&v)[1][CNT]) const {
    const bool cv = col < N;
    const float bv = buf_load_f32(rbias, (bias && cv) ? (uint32_t)col * 4u : OOB);
    uint32_t off[CNT];
    float old[CNT];
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
      int row = row_base + acc_row(i0 + j, g);
      off[j] = (cv && row < M) ? ((uint32_t)row * (uint32_t)ldc + (uint32_t)col) * 4u : OOB;
    }
    if (beta != 0.f) {
#pragma unroll
      for (int j = 0; j < CNT; ++j) old[j] = buf_load_f32(rc, off[j]);
    }
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
      float r = alpha * v[0][j];
      if (bias) r += bv;
      if (beta != 0.f) r += beta * old[j];
      buf_store_f32(rc, off[j], r);
    }
  }
};

// C = alpha * acc + beta * D + eye * I: D is another matrix of C's shape and row stride (or C itself, or NULL)
struct EpiAxpby {
  float* C;
  const float* D;
  int64_t ldc;
  float alpha, beta;
  float eye = 0.f;
  struct Dev {
    __amdgpu_buffer_rsrc_t rc, rd;
    int64_t ldc;
    float alpha, beta, eye;
    bool add;
    __device__ __forceinline__ Dev(const EpiAxpby& p, int M, int N)
        : ldc(p.ldc), alpha(p.alpha), beta(p.beta), eye(p.eye), add(p.D != nullptr && p.beta != 0.f) {
      rc = make_rsrc(p.C, extent_bytes(M, N, p.ldc));
      rd = make_rsrc(p.D, add ? extent_bytes(M, N, p.ldc) : 0u);
    }
    __device__ __forceinline__ void finish() const {}
    template <int CNT>
    __device__ __forceinline__ void part(int M, int N, int row_base, int col, int g, int i0,
                                         const float (&v)[1][CNT]) const {
      uint32_t off[CNT];
      float old[CNT];
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        const int row = row_base + acc_row(i0 + j, g);
        off[j] = (col < N && row < M) ? ((uint32_t)row * (uint32_t)ldc + (uint32_t)col) * 4u : OOB;
        old[j] = buf_load_f32(rd, add ? off[j] : OOB);
      }
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        float r = alpha * v[0][j] + (add ? beta * old[j] : 0.f);
        if (eye != 0.f && row_base + acc_row(i0 + j, g) == col) r += eye;
        buf_store_f32(rc, off[j], r);
      }
    }
  };
};

// Phase-I forward epilogue: z = acc + b, m = (z > 0), x = m ? z : alpha z. With MASK the 32
// sign bits each half-wavefront holds for one output row go out as one 32-bit half of a packed
// mask word (requires N % 32 == 0; the launcher checks).
template <bool MASK>
struct EpiFwdAct {
  float* X;
  const float* bias;
  float alpha;
  uint32_t* mask32;
  float* Z = nullptr;  // debugging aid: the pre-activations themselves, [M][N]; NULL (the normal case): not kept
  struct Dev {
    __amdgpu_buffer_rsrc_t rx, rbias, rmask, rz;
    float alpha;
    bool bias, keep_z;
    __device__ __forceinline__ Dev(const EpiFwdAct& p, int M, int N)
        : alpha(p.alpha), bias(p.bias != nullptr), keep_z(p.Z != nullptr) {
      rx = make_rsrc(p.X, extent_bytes(M, N, N));
      rbias = make_rsrc(p.bias, p.bias ? (uint32_t)N * 4u : 0u);
      rmask = make_rsrc(p.mask32, MASK ? (uint32_t)(((int64_t)M * N + 63) / 64) * 8u : 0u);
      rz = make_rsrc(p.Z, p.Z ? extent_bytes(M, N, N) : 0u);
    }
    __device__ __forceinline__ void finish() const {}
    template <int CNT>
    __device__ __forceinline__ void part(int M, int N, int row_base, int col, int g, int i0,
                                         const float (&v)[1][CNT]) const {
      const bool cv = col < N;
      const float bv = buf_load_f32(rbias, (bias && cv) ? (uint32_t)col * 4u : OOB);
      const int lane = threadIdx.x & 63;
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        int row = row_base + acc_row(i0 + j, g);
        bool valid = cv && row < M;
        uint32_t e = (uint32_t)row * (uint32_t)N + (uint32_t)col;
        float z = v[0][j];
        if (bias) z += bv;
        bool bit = valid && (z > 0.f);
        buf_store_f32(rx, valid ? e * 4u : OOB, bit ? z : alpha * z);
        if (keep_z) buf_store_f32(rz, valid ? e * 4u : OOB, z);  // uniform branch: nothing is issued normally
        if (MASK) {
          unsigned long long bal = __ballot(bit);
          uint32_t word = g ? (uint32_t)(bal >> 32) : (uint32_t)bal;
          buf_store_u32(rmask, ((lane & 31) == 0 && valid) ? (e >> 5) * 4u : OOB, word);
        }
      }
    }
  };
};

// Phase-III epilogue for one layer. v[0] = x_{i-1} W^T (pre-bias), v[1] = h_{i-1} P^T.
//   leaky: m = (z > 0) recomputed; h_y = m ? ct_z : ct_z * (1/alpha).
//   ReLU : m = stored bit; ct_z zeroed where erased; h_y restored from the fragment store at
//          rank = offsets[word] + popcount(erased bits below e in the 64-bit word).
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
  unsigned long long* mismatches;
  struct Dev {
    __amdgpu_buffer_rsrc_t rbias, rmask, roff, rfrag, rx, rh, rc;
    float alpha, inv_alpha;
    bool bias;
    unsigned long long* mismatches;
    uint32_t mism;
    __device__ __forceinline__ Dev(const EpiVijp& p, int M, int N)
        : alpha(p.alpha), inv_alpha(p.inv_alpha), bias(p.bias != nullptr), mismatches(p.mismatches), mism(0) {
      const uint32_t words = (uint32_t)(((int64_t)M * N + 63) / 64);
      rbias = make_rsrc(p.bias, p.bias ? (uint32_t)N * 4u : 0u);
      rmask = make_rsrc(p.mask, words * 8u);
      roff = make_rsrc(p.offsets, RELU ? (words + 1u) * 4u : 0u);
      uint64_t base = RELU ? *p.frag_base : 0ull;
      // the layer's slice of the store; reads past the capacity return 0
      uint64_t room = (RELU && base < p.frag_capacity) ? p.frag_capacity - base : 0ull;
      if (room > 0x1FFFFFFFull) room = 0x1FFFFFFFull;
      rfrag = make_rsrc(RELU ? p.frag + base : nullptr, (uint32_t)room * 4u);
      rx = make_rsrc(p.X, extent_bytes(M, N, N));
      rh = make_rsrc(p.H, extent_bytes(M, N, N));
      rc = make_rsrc(p.CTZ, p.CTZ ? extent_bytes(M, N, N) : 0u);  // NULL: ct_z is not written (stores dropped)
    }
    template <int CNT>
    __device__ __forceinline__ void part(int M, int N, int row_base, int col, int g, int i0,
                                         const float (&v)[2][CNT]) {
      const bool cv = col < N;
      const float bv = buf_load_f32(rbias, (bias && cv) ? (uint32_t)col * 4u : OOB);
      uint32_t e[CNT], lo[CNT], hi[CNT], rank0[CNT];
      bool valid[CNT];
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        int row = row_base + acc_row(i0 + j, g);
        valid[j] = cv && row < M;
        e[j] = (uint32_t)row * (uint32_t)N + (uint32_t)col;
        uint32_t w = e[j] >> 6;
        if (RELU) {
          lo[j] = buf_load_u32(rmask, valid[j] ? w * 8u : OOB);
          hi[j] = buf_load_u32(rmask, valid[j] ? w * 8u + 4u : OOB);
          rank0[j] = buf_load_u32(roff, valid[j] ? w * 4u : OOB);
        } else {
          lo[j] = buf_load_u32(rmask, valid[j] ? (e[j] >> 5) * 4u : OOB);
        }
      }
      float restored[CNT];
      bool stored[CNT];
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        if (RELU) {
          uint64_t w = ((uint64_t)hi[j] << 32) | lo[j];
          uint32_t sh = e[j] & 63u;
          stored[j] = (w >> sh) & 1ull;
          uint32_t idx = rank0[j] + (uint32_t)__popcll(~w & ((1ull << sh) - 1ull));
          restored[j] = buf_load_f32(rfrag, (valid[j] && !stored[j]) ? idx * 4u : OOB);
        } else {
          stored[j] = (lo[j] >> (e[j] & 31u)) & 1u;
        }
      }
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        float z = v[0][j];
        if (bias) z += bv;
        const bool fresh = z > 0.f;
        if (valid[j] && fresh != stored[j]) ++mism;
        const uint32_t off = valid[j] ? e[j] * 4u : OOB;
        if (RELU) {
          const float c = stored[j] ? v[1][j] : 0.f;
          buf_store_f32(rx, off, stored[j] ? z : alpha * z);
          buf_store_f32(rh, off, stored[j] ? c : restored[j]);
          buf_store_f32(rc, off, c);
        } else {
          const float c = v[1][j];
          buf_store_f32(rx, off, fresh ? z : alpha * z);
          buf_store_f32(rh, off, fresh ? c : c * inv_alpha);
          buf_store_f32(rc, off, c);
        }
      }
    }
    __device__ __forceinline__ void finish() const {
      if (mism) atomicAdd(mismatches, (unsigned long long)mism);
    }
  };
};

// The leaky Phase-III epilogue for a layer whose ct_z is already in memory (rebuilt from fragments):
// the product is x_{i-1} W^T only, ct_z is read instead of computed, and not written back.
struct EpiVijpGiven {
  EpiVijp<false> inner;  // inner.CTZ must be NULL
  const float* CT;       // [M][N]
  struct Dev {
    EpiVijp<false>::Dev d;
    __amdgpu_buffer_rsrc_t rct;
    __device__ __forceinline__ Dev(const EpiVijpGiven& p, int M, int N) : d(p.inner, M, N) {
      rct = make_rsrc(p.CT, extent_bytes(M, N, N));
    }
    template <int CNT>
    __device__ __forceinline__ void part(int M, int N, int row_base, int col, int g, int i0, const float (&v)[1][CNT]) {
      float w[2][CNT];
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        const int row = row_base + acc_row(i0 + j, g);
        const bool valid = col < N && row < M;
        w[0][j] = v[0][j];
        w[1][j] = buf_load_f32(rct, valid ? ((uint32_t)row * (uint32_t)N + (uint32_t)col) * 4u : OOB);
      }
      d.template part<CNT>(M, N, row_base, col, g, i0, w);
    }
    __device__ __forceinline__ void finish() const { d.finish(); }
  };
};

// Phase-II epilogue. The product is h, the cotangent at the OUTPUT of the previous layer. It is
// scaled by that layer's activation slope here (bit ? 1 : alpha, bits from its packed mask), so the
// next reverse product consumes ct_z directly; the unscaled h is also kept where a re-seed
// checkpoint is due, and for a ReLU previous layer the erased entries of h go to the fragment
// store at rank = offsets[word] + popcount(erased bits below e in the word).
template <bool RELU>
struct EpiRevSlope {
  float* CT;                  // [M][N] slope-scaled cotangent
  float* RAW;                 // [M][N] unscaled cotangent (checkpoint) or NULL
  const uint64_t* mask;       // previous layer's signs, flat index row * N + col
  float alpha;                // previous layer's slope
  const uint32_t* offsets;    // ReLU only
  float* frag;                // ReLU only: start of the whole store
  const uint64_t* frag_base;  // ReLU only: device scalar
  uint64_t frag_capacity;
  int32_t* overflow;          // ReLU only: raised when the store is too small
  struct Dev {
    __amdgpu_buffer_rsrc_t rct, rraw, rmask, roff, rfrag;
    float alpha;
    bool raw;
    uint32_t room;
    int32_t* overflow;
    bool ovf;
    __device__ __forceinline__ Dev(const EpiRevSlope& p, int M, int N)
        : alpha(p.alpha), raw(p.RAW != nullptr), overflow(p.overflow), ovf(false) {
      const uint32_t words = (uint32_t)(((int64_t)M * N + 63) / 64);
      rct = make_rsrc(p.CT, extent_bytes(M, N, N));
      rraw = make_rsrc(p.RAW, p.RAW ? extent_bytes(M, N, N) : 0u);
      rmask = make_rsrc(p.mask, words * 8u);
      roff = make_rsrc(p.offsets, RELU ? (words + 1u) * 4u : 0u);
      uint64_t base = RELU ? *p.frag_base : 0ull;
      uint64_t left = (RELU && base < p.frag_capacity) ? p.frag_capacity - base : 0ull;
      if (left > 0x1FFFFFFFull) left = 0x1FFFFFFFull;
      room = (uint32_t)left;
      rfrag = make_rsrc(RELU ? p.frag + base : nullptr, room * 4u);  // stores past the room are dropped
    }
    template <int CNT>
    __device__ __forceinline__ void part(int M, int N, int row_base, int col, int g, int i0,
                                         const float (&v)[1][CNT]) {
      const bool cv = col < N;
      uint32_t e[CNT], lo[CNT], hi[CNT], rank0[CNT];
      bool valid[CNT];
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        int row = row_base + acc_row(i0 + j, g);
        valid[j] = cv && row < M;
        e[j] = (uint32_t)row * (uint32_t)N + (uint32_t)col;
        if (RELU) {
          uint32_t w = e[j] >> 6;
          lo[j] = buf_load_u32(rmask, valid[j] ? w * 8u : OOB);
          hi[j] = buf_load_u32(rmask, valid[j] ? w * 8u + 4u : OOB);
          rank0[j] = buf_load_u32(roff, valid[j] ? w * 4u : OOB);
        } else {
          lo[j] = buf_load_u32(rmask, valid[j] ? (e[j] >> 5) * 4u : OOB);
        }
      }
#pragma unroll
      for (int j = 0; j < CNT; ++j) {
        const uint32_t off = valid[j] ? e[j] * 4u : OOB;
        const float h = v[0][j];
        bool bit;
        if (RELU) {
          uint64_t w = ((uint64_t)hi[j] << 32) | lo[j];
          uint32_t sh = e[j] & 63u;
          bit = (w >> sh) & 1ull;
          uint32_t idx = rank0[j] + (uint32_t)__popcll(~w & ((1ull << sh) - 1ull));
          const bool erased = valid[j] && !bit;
          if (erased && idx >= room) ovf = true;
          buf_store_f32(rfrag, erased ? idx * 4u : OOB, h);
        } else {
          bit = (lo[j] >> (e[j] & 31u)) & 1u;
        }
        buf_store_f32(rct, off, h * (bit ? 1.f : alpha));
        if (raw) buf_store_f32(rraw, off, h);
      }
    }
    __device__ __forceinline__ void finish() const {
      if (RELU && ovf) *overflow = 1;
    }
  };
};

// ------------------------------------------------------------------------------------ kernels
// Work descriptions ("tasks") are plain structs passed as kernel arguments; a task's run() is
// the whole life of one workgroup. A launch carries one task, or two independent ones.

template <class Cfg, int LA, int LB, bool VEC, class Xf, class Epi, bool COLSUM>
struct GemmTask {
  int M, N, K;
  const float* A;
  int64_t lda;
  const float* B;
  int64_t ldb;
  Xf xf;
  Epi epi;
  float* colsum_out;
  float colsum_scale;
  int tiles_m, tiles_n;
  float colsum_beta = 0.f;  // colsum_out = colsum_scale * sums + colsum_beta * colsum_out
  static constexpr int LDS_BYTES = lds_bytes<Cfg, LA, LB, 1>();
  __host__ __device__ int blocks() const { return tiles_m * tiles_n; }

  __device__ __forceinline__ void run(int bid, float* __restrict__ lds) const {
    int tm_i, tn_i;
    tile_coords(bid, tiles_m, tiles_n, tm_i, tn_i);
    run_tile(tm_i, tn_i, lds);
  }

  __device__ __forceinline__ void run_tile(int tm_i, int tn_i, float* __restrict__ lds) const {
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
      typename Xf::Dev xd(xf, LA == KCONTIG ? M : K, LA == KCONTIG ? K : M, lda);
      gemm_mainloop<Cfg, LA, LB, VEC, COLSUM>(A, lda, B, ldb, M, N, K, m0, n0, lds, xd, acc[0], asum);
    }
    if (COLSUM) {
#pragma unroll
      for (int t = 0; t < Cfg::WTM; ++t) asum[t] += __shfl_xor(asum[t], 32);
    }
    typename Epi::Dev ed(epi, M, N);
    reduce_and_finish<Cfg, 1>(lds, M, N, m0, n0, acc, asum, ed);
    ed.finish();

    if (COLSUM && n0 == 0 && colsum_out) {
      const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
      const int wk = wave % Cfg::WK, wn = (wave / Cfg::WK) % Cfg::WN, wm = wave / (Cfg::WK * Cfg::WN);
      if (wk == 0 && wn == 0 && lane < 32) {
#pragma unroll
        for (int t = 0; t < Cfg::WTM; ++t) {
          int row = m0 + (wm * Cfg::WTM + t) * 32 + lane;
          if (row < M) {
            float v = colsum_scale * asum[t];
            if (colsum_beta != 0.f) v += colsum_beta * colsum_out[row];
            colsum_out[row] = v;
          }
        }
      }
    }
  }
};

// The same product for several independent operand sets of one shape, in one grid: set g takes
// A[g], B[g], D[g] and writes C[g] (pointer tables in device memory). Small products that would
// leave the chip half empty one at a time fill it together, with the tile a large product takes.
template <class Cfg, int LA, int LB>
struct GroupedGemmTask {
  int n_sets, M, N, K;
  const float* const* A;
  int64_t lda;
  const float* const* B;
  int64_t ldb;
  float* const* C;
  const float* const* D;  // may be NULL: no addend
  int64_t ldc;
  float alpha, beta;
  int tiles_m, tiles_n;
  float eye = 0.f;  // C[g] += eye * I
  using One = GemmTask<Cfg, LA, LB, true, ANone, EpiAxpby, false>;
  static constexpr int LDS_BYTES = One::LDS_BYTES;
  __host__ __device__ int blocks() const { return n_sets * tiles_m * tiles_n; }

  __device__ __forceinline__ void run(int bid, float* __restrict__ lds) const {
    const int per = tiles_m * tiles_n;
    const int g = bid / per;
    const One t{M, N, K, A[g], lda, B[g], ldb, ANone{}, EpiAxpby{C[g], D ? D[g] : nullptr, ldc, alpha, beta, eye},
                nullptr, 0.f, tiles_m, tiles_n};
    t.run(bid - g * per, lds);
  }
};

// One layer of the phase-III sweep: both NT products for the same output tile, then EpiVijp.
//   acc0 = X[M][K] W[N][K]^T ,  acc1 = Hin[M][K] P[N][K]^T
template <class Cfg, bool VEC, bool RELU>
struct VijpTask {
  int M, N, K;
  const float* X;
  const float* W;
  const float* Hin;
  const float* P;
  EpiVijp<RELU> epi;
  int tiles_m, tiles_n;
  static constexpr int LDS_BYTES = lds_bytes<Cfg, KCONTIG, KCONTIG, 2>();
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

    ANone::Dev none;
    if (K > 0 && K % (Cfg::ST * Cfg::BK) == 0) {
      // the second product's first tiles are fetched under the first product's last ones
      TilePipe<Cfg, KCONTIG, KCONTIG, VEC, ANone::Dev> pipe;
      gemm_mainloop_chain<Cfg, KCONTIG, KCONTIG, VEC, false, CHAIN_FIRST>(X, K, W, K, M, N, K, m0, n0, lds, none, acc[0],
                                                                          asum, pipe, Hin, P);
      gemm_mainloop_chain<Cfg, KCONTIG, KCONTIG, VEC, false, CHAIN_SECOND>(Hin, K, P, K, M, N, K, m0, n0, lds, none,
                                                                           acc[1], asum, pipe, nullptr, nullptr);
    } else {
      gemm_mainloop<Cfg, KCONTIG, KCONTIG, VEC, false>(X, K, W, K, M, N, K, m0, n0, lds, none, acc[0], asum);
      gemm_mainloop<Cfg, KCONTIG, KCONTIG, VEC, false>(Hin, K, P, K, M, N, K, m0, n0, lds, none, acc[1], asum);
    }
    typename EpiVijp<RELU>::Dev ed(epi, M, N);
    reduce_and_finish<Cfg, 2>(lds, M, N, m0, n0, acc, asum, ed);
    ed.finish();
  }
};

// Phase III for several independent stretches of the network at once. Between two re-seed points the forward
// sweep needs nothing but the kept activation and the kept cotangent at the stretch's first layer, so the
// stretches can be swept side by side: set g of a launch is one layer of stretch g (all of one shape). What a
// 256-row batch cannot give one layer -- enough 64 x 64 output tiles to fill the chip -- several layers give
// together. The tile is 64 x 64 and walks K in the order that reproduces the bits of the 32 x 32 tile with
// K split over KSETS wavefronts that Phase I takes for such a layer (gemm_mainloop_sets): the recomputed signs
// agree with the stored ones, and gradients do not depend on how many stretches ran together.
constexpr int MAX_GROUP = 16;

struct VijpSet {
  const float *X, *W, *Hin, *P, *bias;
  const uint64_t* mask;
  const uint32_t* offsets;     // ReLU only
  const uint64_t* frag_base;   // ReLU only
  float *Xout, *Hout, *CTZ;
};

template <class Cfg, bool RELU, int KSETS>
struct GroupedVijpTask {
  int n_sets, M, N, K;
  float alpha, inv_alpha;
  const float* frag;
  uint64_t frag_capacity;
  unsigned long long* mismatches;
  int tiles_m, tiles_n;
  VijpSet set[MAX_GROUP];
  static constexpr int LDS_BYTES = lds_bytes<Cfg, KCONTIG, KCONTIG, 2>();
  __host__ __device__ int blocks() const { return n_sets * tiles_m * tiles_n; }

  __device__ __forceinline__ void run(int bid, float* __restrict__ lds) const {
    // XCD-aware over the whole launch, row tiles fastest: an XCD works on whole column panels of one set's weights
    const int per = tiles_m * tiles_n;
    const int id = xcd_remap(bid, n_sets * per);
    const int g = id / per, local = id - g * per;
    const int m0 = (local % tiles_m) * Cfg::BM, n0 = (local / tiles_m) * Cfg::BN;
    const VijpSet& q = set[g];

    f32x16 acc[2][Cfg::NACC];
    ANone::Dev none;
    TilePipe<Cfg, KCONTIG, KCONTIG, true, ANone::Dev> pipe;
    gemm_mainloop_sets<Cfg, KCONTIG, KCONTIG, true, KSETS, CHAIN_FIRST>(q.X, K, q.W, K, M, N, K, m0, n0, lds, none, acc[0],
                                                                       pipe, q.Hin, q.P);
    gemm_mainloop_sets<Cfg, KCONTIG, KCONTIG, true, KSETS, CHAIN_SECOND>(q.Hin, K, q.P, K, M, N, K, m0, n0, lds, none, acc[1],
                                                                        pipe, nullptr, nullptr);
    const EpiVijp<RELU> epi{q.bias, alpha, inv_alpha, q.mask, q.offsets, frag, q.frag_base, frag_capacity,
                            q.Xout, q.Hout, q.CTZ, mismatches};
    typename EpiVijp<RELU>::Dev ed(epi, M, N);
    // the epilogue in quarters of a 32 x 32 tile (four accumulator registers at a time): its index and mask
    // arrays then take a quarter of the registers, which is what lets a third wavefront share a SIMD
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wn = wave % Cfg::WN, wm = wave / Cfg::WN, gl = lane >> 5;
#pragma unroll
    for (int tm = 0; tm < Cfg::WTM; ++tm)
#pragma unroll
      for (int tn = 0; tn < Cfg::WTN; ++tn)
#pragma unroll
        for (int i0 = 0; i0 < 16; i0 += 4) {
          float v[2][4];
#pragma unroll
          for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) v[q][j] = acc[q][tm * Cfg::WTN + tn][i0 + j];
          ed.template part<4>(M, N, m0 + (wm * Cfg::WTM + tm) * 32, n0 + (wn * Cfg::WTN + tn) * 32 + (lane & 31), gl, i0, v);
        }
    ed.finish();
  }
};

// The weight gradients (and bias gradients) of several layers of one shape in one grid: set g is the
// product GemmTask<Cfg, RCONTIG, RCONTIG, .., COLSUM> would compute alone, with the same bits.
struct DwSet {
  const float *CTZ, *X;
  float *dW, *db;
};

template <class Cfg>
struct GroupedDwTask {
  int n_sets, M, N, K;   // d_out, d_in, batch
  float scale, beta;
  int tiles_m, tiles_n;
  DwSet set[MAX_GROUP];
  using One = GemmTask<Cfg, RCONTIG, RCONTIG, true, ANone, EpiStore, true>;
  static constexpr int LDS_BYTES = One::LDS_BYTES;
  __host__ __device__ int blocks() const { return n_sets * tiles_m * tiles_n; }

  __device__ __forceinline__ void run(int bid, float* __restrict__ lds) const {
    const int per = tiles_m * tiles_n;
    // every XCD takes a contiguous range of the launch's tiles in set-major, column-panel order: a set's weight
    // gradient sits on 8 / n_sets XCDs, so its ct_z and x cross into that many L2s instead of all eight
    const int id = xcd_remap(bid, n_sets * per);
    const int g = id / per, tile = id - g * per;
    const DwSet& q = set[g];
    One t{M, N, K, q.CTZ, M, q.X, N, ANone{}, EpiStore{q.dW, N, scale, beta, nullptr}, q.db, scale, tiles_m, tiles_n};
    t.colsum_beta = beta;
    t.run_tile(tile % tiles_m, tile / tiles_m, lds);
  }
};

template <int NT, class Task>
__global__ void __launch_bounds__(NT) task_kernel(Task t) {
  extern __shared__ __align__(16) float lds[];
  t.run((int)blockIdx.x, lds);
}

// The same with a floor on the workgroups resident per CU (the compiler keeps the register count low
// enough for it): for kernels whose long epilogue should overlap another workgroup's main loop.
template <int NT, int MIN_WG, class Task>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(MIN_WG * NT / 256, 8)))
task_kernel_resident(Task t) {
  extern __shared__ __align__(16) float lds[];
  t.run((int)blockIdx.x, lds);
}

// Two independent tasks in one launch: blocks [0, first) run `a` (first = a.blocks() rounded up to
// a multiple of 8, the surplus blocks exit at once), the rest run `b`. The workgroups of both
// share the CUs, so the one task's memory stalls are filled with the other's matrix work, without
// any cross-queue dependency.
template <int NT, class TaskA, class TaskB>
__global__ void __launch_bounds__(NT) task_pair_kernel(TaskA a, TaskB b, int first) {
  extern __shared__ __align__(16) float lds[];
  const int bid = (int)blockIdx.x;
  if (bid < first) {
    if (bid < a.blocks()) a.run(bid, lds);
  } else {
    b.run(bid - first, lds);
  }
}

template <int NT, int MIN_WG, class TaskA, class TaskB>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(MIN_WG * NT / 256, 8)))
task_pair_kernel_resident(TaskA a, TaskB b, int first) {
  extern __shared__ __align__(16) float lds[];
  const int bid = (int)blockIdx.x;
  if (bid < first) {
    if (bid < a.blocks()) a.run(bid, lds);
  } else {
    b.run(bid - first, lds);
  }
}

// ------------------------------------------------------------------------------------ launch helpers

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
// an operand qualifies for dwordx4 staging when every 4-chunk is all-in or all-out and aligned
inline bool operand_vec_ok(const void* p, int64_t ld, int fast_extent) {
  return aligned16(p) && (ld % 4 == 0) && (fast_extent % 4 == 0);
}
// buffer offsets are 31-bit: the byte extent of every operand must stay below 2 GiB
inline bool extent_ok(int64_t n_outer, int64_t n_inner, int64_t ld) {
  return n_outer <= 0 || n_inner <= 0 || ((n_outer - 1) * ld + n_inner) * 4 < (int64_t)0x7FFFFFFF;
}

// Kernels here use up to ~130 KiB of dynamic LDS (the CU has 160 KiB); anything above the
// default limit needs it raised once per kernel.
template <class KernelT>
inline hipError_t ensure_lds(KernelT kernel, int bytes) {
  if (bytes <= 48 * 1024) return hipSuccess;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             bytes);
}

template <int NT, class Task>
inline hipError_t launch_task(const Task& t, hipStream_t stream) {
  auto kernel = task_kernel<NT, Task>;
  static hipError_t attr = ensure_lds(kernel, Task::LDS_BYTES);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kernel, dim3(t.blocks()), dim3(NT), Task::LDS_BYTES, stream, t);
  return hipGetLastError();
}

template <int NT, int MIN_WG, class Task>
inline hipError_t launch_task_resident(const Task& t, hipStream_t stream) {
  auto kernel = task_kernel_resident<NT, MIN_WG, Task>;
  static hipError_t attr = ensure_lds(kernel, Task::LDS_BYTES);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kernel, dim3(t.blocks()), dim3(NT), Task::LDS_BYTES, stream, t);
  return hipGetLastError();
}

template <int NT, class TaskA, class TaskB>
inline hipError_t launch_task_pair(const TaskA& a, const TaskB& b, hipStream_t stream) {
  auto kernel = task_pair_kernel<NT, TaskA, TaskB>;
  constexpr int bytes = TaskA::LDS_BYTES > TaskB::LDS_BYTES ? TaskA::LDS_BYTES : TaskB::LDS_BYTES;
  static hipError_t attr = ensure_lds(kernel, bytes);
  if (attr != hipSuccess) return attr;
  const int first = (a.blocks() + 7) / 8 * 8;
  hipLaunchKernelGGL(kernel, dim3(first + b.blocks()), dim3(NT), bytes, stream, a, b, first);
  return hipGetLastError();
}

template <int NT, int MIN_WG, class TaskA, class TaskB>
inline hipError_t launch_task_pair_resident(const TaskA& a, const TaskB& b, hipStream_t stream) {
  auto kernel = task_pair_kernel_resident<NT, MIN_WG, TaskA, TaskB>;
  constexpr int bytes = TaskA::LDS_BYTES > TaskB::LDS_BYTES ? TaskA::LDS_BYTES : TaskB::LDS_BYTES;
  static hipError_t attr = ensure_lds(kernel, bytes);
  if (attr != hipSuccess) return attr;
  const int first = (a.blocks() + 7) / 8 * 8;
  hipLaunchKernelGGL(kernel, dim3(first + b.blocks()), dim3(NT), bytes, stream, a, b, first);
  return hipGetLastError();
}

template <class Cfg, int LA, int LB, bool VEC, class Xf, class Epi, bool COLSUM>
inline GemmTask<Cfg, LA, LB, VEC, Xf, Epi, COLSUM> make_gemm_task(int M, int N, int K, const float* A, int64_t lda,
                                                                  const float* B, int64_t ldb, const Xf& xf,
                                                                  const Epi& epi, float* colsum_out,
                                                                  float colsum_scale) {
  return GemmTask<Cfg, LA, LB, VEC, Xf, Epi, COLSUM>{M, N, K, A, lda, B, ldb, xf, epi, colsum_out, colsum_scale,
                                                      ceil_div(M, Cfg::BM), ceil_div(N, Cfg::BN)};
}

// Row stride (floats) of the matrix an epilogue writes: its own ldc where it has one, else N (a dense output).
template <class Epi>
inline auto epi_row_stride(const Epi& e, int /*N*/, int) -> decltype((int64_t)e.ldc) { return (int64_t)e.ldc; }
template <class Epi>
inline int64_t epi_row_stride(const Epi&, int N, long) { return N > 0 ? N : 1; }

template <class Cfg, int LA, int LB, class Xf, class Epi, bool COLSUM>
inline hipError_t launch_gemm(int M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb,
                              const Xf& xf, const Epi& epi, bool xf_vec_ok, float* colsum_out, float colsum_scale,
                              hipStream_t stream, float colsum_beta = 0.f) {
  if (M <= 0 || N <= 0) return hipSuccess;
  const bool a_k = (LA == KCONTIG), b_k = (LB == KCONTIG);
  if (!extent_ok(a_k ? M : K, a_k ? K : M, lda) || !extent_ok(b_k ? N : K, b_k ? K : N, ldb) ||
      !extent_ok(M, N, epi_row_stride(epi, N, 0)))
    return hipErrorInvalidValue;
  const bool vec = xf_vec_ok && operand_vec_ok(A, lda, a_k ? K : M) && operand_vec_ok(B, ldb, b_k ? K : N);
  if (vec) {
    auto t = make_gemm_task<Cfg, LA, LB, true, Xf, Epi, COLSUM>(M, N, K, A, lda, B, ldb, xf, epi, colsum_out, colsum_scale);
    t.colsum_beta = colsum_beta;
    return launch_task<Cfg::NT>(t, stream);
  }
  auto t = make_gemm_task<Cfg, LA, LB, false, Xf, Epi, COLSUM>(M, N, K, A, lda, B, ldb, xf, epi, colsum_out, colsum_scale);
  t.colsum_beta = colsum_beta;
  return launch_task<Cfg::NT>(t, stream);
}

inline bool vijp_vec_ok(int K, const float* X, const float* W, const float* Hin, const float* P) {
  return (K % 4 == 0) && aligned16(X) && aligned16(W) && aligned16(Hin) && aligned16(P);
}

template <class Cfg, bool VEC, bool RELU>
inline VijpTask<Cfg, VEC, RELU> make_vijp_task(int M, int N, int K, const float* X, const float* W, const float* Hin,
                                               const float* P, const EpiVijp<RELU>& epi) {
  return VijpTask<Cfg, VEC, RELU>{M, N, K, X, W, Hin, P, epi, ceil_div(M, Cfg::BM), ceil_div(N, Cfg::BN)};
}

template <class Cfg, bool RELU>
inline hipError_t launch_vijp_dual(int M, int N, int K, const float* X, const float* W, const float* Hin,
                                   const float* P, const EpiVijp<RELU>& epi, hipStream_t stream) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (!extent_ok(M, K, K) || !extent_ok(N, K, K) || !extent_ok(M, N, N)) return hipErrorInvalidValue;
  if (vijp_vec_ok(K, X, W, Hin, P))
    return launch_task<Cfg::NT>(make_vijp_task<Cfg, true, RELU>(M, N, K, X, W, Hin, P, epi), stream);
  return launch_task<Cfg::NT>(make_vijp_task<Cfg, false, RELU>(M, N, K, X, W, Hin, P, epi), stream);
}

}  // namespace mw
