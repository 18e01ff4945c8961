// HBM-bound elementwise, bit-pack and stream-compaction kernels (wave64, gfx950).
//
// Packed masks: flat row-major element e is bit (e % 64) of uint64 word e / 64, LSB first, which
// is exactly the order of a wave64 ballot when lane l handles element 64 w + l. All kernels
// below give every wavefront whole 64-element words, so loads and stores are fully coalesced
// (256 B per wavefront per access) and the integer work is a ballot or a popcount per word.
#include "mw_internal.h"

#include <mutex>

namespace mw {

namespace {

typedef float f4v __attribute__((ext_vector_type(4)));  // what the non-temporal builtins take

constexpr int EW_THREADS = 256;
constexpr int EW_WAVES = EW_THREADS / 64;
// Measured on MI355X with 1 GiB tensors: a copy with plain 128-bit accesses from 8 workgroups per CU moves
// 4.8 TB/s; with accesses marked non-temporal (streamed past the caches: every element here is touched
// once) and up to 128 workgroups per CU it moves 6.3 TB/s. Reads alone: 6.2 against 7.0 TB/s.
constexpr int EW_MAX_BLOCKS = 256 * 128;
constexpr int UNROLL = 4;               // words per wavefront per trip

inline int ew_blocks(int64_t n_words, int words_per_block) {
  int64_t b = (n_words + words_per_block - 1) / words_per_block;
  if (b < 1) b = 1;
  if (b > EW_MAX_BLOCKS) b = EW_MAX_BLOCKS;
  return (int)b;
}

__device__ __forceinline__ int64_t global_wave() { return (int64_t)blockIdx.x * EW_WAVES + (threadIdx.x >> 6); }
__device__ __forceinline__ int64_t total_waves() { return (int64_t)gridDim.x * EW_WAVES; }

// ---------------------------------------------------------------- 128-bit path
// With 16-byte aligned tensors every lane moves a float4 (elements 4l .. 4l+3 of a 256-element
// group, i.e. 4 mask words per wavefront trip). The four ballots (one per component) hold bit
// j of lane l at position l; word w of the group wants lanes 16w .. 16w+15, components
// interleaved: element 4(l-16w)+j. spread16x4 moves bit i of a 16-bit field to bit 4i.
constexpr int VUNROLL = 2;  // 256-element groups per wavefront trip

__device__ __forceinline__ uint64_t spread16x4(uint64_t v) {
  v &= 0xFFFFull;
  v = (v | (v << 24)) & 0x000000FF000000FFull;
  v = (v | (v << 12)) & 0x000F000F000F000Full;
  v = (v | (v << 6)) & 0x0303030303030303ull;
  v = (v | (v << 3)) & 0x1111111111111111ull;
  return v;
}
// the mask word this lane should store (lanes 0..3 hold words 0..3 of the group)
__device__ __forceinline__ uint64_t group_word(bool b0, bool b1, bool b2, bool b3, int lane) {
  const unsigned long long q0 = __ballot(b0), q1 = __ballot(b1), q2 = __ballot(b2), q3 = __ballot(b3);
  const int sh = 16 * (lane & 3);
  return spread16x4(q0 >> sh) | (spread16x4(q1 >> sh) << 1) | (spread16x4(q2 >> sh) << 2) |
         (spread16x4(q3 >> sh) << 3);
}
__device__ __forceinline__ float4 ld4(const float* __restrict__ p, int64_t e, int64_t n) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (e + 3 < n) {
    const f4v t = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(p + e));
    v = make_float4(t.x, t.y, t.z, t.w);
  } else if (e < n) {
    v.x = p[e];
    if (e + 1 < n) v.y = p[e + 1];
    if (e + 2 < n) v.z = p[e + 2];
  }
  return v;
}
__device__ __forceinline__ void st4(float* __restrict__ p, int64_t e, int64_t n, float4 v) {
  if (e + 3 < n) {
    const f4v t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<f4v*>(p + e));
  } else if (e < n) {
    p[e] = v.x;
    if (e + 1 < n) p[e + 1] = v.y;
    if (e + 2 < n) p[e + 2] = v.z;
  }
}
__device__ __forceinline__ float pick(const float4& v, int j) { return j == 0 ? v.x : j == 1 ? v.y : j == 2 ? v.z : v.w; }
__device__ __forceinline__ void put(float4& v, int j, float x) {
  if (j == 0) v.x = x; else if (j == 1) v.y = x; else if (j == 2) v.z = x; else v.w = x;
}

template <bool HAS_BIAS>
__global__ void __launch_bounds__(EW_THREADS)
k_bias_act_mask_v4(const float* __restrict__ zin, const float* __restrict__ bias, int64_t n, int d, float alpha,
                   float* __restrict__ x, uint64_t* __restrict__ mask) {
  const int lane = threadIdx.x & 63;
  const int64_t n_words = (n + 63) >> 6, n_groups = (n + 255) >> 8;
  const int64_t stride = total_waves() * VUNROLL;
  for (int64_t g0 = global_wave() * VUNROLL; g0 < n_groups; g0 += stride) {
    float4 z[VUNROLL];
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) z[u] = ld4(zin, (g0 + u) * 256 + 4 * lane, n);
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) {
      const int64_t e = (g0 + u) * 256 + 4 * lane;
      if (HAS_BIAS && e < n) {
        const int c = (int)(e % d);  // d % 4 == 0 on this path: the 4 columns are c .. c+3
        const float4 b = *reinterpret_cast<const float4*>(bias + c);
        z[u].x += b.x; z[u].y += b.y; z[u].z += b.z; z[u].w += b.w;
      }
      const bool b0 = e < n && z[u].x > 0.f, b1 = e + 1 < n && z[u].y > 0.f, b2 = e + 2 < n && z[u].z > 0.f,
                 b3 = e + 3 < n && z[u].w > 0.f;
      float4 o;
      o.x = b0 ? z[u].x : alpha * z[u].x; o.y = b1 ? z[u].y : alpha * z[u].y;
      o.z = b2 ? z[u].z : alpha * z[u].z; o.w = b3 ? z[u].w : alpha * z[u].w;
      st4(x, e, n, o);
      const uint64_t word = group_word(b0, b1, b2, b3, lane);
      const int64_t wi = (g0 + u) * 4 + lane;
      if (mask && lane < 4 && wi < n_words) mask[wi] = word;
    }
  }
}

__global__ void __launch_bounds__(EW_THREADS)
k_mask_from_act_v4(const float* __restrict__ x, int64_t n, uint64_t* __restrict__ mask) {
  const int lane = threadIdx.x & 63;
  const int64_t n_words = (n + 63) >> 6, n_groups = (n + 255) >> 8;
  const int64_t stride = total_waves() * VUNROLL;
  for (int64_t g0 = global_wave() * VUNROLL; g0 < n_groups; g0 += stride) {
    float4 v[VUNROLL];
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) v[u] = ld4(x, (g0 + u) * 256 + 4 * lane, n);
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) {
      const uint64_t word = group_word(v[u].x > 0.f, v[u].y > 0.f, v[u].z > 0.f, v[u].w > 0.f, lane);
      const int64_t wi = (g0 + u) * 4 + lane;
      if (lane < 4 && wi < n_words) mask[wi] = word;
    }
  }
}

__global__ void __launch_bounds__(EW_THREADS)
k_rev_scale_v4(const float* __restrict__ h, const uint64_t* __restrict__ mask, int64_t n, float alpha,
               float* __restrict__ ct_z) {
  const int lane = threadIdx.x & 63;
  const int64_t n_words = (n + 63) >> 6, n_groups = (n + 255) >> 8;
  const int64_t stride = total_waves() * VUNROLL;
  for (int64_t g0 = global_wave() * VUNROLL; g0 < n_groups; g0 += stride) {
    float4 v[VUNROLL];
    uint64_t m[VUNROLL];
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) {
      v[u] = ld4(h, (g0 + u) * 256 + 4 * lane, n);
      const int64_t wi = (g0 + u) * 4 + (lane >> 4);
      m[u] = wi < n_words ? mask[wi] : 0ull;
    }
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) {
      const uint32_t bits = (uint32_t)(m[u] >> (4 * (lane & 15))) & 15u;
      float4 o;
      o.x = v[u].x * ((bits & 1u) ? 1.f : alpha); o.y = v[u].y * ((bits & 2u) ? 1.f : alpha);
      o.z = v[u].z * ((bits & 4u) ? 1.f : alpha); o.w = v[u].w * ((bits & 8u) ? 1.f : alpha);
      st4(ct_z, (g0 + u) * 256 + 4 * lane, n, o);
    }
  }
}

// A wavefront's 256 elements hold a contiguous run of the store (about half of them are erased). The erased
// values are first put in order into the wavefront's own LDS slot, then written out 64 at a time, lane k next
// to lane k + 1: full 256-byte stores instead of four scattered ones per lane.
__global__ void __launch_bounds__(EW_THREADS)
k_frag_compact_v4(const float* __restrict__ h, const uint64_t* __restrict__ mask, const uint32_t* __restrict__ offsets,
                  int64_t n, float* __restrict__ frag, const uint64_t* __restrict__ base_ptr, uint64_t capacity,
                  int32_t* __restrict__ overflow_flag) {
  __shared__ float stage[EW_WAVES][VUNROLL][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t n_words = (n + 63) >> 6, n_groups = (n + 255) >> 8;
  const int64_t stride = total_waves() * VUNROLL;
  const uint64_t base = base_ptr ? *base_ptr : 0ull;
  const int pos0 = 4 * (lane & 15);
  for (int64_t g0 = global_wave() * VUNROLL; g0 < n_groups; g0 += stride) {
    float4 v[VUNROLL];
    uint64_t m[VUNROLL];
    uint32_t off[VUNROLL], first[VUNROLL], end[VUNROLL];
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) {
      v[u] = ld4(h, (g0 + u) * 256 + 4 * lane, n);
      const int64_t w0 = (g0 + u) * 4, wi = w0 + (lane >> 4);
      m[u] = wi < n_words ? mask[wi] : ~0ull;
      off[u] = wi < n_words ? offsets[wi] : 0u;
      // the group's run of the store: [first, end)
      first[u] = w0 < n_words ? offsets[w0] : 0u;
      end[u] = w0 < n_words ? offsets[w0 + 4 < n_words ? w0 + 4 : n_words] : 0u;
    }
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) {
      const int64_t e = (g0 + u) * 256 + 4 * lane;
      // erased elements of this word below this lane's first position, then one by one
      uint32_t idx = off[u] - first[u] + (uint32_t)__popcll(~m[u] & ((1ull << pos0) - 1ull));
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool erased = (e + j < n) && !((m[u] >> (pos0 + j)) & 1ull);
        if (erased) stage[wave][u][idx++] = pick(v[u], j);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) {
      const uint32_t count = end[u] - first[u];
      const uint64_t dst = base + first[u];
      for (uint32_t k = lane; k < count; k += 64) {
        if (dst + k < capacity) __builtin_nontemporal_store(stage[wave][u][k], frag + dst + k);
        else if (overflow_flag) *overflow_flag = 1;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

template <bool RELU>
__global__ void __launch_bounds__(EW_THREADS)
k_vijp_epilogue_v4(const float* __restrict__ z, float* __restrict__ ct_z, int64_t n, float alpha, float inv_alpha,
                   const uint64_t* __restrict__ mask, const uint32_t* __restrict__ offsets,
                   const float* __restrict__ frag, const uint64_t* __restrict__ base_ptr, uint64_t capacity,
                   float* __restrict__ x, float* __restrict__ h_y, unsigned long long* __restrict__ mismatches) {
  const int lane = threadIdx.x & 63;
  const int64_t n_words = (n + 63) >> 6, n_groups = (n + 255) >> 8;
  const int64_t stride = total_waves() * VUNROLL;
  const uint64_t base = (RELU && base_ptr) ? *base_ptr : 0ull;
  const int pos0 = 4 * (lane & 15);
  uint32_t mism = 0;
  for (int64_t g0 = global_wave() * VUNROLL; g0 < n_groups; g0 += stride) {
    float4 zz[VUNROLL], cc[VUNROLL];
    uint64_t m[VUNROLL];
    uint32_t off[VUNROLL];
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) {
      const int64_t e = (g0 + u) * 256 + 4 * lane;
      zz[u] = ld4(z, e, n);
      cc[u] = ld4(ct_z, e, n);
      const int64_t wi = (g0 + u) * 4 + (lane >> 4);
      m[u] = (mask && wi < n_words) ? mask[wi] : 0ull;
      off[u] = (RELU && wi < n_words) ? offsets[wi] : 0u;
    }
#pragma unroll
    for (int u = 0; u < VUNROLL; ++u) {
      const int64_t e = (g0 + u) * 256 + 4 * lane;
      float4 xo, ho, co;
      uint64_t idx = base + off[u] + (uint64_t)__popcll(~m[u] & ((1ull << pos0) - 1ull));
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float zj = pick(zz[u], j), cj = pick(cc[u], j);
        const bool in = e + j < n;
        const bool fresh = zj > 0.f;
        const bool stored = (m[u] >> (pos0 + j)) & 1ull;
        if (mask && in && fresh != stored) ++mism;
        if (RELU) {
          const float c = stored ? cj : 0.f;
          float hy = c;
          if (in && !stored) {
            hy = idx < capacity ? frag[idx] : 0.f;
            ++idx;
          }
          put(xo, j, stored ? zj : alpha * zj);
          put(co, j, c);
          put(ho, j, hy);
        } else {
          put(xo, j, fresh ? zj : alpha * zj);
          put(ho, j, fresh ? cj : cj * inv_alpha);
        }
      }
      st4(x, e, n, xo);
      st4(h_y, e, n, ho);
      if (RELU) st4(ct_z, e, n, co);
    }
  }
  if (mismatches && mism) atomicAdd(mismatches, (unsigned long long)mism);
}

// ---------------------------------------------------------------- phase I: bias + mask + activation
template <bool HAS_BIAS>
__global__ void __launch_bounds__(EW_THREADS)
k_bias_act_mask(const float* __restrict__ zin, const float* __restrict__ bias, int64_t n, int d, float alpha,
                float* __restrict__ x, uint64_t* __restrict__ mask) {
  const int lane = threadIdx.x & 63;
  const int64_t n_words = (n + 63) >> 6;
  const int64_t stride_words = total_waves() * UNROLL;
  const int step64 = 64 % d;                                  // column advance per word
  const int step_trip = (int)((stride_words * 64) % d);       // column advance per trip
  int64_t w0 = global_wave() * UNROLL;
  int col0 = HAS_BIAS ? (int)((w0 * 64 + lane) % d) : 0;      // one wide modulo per thread
  for (; w0 < n_words; w0 += stride_words) {
    float z[UNROLL];
    int col = col0;
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) {
      int64_t e = (w0 + j) * 64 + lane;
      z[j] = 0.f;
      if (e < n) {
        z[j] = zin[e];
        if (HAS_BIAS) z[j] += bias[col];
      }
      if (HAS_BIAS) { col += step64; if (col >= d) col -= d; }
    }
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) {
      int64_t e = (w0 + j) * 64 + lane;
      bool bit = (e < n) && (z[j] > 0.f);
      if (e < n) x[e] = bit ? z[j] : alpha * z[j];
      unsigned long long bal = __ballot(bit);
      if (mask && lane == 0 && w0 + j < n_words) mask[w0 + j] = bal;
    }
    if (HAS_BIAS) { col0 += step_trip; if (col0 >= d) col0 -= d; }
  }
}

// mask bit = (x > 0): equals (z > 0) because alpha >= 0 keeps the sign (and maps z <= 0 to x <= 0)
__global__ void __launch_bounds__(EW_THREADS)
k_mask_from_act(const float* __restrict__ x, int64_t n, uint64_t* __restrict__ mask) {
  const int lane = threadIdx.x & 63;
  const int64_t n_words = (n + 63) >> 6;
  const int64_t stride_words = total_waves() * UNROLL;
  for (int64_t w0 = global_wave() * UNROLL; w0 < n_words; w0 += stride_words) {
    float v[UNROLL];
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) {
      int64_t e = (w0 + j) * 64 + lane;
      v[j] = e < n ? x[e] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) {
      unsigned long long bal = __ballot(v[j] > 0.f);
      if (lane == 0 && w0 + j < n_words) mask[w0 + j] = bal;
    }
  }
}

// ---------------------------------------------------------------- phase II: slope scaling
__global__ void __launch_bounds__(EW_THREADS)
k_rev_scale(const float* __restrict__ h, const uint64_t* __restrict__ mask, int64_t n, float alpha,
            float* __restrict__ ct_z) {
  const int lane = threadIdx.x & 63;
  const int64_t n_words = (n + 63) >> 6;
  const int64_t stride_words = total_waves() * UNROLL;
  for (int64_t w0 = global_wave() * UNROLL; w0 < n_words; w0 += stride_words) {
    float v[UNROLL];
    uint64_t m[UNROLL];
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) {
      int64_t e = (w0 + j) * 64 + lane;
      v[j] = e < n ? h[e] : 0.f;
      m[j] = (w0 + j < n_words) ? mask[w0 + j] : 0ull;
    }
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) {
      int64_t e = (w0 + j) * 64 + lane;
      if (e < n) ct_z[e] = v[j] * (((m[j] >> lane) & 1ull) ? 1.f : alpha);
    }
  }
}

// ---------------------------------------------------------------- fragment index: erased-count scan
// offsets[w] = number of erased (zero) bits in all words before w; offsets[n_words] = total.
// Every workgroup owns a contiguous chunk of words. It first counts the erased bits of ALL
// earlier chunks (the mask is small and L2-resident, so this redundant read is cheaper than a
// second launch or a cross-workgroup hand-off), then scans its own chunk through LDS.
// Integer arithmetic only: the result does not depend on scheduling.
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_WORDS_PER_THREAD = 8;

__device__ __forceinline__ uint32_t erased_in_word(uint64_t w, int64_t word_index, int64_t n) {
  int64_t valid = n - word_index * 64;
  if (valid >= 64) return (uint32_t)__popcll(~w);
  uint64_t keep = (valid <= 0) ? 0ull : ((1ull << valid) - 1ull);
  return (uint32_t)__popcll(~w & keep);
}

// block-wide sum of one value per thread; every thread gets the total
__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t* red) {
  red[threadIdx.x] = v;
  __syncthreads();
  for (int s = SCAN_THREADS / 2; s > 0; s >>= 1) {
    if (threadIdx.x < (unsigned)s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  uint32_t t = red[0];
  __syncthreads();
  return t;
}

// Two-level scan over chunks of SCAN_CHUNK_WORDS mask words. First launch: one workgroup per chunk counts the
// erased bits of its chunk into sums[chunk]. Second launch: workgroup c adds up sums[0 .. c) (at most a few
// thousand values, whatever the layer's size), then scans its own chunk and writes the offsets. Every mask word is
// read twice and nothing is counted more often than that, so the scan stays bound by memory for any size.
constexpr int64_t SCAN_CHUNK_WORDS = (int64_t)SCAN_THREADS * SCAN_WORDS_PER_THREAD;

__device__ __forceinline__ void frag_chunk_sum(const uint64_t* __restrict__ mask, int64_t n, uint32_t* __restrict__ sums,
                                               uint32_t* red) {
  const int64_t n_words = (n + 63) >> 6;
  const int64_t c0 = (int64_t)blockIdx.x * SCAN_CHUNK_WORDS;
  if (c0 >= n_words) return;
  const int64_t c1 = c0 + SCAN_CHUNK_WORDS < n_words ? c0 + SCAN_CHUNK_WORDS : n_words;
  uint32_t cnt = 0;
  for (int64_t w = c0 + threadIdx.x; w < c1; w += SCAN_THREADS) cnt += erased_in_word(mask[w], w, n);
  cnt = block_sum(cnt, red);
  if (threadIdx.x == 0) sums[blockIdx.x] = cnt;
}

__device__ __forceinline__ void frag_offsets_chunk(const uint64_t* __restrict__ mask, int64_t n,
                                                   uint32_t* __restrict__ offsets, const uint32_t* __restrict__ sums,
                                                   uint32_t* red) {
  const int64_t n_words = (n + 63) >> 6;
  const int64_t c0 = (int64_t)blockIdx.x * SCAN_CHUNK_WORDS;
  if (c0 >= n_words) {  // nothing to scan here; an empty mask still gets its total
    if (n_words == 0 && blockIdx.x == 0 && threadIdx.x == 0) offsets[0] = 0u;
    return;
  }
  const int64_t c1 = c0 + SCAN_CHUNK_WORDS < n_words ? c0 + SCAN_CHUNK_WORDS : n_words;
  // erased bits before this chunk
  uint32_t before = 0;
  for (int64_t c = threadIdx.x; c < (int64_t)blockIdx.x; c += SCAN_THREADS) before += sums[c];
  before = block_sum(before, red);
  // this chunk: each thread takes a contiguous run of words
  const int64_t lo = c0 + (int64_t)threadIdx.x * SCAN_WORDS_PER_THREAD;
  const int64_t hi = lo + SCAN_WORDS_PER_THREAD < c1 ? lo + SCAN_WORDS_PER_THREAD : c1;
  uint32_t each[SCAN_WORDS_PER_THREAD];
  uint32_t cnt = 0;
#pragma unroll
  for (int j = 0; j < SCAN_WORDS_PER_THREAD; ++j) {
    each[j] = lo + j < hi ? erased_in_word(mask[lo + j], lo + j, n) : 0u;
    cnt += each[j];
  }
  red[threadIdx.x] = cnt;
  __syncthreads();
  for (int off = 1; off < SCAN_THREADS; off <<= 1) {  // inclusive Hillis-Steele scan
    uint32_t add = threadIdx.x >= (unsigned)off ? red[threadIdx.x - off] : 0u;
    __syncthreads();
    red[threadIdx.x] += add;
    __syncthreads();
  }
  uint32_t run = before + red[threadIdx.x] - cnt;
#pragma unroll
  for (int j = 0; j < SCAN_WORDS_PER_THREAD; ++j) {
    if (lo + j < hi) offsets[lo + j] = run;
    run += each[j];
  }
  if (c1 == n_words && threadIdx.x == SCAN_THREADS - 1) offsets[n_words] = before + red[SCAN_THREADS - 1];
}

__global__ void __launch_bounds__(SCAN_THREADS)
k_frag_chunk_sums(const uint64_t* __restrict__ mask, int64_t n, uint32_t* __restrict__ sums) {
  __shared__ uint32_t red[SCAN_THREADS];
  frag_chunk_sum(mask, n, sums, red);
}

__global__ void __launch_bounds__(SCAN_THREADS)
k_frag_offsets(const uint64_t* __restrict__ mask, int64_t n, uint32_t* __restrict__ offsets, const uint32_t* __restrict__ sums) {
  __shared__ uint32_t red[SCAN_THREADS];
  frag_offsets_chunk(mask, n, offsets, sums, red);
}

// The same for several layers in one launch each: blockIdx.y selects the layer.
__global__ void __launch_bounds__(SCAN_THREADS) k_frag_chunk_sums_layers(const FragLayer* __restrict__ layers) {
  __shared__ uint32_t red[SCAN_THREADS];
  const FragLayer l = layers[blockIdx.y];
  frag_chunk_sum(l.mask, l.n, l.sums, red);
}

__global__ void __launch_bounds__(SCAN_THREADS) k_frag_offsets_layers(const FragLayer* __restrict__ layers) {
  __shared__ uint32_t red[SCAN_THREADS];
  const FragLayer l = layers[blockIdx.y];
  frag_offsets_chunk(l.mask, l.n, l.offsets, l.sums, red);
}

// Layer bases: exclusive scan of the erased counts in the order given (reverse-pass order).
// The counts are fetched 256 at a time by the whole workgroup; one thread adds them up.
__global__ void __launch_bounds__(SCAN_THREADS)
k_frag_bases(const uint32_t* const* __restrict__ count_ptrs, int n_relu, uint64_t* __restrict__ bases,
             uint64_t* __restrict__ total) {
  __shared__ uint32_t cnt[SCAN_THREADS];
  __shared__ uint64_t carry;
  if (threadIdx.x == 0) carry = 0;
  for (int j0 = 0; j0 < n_relu; j0 += SCAN_THREADS) {
    const int j = j0 + threadIdx.x;
    cnt[threadIdx.x] = j < n_relu ? *count_ptrs[j] : 0u;
    __syncthreads();
    if (threadIdx.x == 0) {
      uint64_t run = carry;
      const int m = n_relu - j0 < SCAN_THREADS ? n_relu - j0 : SCAN_THREADS;
      for (int k = 0; k < m; ++k) {
        bases[j0 + k] = run;
        run += cnt[k];
      }
      carry = run;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) *total = carry;
}

// ---------------------------------------------------------------- phase II: fragment compaction
__global__ void __launch_bounds__(EW_THREADS)
k_frag_compact(const float* __restrict__ h, const uint64_t* __restrict__ mask, const uint32_t* __restrict__ offsets,
               int64_t n, float* __restrict__ frag, const uint64_t* __restrict__ base_ptr, uint64_t capacity,
               int32_t* __restrict__ overflow_flag) {
  const int lane = threadIdx.x & 63;
  const int64_t n_words = (n + 63) >> 6;
  const int64_t stride_words = total_waves() * UNROLL;
  const uint64_t base = base_ptr ? *base_ptr : 0ull;
  const uint64_t below = (1ull << lane) - 1ull;
  for (int64_t w0 = global_wave() * UNROLL; w0 < n_words; w0 += stride_words) {
    float v[UNROLL];
    uint64_t m[UNROLL];
    uint32_t off[UNROLL];
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) {
      int64_t e = (w0 + j) * 64 + lane;
      bool in = w0 + j < n_words;
      v[j] = e < n ? h[e] : 0.f;
      m[j] = in ? mask[w0 + j] : ~0ull;
      off[j] = in ? offsets[w0 + j] : 0u;
    }
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) {
      int64_t e = (w0 + j) * 64 + lane;
      bool erased = (e < n) && !((m[j] >> lane) & 1ull);
      if (erased) {
        uint64_t idx = base + off[j] + (uint64_t)__popcll(~m[j] & below);
        if (idx < capacity) frag[idx] = v[j];
        else if (overflow_flag) *overflow_flag = 1;
      }
    }
  }
}

// ---------------------------------------------------------------- phase III: stand-alone epilogue
template <bool RELU>
__global__ void __launch_bounds__(EW_THREADS)
k_vijp_epilogue(const float* __restrict__ z, float* __restrict__ ct_z, int64_t n, float alpha, float inv_alpha,
                const uint64_t* __restrict__ mask, const uint32_t* __restrict__ offsets,
                const float* __restrict__ frag, const uint64_t* __restrict__ base_ptr, uint64_t capacity,
                float* __restrict__ x, float* __restrict__ h_y, unsigned long long* __restrict__ mismatches) {
  const int lane = threadIdx.x & 63;
  const int64_t n_words = (n + 63) >> 6;
  const int64_t stride_words = total_waves() * UNROLL;
  const uint64_t below = (1ull << lane) - 1ull;
  const uint64_t base = (RELU && base_ptr) ? *base_ptr : 0ull;
  for (int64_t w0 = global_wave() * UNROLL; w0 < n_words; w0 += stride_words) {
    float zz[UNROLL], cc[UNROLL];
    uint64_t m[UNROLL];
    uint32_t off[UNROLL];
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) {
      int64_t e = (w0 + j) * 64 + lane;
      bool in = w0 + j < n_words;
      zz[j] = e < n ? z[e] : 0.f;
      cc[j] = e < n ? ct_z[e] : 0.f;
      m[j] = (mask && in) ? mask[w0 + j] : 0ull;
      off[j] = (RELU && in) ? offsets[w0 + j] : 0u;
    }
#pragma unroll
    for (int j = 0; j < UNROLL; ++j) {
      int64_t e = (w0 + j) * 64 + lane;
      if (e >= n) continue;
      bool fresh = zz[j] > 0.f;
      bool stored = (m[j] >> lane) & 1ull;
      if (mask && mismatches && fresh != stored) atomicAdd(mismatches, 1ull);
      if (RELU) {
        float c = stored ? cc[j] : 0.f;
        float hy = c;
        if (!stored) {
          uint64_t idx = base + off[j] + (uint64_t)__popcll(~m[j] & below);
          hy = idx < capacity ? frag[idx] : 0.f;
        }
        x[e] = stored ? zz[j] : alpha * zz[j];
        ct_z[e] = c;
        h_y[e] = hy;
      } else {
        x[e] = fresh ? zz[j] : alpha * zz[j];
        h_y[e] = fresh ? cc[j] : cc[j] * inv_alpha;
      }
    }
  }
}

// ---------------------------------------------------------------- column sums (bias gradient)
// Thread j of a workgroup owns column j and walks a contiguous range of rows; partial sums over
// COLSUM_SPLIT row ranges are combined in LDS in a fixed order.
constexpr int COLSUM_COLS = 32, COLSUM_SPLIT = 32;
// Workgroup (bx, by) sums rows [by * rows_per_block, ...) of columns [32 bx, 32 bx + 32) into
// out[by * d + col] (times scale).
__global__ void __launch_bounds__(COLSUM_COLS* COLSUM_SPLIT)
k_colsum(const float* __restrict__ a, int64_t rows, int64_t rows_per_block, int d, float scale, float* __restrict__ out) {
  __shared__ float part[COLSUM_SPLIT][COLSUM_COLS];
  const int c = threadIdx.x % COLSUM_COLS, s = threadIdx.x / COLSUM_COLS;
  const int col = blockIdx.x * COLSUM_COLS + c;
  const int64_t first = (int64_t)blockIdx.y * rows_per_block;
  const int64_t last = first + rows_per_block < rows ? first + rows_per_block : rows;
  const int64_t per = (last - first + COLSUM_SPLIT - 1) / COLSUM_SPLIT;
  const int64_t lo = first + s * per, hi = lo + per < last ? lo + per : last;
  float acc = 0.f;
  if (col < d) {
    const float* p = a + col;
    int64_t r = lo;
    for (; r + 4 <= hi; r += 4) {  // four rows in flight; added in row order
      float v0 = p[r * d], v1 = p[(r + 1) * d], v2 = p[(r + 2) * d], v3 = p[(r + 3) * d];
      acc += v0;
      acc += v1;
      acc += v2;
      acc += v3;
    }
    for (; r < hi; ++r) acc += p[r * d];
  }
  part[s][c] = acc;
  __syncthreads();
  if (s == 0 && col < d) {
    float t = part[0][c];
    for (int k = 1; k < COLSUM_SPLIT; ++k) t += part[k][c];
    out[(int64_t)blockIdx.y * d + col] = scale * t;
  }
}

// The same with 128-bit accesses, for d % 4 == 0 and a 16-byte aligned matrix: a workgroup takes 128
// columns (32 lanes x 4) and splits its row range over 8 lanes of rows; each thread has eight rows in
// flight and adds them in row order; the 8 partial sums are combined in LDS in a fixed order.
constexpr int COLSUM4_QUADS = 32, COLSUM4_SPLIT = 8, COLSUM4_ROWS = 8;
constexpr int COLSUM4_BLOCK_ROWS = COLSUM4_SPLIT * COLSUM4_ROWS;  // rows one workgroup takes per trip
// Workgroup (bx, by) takes the row blocks by, by + gridDim.y, ... of COLSUM4_BLOCK_ROWS rows each (so the
// workgroups running at one time read one compact stretch of the matrix); inside a block row lane s takes the
// rows s, s + 8, ... (the two row lanes of a wavefront read neighbouring rows), eight of them in flight, added in
// row order. rows_per_block is unused here (the slice count alone fixes the order of the sums).
__global__ void __launch_bounds__(COLSUM4_QUADS* COLSUM4_SPLIT)
k_colsum_v4(const float* __restrict__ a, int64_t rows, int64_t /*rows_per_block*/, int d, float scale, float* __restrict__ out) {
  __shared__ f4v part[COLSUM4_SPLIT][COLSUM4_QUADS];
  const int q = threadIdx.x % COLSUM4_QUADS, s = threadIdx.x / COLSUM4_QUADS;
  const int col = 4 * (blockIdx.x * COLSUM4_QUADS + q);
  f4v acc = {0.f, 0.f, 0.f, 0.f};
  if (col < d) {
    const float* p = a + col;
    for (int64_t r0 = (int64_t)blockIdx.y * COLSUM4_BLOCK_ROWS; r0 < rows; r0 += (int64_t)gridDim.y * COLSUM4_BLOCK_ROWS) {
      f4v v[COLSUM4_ROWS];
#pragma unroll
      for (int j = 0; j < COLSUM4_ROWS; ++j) {
        const int64_t r = r0 + s + (int64_t)j * COLSUM4_SPLIT;
        v[j] = f4v{0.f, 0.f, 0.f, 0.f};
        if (r < rows) v[j] = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(p + r * d));
      }
#pragma unroll
      for (int j = 0; j < COLSUM4_ROWS; ++j) acc += v[j];
    }
  }
  part[s][q] = acc;
  __syncthreads();
  if (s == 0 && col < d) {
    f4v t = part[0][q];
    for (int k = 1; k < COLSUM4_SPLIT; ++k) t += part[k][q];
    t *= scale;
    *reinterpret_cast<f4v*>(out + (int64_t)blockIdx.y * d + col) = t;
  }
}

// The same sum for short vectors and many slices, where one thread per element would walk the slices
// one memory round trip at a time: REDUCE_GROUPS threads share an element, thread g adds the slices
// g, g + REDUCE_GROUPS, ... and the group sums are added in group order. (A different, equally fixed,
// association of the same terms.)
constexpr int REDUCE_ELEMS = 4, REDUCE_GROUPS = 64;
__global__ void __launch_bounds__(REDUCE_ELEMS* REDUCE_GROUPS)
k_reduce_slices_short(const float* __restrict__ part, int slices, int64_t n, float scale, float beta, float* __restrict__ out) {
  __shared__ float sums[REDUCE_GROUPS][REDUCE_ELEMS];
  const int e = threadIdx.x % REDUCE_ELEMS, g = threadIdx.x / REDUCE_ELEMS;
  const int64_t i = (int64_t)blockIdx.x * REDUCE_ELEMS + e;
  float t = 0.f;
  if (i < n) {
    int k = g;
    for (; k + 7 * REDUCE_GROUPS < slices; k += 8 * REDUCE_GROUPS) {  // eight slices in flight, added in slice order
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = part[(int64_t)(k + j * REDUCE_GROUPS) * n + i];
#pragma unroll
      for (int j = 0; j < 8; ++j) t += v[j];
    }
    for (; k < slices; k += REDUCE_GROUPS) t += part[(int64_t)k * n + i];
  }
  sums[g][e] = t;
  __syncthreads();
  if (g == 0 && i < n) {
    float r = sums[0][e];
    for (int q = 1; q < REDUCE_GROUPS; ++q) r += sums[q][e];
    r *= scale;
    if (beta != 0.f) r += beta * out[i];
    out[i] = r;
  }
}

// out[i] = scale * (part[0][i] + part[1][i] + ... in slice order) + beta * out[i]
__global__ void __launch_bounds__(EW_THREADS)
k_reduce_slices(const float* __restrict__ part, int slices, int64_t n, float scale, float beta, float* __restrict__ out,
                int vec) {
  const int64_t tid = (int64_t)blockIdx.x * EW_THREADS + threadIdx.x;
  if (vec) {
    const int64_t e = tid * 4;
    if (e >= n) return;
    float4 t = *reinterpret_cast<const float4*>(part + e);
    for (int k = 1; k < slices; ++k) {
      const float4 v = *reinterpret_cast<const float4*>(part + (int64_t)k * n + e);
      t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
    }
    float4 r = make_float4(scale * t.x, scale * t.y, scale * t.z, scale * t.w);
    if (beta != 0.f) {
      const float4 o = *reinterpret_cast<const float4*>(out + e);
      r.x += beta * o.x; r.y += beta * o.y; r.z += beta * o.z; r.w += beta * o.w;
    }
    *reinterpret_cast<float4*>(out + e) = r;
  } else {
    if (tid >= n) return;
    float t = part[tid];
    for (int k = 1; k < slices; ++k) t += part[(int64_t)k * n + tid];
    float r = scale * t;
    if (beta != 0.f) r += beta * out[tid];
    out[tid] = r;
  }
}

// ---------------------------------------------------------------- loss value and output cotangent
constexpr int LOSS_UNROLL = 4;
__global__ void __launch_bounds__(EW_THREADS)
k_loss_grad(const float* __restrict__ xL, const float* __restrict__ t, int64_t n, float cot_scale,
            float* __restrict__ hL, double* __restrict__ partial, int vec) {
  __shared__ double red[EW_WAVES];
  double acc = 0.0;
  const int64_t tid = (int64_t)blockIdx.x * EW_THREADS + threadIdx.x, stride = (int64_t)gridDim.x * EW_THREADS;
  int64_t done = 0;
  if (vec) {  // all three arrays 16-byte aligned
    const int64_t n4 = n >> 2;
    // a wavefront takes LOSS_UNROLL KiB of each array per trip (one contiguous stretch: a thread's quads are 64
    // quads apart), all of it in flight before the first use; the trips of all wavefronts interleave
    const int lane = threadIdx.x & 63;
    for (int64_t q = global_wave() * (64 * LOSS_UNROLL) + lane; q - lane < n4; q += total_waves() * (64 * LOSS_UNROLL)) {
      f4v a[LOSS_UNROLL], b[LOSS_UNROLL];
#pragma unroll
      for (int u = 0; u < LOSS_UNROLL; ++u) {
        const int64_t qu = q + u * 64;
        a[u] = f4v{0.f, 0.f, 0.f, 0.f};
        b[u] = a[u];
        if (qu < n4) {
          a[u] = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(xL + 4 * qu));
          b[u] = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(t + 4 * qu));
        }
      }
#pragma unroll
      for (int u = 0; u < LOSS_UNROLL; ++u) {
        const int64_t qu = q + u * 64;
        if (qu < n4) {
          const f4v r = a[u] - b[u];
          __builtin_nontemporal_store(r * cot_scale, reinterpret_cast<f4v*>(hL + 4 * qu));
          acc += (double)r.x * (double)r.x + (double)r.y * (double)r.y;
          acc += (double)r.z * (double)r.z + (double)r.w * (double)r.w;
        }
      }
    }
    done = n4 << 2;
  }
  for (int64_t e = done + tid; e < n; e += stride) {
    float r = xL[e] - t[e];
    hL[e] = cot_scale * r;
    acc += (double)r * (double)r;
  }
  // fixed tree: lanes of a wavefront by halving distances, then the wavefronts in order
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = red[0];
    for (int w = 1; w < EW_WAVES; ++w) s += red[w];
    partial[blockIdx.x] = s;
  }
}

// Sum of the per-workgroup partials in a fixed order (thread t takes partials t, t + 256, ...;
// then a fixed tree), so the loss does not depend on scheduling.
__global__ void __launch_bounds__(EW_THREADS)
k_loss_final(const double* __restrict__ partial, int n_partial, double factor, float* __restrict__ loss,
             uint32_t* __restrict__ nonfinite) {
  __shared__ double red[EW_THREADS];
  double acc = 0.0;
  for (int i = threadIdx.x; i < n_partial; i += EW_THREADS) acc += partial[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = EW_THREADS / 2; s > 0; s >>= 1) {
    if (threadIdx.x < (unsigned)s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const float v = (float)(factor * red[0]);
    if (loss) *loss = v;
    if (nonfinite) *nonfinite = (fabsf(v) <= 3.402823466e38f) ? 0u : 1u;  // NaN or infinity
  }
}

// ---------------------------------------------------------------- slope from a stored activation
// out = h * (act > 0 ? 1 : alpha): the activation's vjp when the activation itself was kept
// (x > 0 <=> z > 0 for a leaky ReLU with alpha > 0).
__global__ void __launch_bounds__(EW_THREADS)
k_scale_by_act_slope(const float* __restrict__ h, const float* __restrict__ act, int64_t n, float alpha,
                     float* __restrict__ out, int vec) {
  const int64_t tid = (int64_t)blockIdx.x * EW_THREADS + threadIdx.x, stride = (int64_t)gridDim.x * EW_THREADS;
  int64_t done = 0;
  if (vec) {
    const int64_t n4 = n >> 2;
    for (int64_t q = tid; q < n4; q += stride) {
      const float4 a = *reinterpret_cast<const float4*>(act + 4 * q), v = *reinterpret_cast<const float4*>(h + 4 * q);
      *reinterpret_cast<float4*>(out + 4 * q) =
          make_float4(v.x * (a.x > 0.f ? 1.f : alpha), v.y * (a.y > 0.f ? 1.f : alpha), v.z * (a.z > 0.f ? 1.f : alpha),
                      v.w * (a.w > 0.f ? 1.f : alpha));
    }
    done = n4 << 2;
  }
  for (int64_t e = done + tid; e < n; e += stride) out[e] = h[e] * (act[e] > 0.f ? 1.f : alpha);
}

// ---------------------------------------------------------------- residual of an approximate inverse
__global__ void __launch_bounds__(EW_THREADS)
k_identity_residual(const float* __restrict__ E, int n, double* __restrict__ partial) {
  __shared__ double red[EW_THREADS];
  const int64_t total = (int64_t)n * n;
  double acc = 0.0;
  for (int64_t e = (int64_t)blockIdx.x * EW_THREADS + threadIdx.x; e < total; e += (int64_t)gridDim.x * EW_THREADS) {
    const int64_t r = e / n, c = e - r * n;
    const float d = E[e] - (r == c ? 1.f : 0.f);
    acc += (double)d * (double)d;
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = EW_THREADS / 2; s > 0; s >>= 1) {
    if (threadIdx.x < (unsigned)s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

__global__ void __launch_bounds__(EW_THREADS)
k_identity_residual_final(const double* __restrict__ partial, int n_partial, float* __restrict__ out) {
  __shared__ double red[EW_THREADS];
  double acc = 0.0;
  for (int i = threadIdx.x; i < n_partial; i += EW_THREADS) acc += partial[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = EW_THREADS / 2; s > 0; s >>= 1) {
    if (threadIdx.x < (unsigned)s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const float r = (float)sqrt(red[0]);
    if (!(r <= *out)) *out = r;  // running maximum; a NaN residual is kept
  }
}

// The same for several matrices `stride` floats apart (blockIdx.y selects one): partial sums of matrix j
// in partial[j * gridDim.x ..]; the final kernel folds the largest of the residuals into *out.
__global__ void __launch_bounds__(EW_THREADS)
k_identity_residual_sets(const float* __restrict__ E, int64_t stride, int n, double* __restrict__ partial, float eye) {
  __shared__ double red[EW_WAVES];
  const float* Ej = E + (int64_t)blockIdx.y * stride;
  const int64_t total = (int64_t)n * n;
  double acc = 0.0;
  // whole rows are dealt to the threads in runs of four elements when the rows allow it (no division per element)
  if (n % 4 == 0 && ((uintptr_t)Ej & 15) == 0 && total < ((int64_t)1 << 31)) {
    const uint32_t quads = (uint32_t)(total >> 2), per_row = (uint32_t)n >> 2;
    for (uint32_t q = blockIdx.x * EW_THREADS + threadIdx.x; q < quads; q += gridDim.x * EW_THREADS) {
      const uint32_t r = q / per_row, c = 4u * (q - r * per_row);
      const f4v v = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(Ej) + q);
      const float d0 = v.x - (r == c ? eye : 0.f), d1 = v.y - (r == c + 1 ? eye : 0.f), d2 = v.z - (r == c + 2 ? eye : 0.f),
                  d3 = v.w - (r == c + 3 ? eye : 0.f);
      acc += (double)d0 * (double)d0 + (double)d1 * (double)d1;
      acc += (double)d2 * (double)d2 + (double)d3 * (double)d3;
    }
  } else {
    for (int64_t e = (int64_t)blockIdx.x * EW_THREADS + threadIdx.x; e < total; e += (int64_t)gridDim.x * EW_THREADS) {
      const int64_t r = e / n, c = e - r * n;
      const float d = Ej[e] - (r == c ? eye : 0.f);
      acc += (double)d * (double)d;
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = red[0];
    for (int w = 1; w < EW_WAVES; ++w) t += red[w];
    partial[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = t;
  }
}

// one wavefront per matrix (in turns), a fixed tree inside it
__global__ void __launch_bounds__(EW_THREADS)
k_identity_residual_sets_final(const double* __restrict__ partial, int n_partial, int n_sets, float* __restrict__ out) {
  __shared__ float worst[EW_WAVES];
  __shared__ int any_nan[EW_WAVES];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float w = 0.f;
  int bad = 0;
  for (int j = wave; j < n_sets; j += EW_WAVES) {
    double acc = 0.0;
    for (int i = lane; i < n_partial; i += 64) acc += partial[(int64_t)j * n_partial + i];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off);
    const float r = (float)sqrt(acc);
    if (r != r) bad = 1;
    else if (r > w) w = r;
  }
  if (lane == 0) {
    worst[wave] = w;
    any_nan[wave] = bad;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float r = worst[0];
    int nan = any_nan[0];
    for (int k = 1; k < EW_WAVES; ++k) {
      if (worst[k] > r) r = worst[k];
      nan |= any_nan[k];
    }
    if (nan) r = __builtin_nanf("");
    if (!(r <= *out)) *out = r;  // running maximum; a NaN residual is kept
  }
}

// ---------------------------------------------------------------- copy / fill
__global__ void __launch_bounds__(EW_THREADS)
k_copy(const float* __restrict__ src, float* __restrict__ dst, int64_t n) {
  const int64_t n4 = n >> 2;
  const bool vec = (((uintptr_t)src | (uintptr_t)dst) & 15) == 0;
  int64_t i = (int64_t)blockIdx.x * EW_THREADS + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * EW_THREADS;
  if (vec) {
    // four 16-byte accesses per thread and trip, all loads before the first store, none kept in the caches
    const f4v* s4 = reinterpret_cast<const f4v*>(src);
    f4v* d4 = reinterpret_cast<f4v*>(dst);
    for (int64_t k0 = (int64_t)blockIdx.x * EW_THREADS * 4 + threadIdx.x; k0 < n4; k0 += stride * 4) {
      f4v v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (k0 + u * EW_THREADS < n4) v[u] = __builtin_nontemporal_load(s4 + k0 + u * EW_THREADS);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (k0 + u * EW_THREADS < n4) __builtin_nontemporal_store(v[u], d4 + k0 + u * EW_THREADS);
    }
    for (int64_t k = n4 * 4 + i; k < n; k += stride) dst[k] = src[k];
  } else {
    for (int64_t k = i; k < n; k += stride) dst[k] = src[k];
  }
}

__global__ void __launch_bounds__(EW_THREADS)
k_fill_u32(uint32_t* __restrict__ p, uint32_t value, int64_t n) {
  for (int64_t k = (int64_t)blockIdx.x * EW_THREADS + threadIdx.x; k < n; k += (int64_t)gridDim.x * EW_THREADS)
    p[k] = value;
}

// ---------------------------------------------------------------- operand-stream probe
// Load-only model of a GEMM workgroup: the workgroup of output tile (tm, tn) reads the R x K row
// panels A[tm*R ..][:] and B[tn*R ..][:] exactly as the tiled kernels do (dwordx4 per lane, 128
// floats of k per pass, two passes in flight) and keeps only a checksum. What it measures is the
// rate at which the CUs can pull operand panels through their L1 caches, which is what bounds the
// small-batch products.
template <int R>
__global__ void __launch_bounds__(EW_THREADS)
k_operand_stream(const float* __restrict__ A, const float* __restrict__ B, int K, int tiles_m, int tiles_n,
                 float* __restrict__ sink) {
  constexpr int RPP = EW_THREADS / 32;  // rows per pass: 32 lanes x 16 B cover 128 floats of one row
  constexpr int P = R / RPP;
  static_assert(R % RPP == 0, "tile rows must be a multiple of the rows per pass");
  const int nblocks = tiles_m * tiles_n;
  const int xcd = blockIdx.x % 8, local = blockIdx.x / 8;
  const int id = xcd * (nblocks / 8) + (xcd < nblocks % 8 ? xcd : nblocks % 8) + local;  // one XCD per id range
  const int tm = id % tiles_m, tn = id / tiles_m;
  const int row = threadIdx.x / 32, col = (threadIdx.x % 32) * 4;
  const float* pa = A + (size_t)(tm * R + row) * K + col;
  const float* pb = B + (size_t)(tn * R + row) * K + col;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int k = 0; k < K; k += 256) {
    float4 va[2][P], vb[2][P];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int q = 0; q < P; ++q) {
        va[u][q] = *reinterpret_cast<const float4*>(pa + (size_t)q * RPP * K + k + u * 128);
        vb[u][q] = *reinterpret_cast<const float4*>(pb + (size_t)q * RPP * K + k + u * 128);
      }
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int q = 0; q < P; ++q) {
        acc.x += va[u][q].x + vb[u][q].x;
        acc.y += va[u][q].y + vb[u][q].y;
        acc.z += va[u][q].z + vb[u][q].z;
        acc.w += va[u][q].w + vb[u][q].w;
      }
  }
  sink[(size_t)blockIdx.x * EW_THREADS + threadIdx.x] = acc.x + acc.y + acc.z + acc.w;
}

}  // namespace

// ------------------------------------------------------------------------------------ launchers

inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline int ew_blocks_v4(int64_t n) { return ew_blocks((n + 255) >> 8, EW_WAVES * VUNROLL); }

hipError_t ew_bias_act_mask(const float* zin, const float* bias, int64_t rows, int d, float alpha, float* x,
                            uint64_t* mask, hipStream_t stream) {
  int64_t n = rows * d;
  if (n <= 0) return hipSuccess;
  if (al16(zin) && al16(x) && (!bias || (al16(bias) && d % 4 == 0))) {
    if (bias)
      hipLaunchKernelGGL(k_bias_act_mask_v4<true>, dim3(ew_blocks_v4(n)), dim3(EW_THREADS), 0, stream, zin, bias, n, d,
                         alpha, x, mask);
    else
      hipLaunchKernelGGL(k_bias_act_mask_v4<false>, dim3(ew_blocks_v4(n)), dim3(EW_THREADS), 0, stream, zin, bias, n, d,
                         alpha, x, mask);
    return hipGetLastError();
  }
  int blocks = ew_blocks((n + 63) >> 6, EW_WAVES * UNROLL);
  if (bias)
    hipLaunchKernelGGL(k_bias_act_mask<true>, dim3(blocks), dim3(EW_THREADS), 0, stream, zin, bias, n, d, alpha, x,
                       mask);
  else
    hipLaunchKernelGGL(k_bias_act_mask<false>, dim3(blocks), dim3(EW_THREADS), 0, stream, zin, bias, n, d, alpha, x,
                       mask);
  return hipGetLastError();
}

hipError_t ew_mask_from_act(const float* x, int64_t n, uint64_t* mask, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  if (al16(x)) {
    hipLaunchKernelGGL(k_mask_from_act_v4, dim3(ew_blocks_v4(n)), dim3(EW_THREADS), 0, stream, x, n, mask);
    return hipGetLastError();
  }
  int blocks = ew_blocks((n + 63) >> 6, EW_WAVES * UNROLL);
  hipLaunchKernelGGL(k_mask_from_act, dim3(blocks), dim3(EW_THREADS), 0, stream, x, n, mask);
  return hipGetLastError();
}

hipError_t ew_rev_scale(const float* h, const uint64_t* mask, int64_t n, float alpha, float* ct_z,
                        hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  if (al16(h) && al16(ct_z)) {
    hipLaunchKernelGGL(k_rev_scale_v4, dim3(ew_blocks_v4(n)), dim3(EW_THREADS), 0, stream, h, mask, n, alpha, ct_z);
    return hipGetLastError();
  }
  int blocks = ew_blocks((n + 63) >> 6, EW_WAVES * UNROLL);
  hipLaunchKernelGGL(k_rev_scale, dim3(blocks), dim3(EW_THREADS), 0, stream, h, mask, n, alpha, ct_z);
  return hipGetLastError();
}

size_t ew_frag_scan_words(int64_t n) {
  const int64_t n_words = n > 0 ? (n + 63) >> 6 : 0;
  const int64_t chunks = (n_words + SCAN_CHUNK_WORDS - 1) / SCAN_CHUNK_WORDS;
  return (size_t)(chunks < 1 ? 1 : chunks);
}

hipError_t ew_frag_offsets(const uint64_t* mask, int64_t n, uint32_t* offsets, uint32_t* sums, hipStream_t stream) {
  if (n < 0) return hipErrorInvalidValue;
  const size_t chunks = ew_frag_scan_words(n);
  if (chunks > 0x7FFFFFFFu) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_frag_chunk_sums, dim3((unsigned)chunks), dim3(SCAN_THREADS), 0, stream, mask, n, sums);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_frag_offsets, dim3((unsigned)chunks), dim3(SCAN_THREADS), 0, stream, mask, n, offsets, sums);
  return hipGetLastError();
}

hipError_t ew_frag_offsets_layers(const FragLayer* layers, int n_layers, int64_t max_n, hipStream_t stream) {
  if (n_layers <= 0) return hipSuccess;
  if (max_n < 0 || n_layers > 65535) return hipErrorInvalidValue;
  const size_t chunks = ew_frag_scan_words(max_n);
  if (chunks > 0x7FFFFFFFu) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_frag_chunk_sums_layers, dim3((unsigned)chunks, n_layers), dim3(SCAN_THREADS), 0, stream, layers);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_frag_offsets_layers, dim3((unsigned)chunks, n_layers), dim3(SCAN_THREADS), 0, stream, layers);
  return hipGetLastError();
}

hipError_t ew_frag_bases(const uint32_t* const* count_ptrs, int n_relu, uint64_t* bases, uint64_t* total,
                         hipStream_t stream) {
  hipLaunchKernelGGL(k_frag_bases, dim3(1), dim3(SCAN_THREADS), 0, stream, count_ptrs, n_relu, bases, total);
  return hipGetLastError();
}

hipError_t ew_frag_compact(const float* h, const uint64_t* mask, const uint32_t* offsets, int64_t n, float* frag,
                           const uint64_t* base, uint64_t capacity, int32_t* overflow_flag, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  if (al16(h)) {
    hipLaunchKernelGGL(k_frag_compact_v4, dim3(ew_blocks_v4(n)), dim3(EW_THREADS), 0, stream, h, mask, offsets, n, frag,
                       base, capacity, overflow_flag);
    return hipGetLastError();
  }
  int blocks = ew_blocks((n + 63) >> 6, EW_WAVES * UNROLL);
  hipLaunchKernelGGL(k_frag_compact, dim3(blocks), dim3(EW_THREADS), 0, stream, h, mask, offsets, n, frag, base,
                     capacity, overflow_flag);
  return hipGetLastError();
}

hipError_t ew_vijp_epilogue(const float* z, float* ct_z, int64_t rows, int d, float alpha, const uint64_t* mask,
                            const uint32_t* offsets, const float* frag, const uint64_t* base, uint64_t capacity,
                            float* x, float* h_y, unsigned long long* mismatches, hipStream_t stream) {
  int64_t n = rows * d;
  if (n <= 0) return hipSuccess;
  if (alpha == 0.f && (!mask || !offsets || !frag)) return hipErrorInvalidValue;
  if (al16(z) && al16(ct_z) && al16(x) && al16(h_y)) {
    const int vb = ew_blocks_v4(n);
    if (alpha == 0.f)
      hipLaunchKernelGGL(k_vijp_epilogue_v4<true>, dim3(vb), dim3(EW_THREADS), 0, stream, z, ct_z, n, alpha, 0.f, mask,
                         offsets, frag, base, capacity, x, h_y, mismatches);
    else
      hipLaunchKernelGGL(k_vijp_epilogue_v4<false>, dim3(vb), dim3(EW_THREADS), 0, stream, z, ct_z, n, alpha,
                         1.0f / alpha, mask, offsets, frag, base, capacity, x, h_y, mismatches);
    return hipGetLastError();
  }
  int blocks = ew_blocks((n + 63) >> 6, EW_WAVES * UNROLL);
  if (alpha == 0.f) {
    hipLaunchKernelGGL(k_vijp_epilogue<true>, dim3(blocks), dim3(EW_THREADS), 0, stream, z, ct_z, n, alpha, 0.f,
                       mask, offsets, frag, base, capacity, x, h_y, mismatches);
  } else {
    hipLaunchKernelGGL(k_vijp_epilogue<false>, dim3(blocks), dim3(EW_THREADS), 0, stream, z, ct_z, n, alpha,
                       1.0f / alpha, mask, offsets, frag, base, capacity, x, h_y, mismatches);
  }
  return hipGetLastError();
}

hipError_t ew_colsum(const float* a, int64_t rows, int d, float scale, float* out, hipStream_t stream) {
  if (d <= 0) return hipSuccess;
  int blocks = (d + COLSUM_COLS - 1) / COLSUM_COLS;
  hipLaunchKernelGGL(k_colsum, dim3(blocks), dim3(COLSUM_COLS * COLSUM_SPLIT), 0, stream, a, rows, rows > 0 ? rows : 1, d, scale,
                     out);
  return hipGetLastError();
}

int ew_colsum_slices(int64_t rows, int d, bool vec) {
  // enough workgroups to keep every memory channel busy (2048 of the 128-bit kernel's, 1024 of the other's),
  // at least 256 or 1024 rows each
  const int col_blocks = vec ? (d + 4 * COLSUM4_QUADS - 1) / (4 * COLSUM4_QUADS) : (d + COLSUM_COLS - 1) / COLSUM_COLS;
  int64_t want = ((vec ? 2048 : 1024) + col_blocks - 1) / col_blocks;
  const int64_t rows_min = vec ? 256 : 1024;
  const int64_t most = (rows + rows_min - 1) / rows_min;
  if (want > most) want = most;
  if (want > COLSUM_MAX_SLICES) want = COLSUM_MAX_SLICES;
  return want < 1 ? 1 : (int)want;
}

hipError_t ew_colsum_wide(const float* a, int64_t rows, int d, float scale, float beta, float* out, float* scratch,
                          hipStream_t stream) {
  if (d <= 0) return hipSuccess;
  const bool vec = d % 4 == 0 && al16(a) && al16(scratch);
  const int slices = ew_colsum_slices(rows, d, vec);
  const int64_t per = (rows + slices - 1) / slices;
  if (vec) {
    const int col_blocks = (d + 4 * COLSUM4_QUADS - 1) / (4 * COLSUM4_QUADS);
    hipLaunchKernelGGL(k_colsum_v4, dim3(col_blocks, slices), dim3(COLSUM4_QUADS * COLSUM4_SPLIT), 0, stream, a, rows,
                       per > 0 ? per : 1, d, 1.f, scratch);
  } else {
    const int col_blocks = (d + COLSUM_COLS - 1) / COLSUM_COLS;
    hipLaunchKernelGGL(k_colsum, dim3(col_blocks, slices), dim3(COLSUM_COLS * COLSUM_SPLIT), 0, stream, a, rows, per > 0 ? per : 1,
                       d, 1.f, scratch);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return ew_reduce_slices(scratch, slices, d, scale, beta, out, stream);
}

// ---------------------------------------------------------------- column sums without a workspace argument
// The row-range partial sums of ew_colsum_wide in an array that belongs to the library's code object
// instead of a buffer somebody allocated: for callers that cannot allocate. Every GPU holds its own
// copy of the array from the moment the library is loaded there until the process ends; its address on
// a GPU is looked up once, with that GPU current, and kept. In host code the array's name is only a
// handle for that lookup: kernels, and anything else that touches the memory, get the looked-up pointer.
constexpr size_t STATIC_SCRATCH_FLOATS = (size_t)1 << 20;  // 4 MiB per GPU
static __device__ __align__(256) float scratch[STATIC_SCRATCH_FLOATS];

constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
static float* g_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES];
static std::mutex g_scratch_lock;

static hipError_t static_scratch_ptr(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> guard(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

size_t ew_colsum_static_floats() { return STATIC_SCRATCH_FLOATS; }

hipError_t ew_colsum_wide_static(const float* a, int64_t rows, int d, float scale, float* out, hipStream_t stream,
                                 bool* too_large) {
  *too_large = false;
  if (d <= 0) return hipSuccess;
  // the partial sums take slices * d floats; the array is 256-byte aligned, so the choice of kernel (and with
  // it the slice count and the summation order) is the one ew_colsum_wide makes for an aligned workspace
  const bool vec = d % 4 == 0 && al16(a);
  if ((size_t)ew_colsum_slices(rows, d, vec) * (size_t)d > STATIC_SCRATCH_FLOATS) {
    *too_large = true;
    return hipSuccess;
  }
  float* work = nullptr;
  hipError_t e = static_scratch_ptr(&work);
  if (e != hipSuccess) return e;
  // every slot the reduction reads is written by this call's first kernel: nothing has to start at zero
  return ew_colsum_wide(a, rows, d, scale, 0.f, out, work, stream);
}

hipError_t ew_reduce_slices(const float* part, int slices, int64_t n, float scale, float beta, float* out, hipStream_t stream) {
  if (n <= 0 || slices <= 0) return hipSuccess;
  if (n <= 8192 && slices >= 32) {
    hipLaunchKernelGGL(k_reduce_slices_short, dim3((unsigned)((n + REDUCE_ELEMS - 1) / REDUCE_ELEMS)),
                       dim3(REDUCE_ELEMS * REDUCE_GROUPS), 0, stream, part, slices, n, scale, beta, out);
    return hipGetLastError();
  }
  const int vec = (n % 4 == 0) && al16(part) && al16(out);
  const int64_t threads = vec ? n / 4 : n;
  hipLaunchKernelGGL(k_reduce_slices, dim3((unsigned)((threads + EW_THREADS - 1) / EW_THREADS)), dim3(EW_THREADS), 0, stream,
                     part, slices, n, scale, beta, out, vec);
  return hipGetLastError();
}

hipError_t ew_loss_grad(const float* xL, const float* t, int64_t rows, int d, float scale, float* hL, float* loss,
                        double* scratch, hipStream_t stream, uint32_t* nonfinite) {
  int64_t n = rows * d;
  if (n <= 0 || rows <= 0) return hipErrorInvalidValue;
  // scale and 1/rows are folded into one fp32 factor; with a power-of-two scale this is the
  // correctly rounded scale/rows either way
  float cot_scale = scale / (float)rows;
  const int vec = al16(xL) && al16(t) && al16(hL);
  // one workgroup per LOSS_UNROLL quads per thread, up to LOSS_BLOCKS of them (64 per CU)
  int64_t want = ((vec ? (n + 3) / 4 : n) + (int64_t)EW_THREADS * LOSS_UNROLL - 1) / ((int64_t)EW_THREADS * LOSS_UNROLL);
  const int blocks = (int)(want < 1 ? 1 : (want > LOSS_BLOCKS ? LOSS_BLOCKS : want));
  hipLaunchKernelGGL(k_loss_grad, dim3(blocks), dim3(EW_THREADS), 0, stream, xL, t, n, cot_scale, hL, scratch, vec);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (loss || nonfinite) {
    hipLaunchKernelGGL(k_loss_final, dim3(1), dim3(EW_THREADS), 0, stream, scratch, blocks, 0.5 / (double)rows, loss, nonfinite);
    e = hipGetLastError();
  }
  return e;
}

hipError_t ew_scale_by_act_slope(const float* h, const float* act, int64_t n, float alpha, float* out, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  const int vec = al16(h) && al16(act) && al16(out);
  hipLaunchKernelGGL(k_scale_by_act_slope, dim3(ew_blocks((n + 3) / 4, EW_THREADS * 4)), dim3(EW_THREADS), 0, stream, h, act, n,
                     alpha, out, vec);
  return hipGetLastError();
}

hipError_t ew_identity_residual(const float* E, int n, double* scratch, float* out, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  int64_t want = ((int64_t)n * n + EW_THREADS - 1) / EW_THREADS;
  const int blocks = (int)(want > LOSS_BLOCKS ? LOSS_BLOCKS : want);
  hipLaunchKernelGGL(k_identity_residual, dim3(blocks), dim3(EW_THREADS), 0, stream, E, n, scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_identity_residual_final, dim3(1), dim3(EW_THREADS), 0, stream, scratch, blocks, out);
  return hipGetLastError();
}

hipError_t ew_identity_residual_sets(const float* E, int64_t stride, int n_sets, int n, double* scratch, float* out,
                                     hipStream_t stream, bool minus_identity) {
  if (n <= 0 || n_sets <= 0) return hipSuccess;
  if (n_sets > LOSS_BLOCKS) return hipErrorInvalidValue;
  int64_t want = ((int64_t)n * n + EW_THREADS - 1) / EW_THREADS;
  int64_t cap = LOSS_BLOCKS / n_sets;  // the scratch holds LOSS_BLOCKS doubles in all
  if (cap > 256) cap = 256;            // a workgroup per CU and matrix is plenty; the final kernel reads them all
  const int blocks = (int)(want > cap ? cap : want);
  hipLaunchKernelGGL(k_identity_residual_sets, dim3(blocks, n_sets), dim3(EW_THREADS), 0, stream, E, stride, n, scratch,
                     minus_identity ? 1.f : 0.f);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_identity_residual_sets_final, dim3(1), dim3(EW_THREADS), 0, stream, scratch, blocks, n_sets, out);
  return hipGetLastError();
}

hipError_t ew_copy(const float* src, float* dst, int64_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  int blocks = ew_blocks((n + 3) / 4, EW_THREADS * 4);
  hipLaunchKernelGGL(k_copy, dim3(blocks), dim3(EW_THREADS), 0, stream, src, dst, n);
  return hipGetLastError();
}

hipError_t ew_operand_stream(const float* A, const float* B, int M, int N, int K, int tile, float* sink,
                             hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || M % tile || N % tile || K % 256 || !al16(A) || !al16(B)) return hipErrorInvalidValue;
  const int tiles_m = M / tile, tiles_n = N / tile;
  const dim3 grid(tiles_m * tiles_n), block(EW_THREADS);
  switch (tile) {
    case 16: hipLaunchKernelGGL(k_operand_stream<16>, grid, block, 0, stream, A, B, K, tiles_m, tiles_n, sink); break;
    case 32: hipLaunchKernelGGL(k_operand_stream<32>, grid, block, 0, stream, A, B, K, tiles_m, tiles_n, sink); break;
    case 64: hipLaunchKernelGGL(k_operand_stream<64>, grid, block, 0, stream, A, B, K, tiles_m, tiles_n, sink); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t ew_fill_u32(uint32_t* p, uint32_t value, int64_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  int blocks = ew_blocks(n, EW_THREADS * 4);
  hipLaunchKernelGGL(k_fill_u32, dim3(blocks), dim3(EW_THREADS), 0, stream, p, value, n);
  return hipGetLastError();
}

}  // namespace mw
