// Gather kernels that turn a channels-last convolution into the library's GEMMs, and the small
// triangular inverse behind the convolution's vijp (lemma on submersive convolutional layers).
//
// Activations are [B][H][W][C] fp32, kernels [k][k][C][C'] (tap-major, then input channel, then
// output channel), one stride s and padding p for both spatial dimensions. Row r of a patch
// matrix is output position (b, i', j'), r = (b * H' + i') * W' + j'; column q = (u * k + v) * C + c.
#include "mw_internal.h"

namespace mw {
namespace {

constexpr int CV_THREADS = 256;

// patches[r][q] = x[b, s i' + u - p, s j' + v - p, c]  (0 outside the image), rows [row0, row0 + n_rows)
// of the layer's patch matrix. One thread per 4 consecutive channels when C % 4 == 0 (VEC), else per element.
template <bool VEC>
__global__ void __launch_bounds__(CV_THREADS)
k_im2col(const float* __restrict__ x, int H, int W, int C, int Ho, int Wo, int k, int s, int p, int64_t row0,
         int64_t n_rows, float* __restrict__ patches) {
  const int K = k * k * C;
  const int per_row = VEC ? K / 4 : K;
  const int64_t total = n_rows * per_row;
  for (int64_t t = (int64_t)blockIdx.x * CV_THREADS + threadIdx.x; t < total; t += (int64_t)gridDim.x * CV_THREADS) {
    const int64_t rl = t / per_row;
    const int q = (int)(t - rl * per_row) * (VEC ? 4 : 1);
    const int64_t r = row0 + rl;
    const int j = (int)(r % Wo);
    const int64_t bi = r / Wo;
    const int i = (int)(bi % Ho);
    const int64_t b = bi / Ho;
    const int tap = q / C, c = q - tap * C;
    const int u = tap / k, v = tap - u * k;
    const int y = s * i + u - p, xx = s * j + v - p;
    const bool in = y >= 0 && y < H && xx >= 0 && xx < W;
    const int64_t src = ((b * H + y) * (int64_t)W + xx) * C + c;
    if (VEC) {
      float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
      if (in) val = *reinterpret_cast<const float4*>(x + src);
      *reinterpret_cast<float4*>(patches + rl * K + q) = val;
    } else {
      patches[rl * K + q] = in ? x[src] : 0.f;
    }
  }
}

// Input cotangent from patch cotangents (the transpose of im2col, as a gather so that the sum
// has a fixed order): h[b, y, x, c] = sum over the taps (u, v) and output positions (i', j') with
// s i' + u - p = y, s j' + v - p = x of dpatches[(b, i', j')][(u, v, c)], taps in ascending order.
// Covers the images [img0, img0 + n_img); dpatches holds exactly their rows.
template <bool VEC>
__global__ void __launch_bounds__(CV_THREADS)
k_col2im(const float* __restrict__ dpatches, int H, int W, int C, int Ho, int Wo, int k, int s, int p, int64_t img0,
         int64_t n_img, float* __restrict__ h) {
  const int K = k * k * C;
  const int per_px = VEC ? C / 4 : C;
  const int64_t total = n_img * H * W * per_px;
  for (int64_t t = (int64_t)blockIdx.x * CV_THREADS + threadIdx.x; t < total; t += (int64_t)gridDim.x * CV_THREADS) {
    const int64_t px = t / per_px;
    const int c = (int)(t - px * per_px) * (VEC ? 4 : 1);
    const int xx = (int)(px % W);
    const int64_t by = px / W;
    const int y = (int)(by % H);
    const int64_t bl = by / H;  // image within the chunk
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int u = 0; u < k; ++u) {
      const int yy = y + p - u;
      if (yy < 0 || yy % s != 0) continue;
      const int i = yy / s;
      if (i >= Ho) continue;
      for (int v = 0; v < k; ++v) {
        const int xv = xx + p - v;
        if (xv < 0 || xv % s != 0) continue;
        const int j = xv / s;
        if (j >= Wo) continue;
        const int64_t r = (bl * Ho + i) * (int64_t)Wo + j;
        const float* src = dpatches + r * K + (u * k + v) * C + c;
        if (VEC) {
          const float4 d = *reinterpret_cast<const float4*>(src);
          acc.x += d.x; acc.y += d.y; acc.z += d.z; acc.w += d.w;
        } else {
          acc.x += src[0];
        }
      }
    }
    float* dst = h + ((img0 + bl) * H * (int64_t)W + (int64_t)y * W + xx) * C + c;
    if (VEC) *reinterpret_cast<float4*>(dst) = acc;
    else dst[0] = acc.x;
  }
}

// out[r][c'] = h[b, s i', s j', c'] for c' < Co: the right-hand sides of the per-position channel solve.
__global__ void __launch_bounds__(CV_THREADS)
k_strided_gather(const float* __restrict__ h, int H, int W, int C, int Ho, int Wo, int Co, int s, int64_t n_rows,
                 float* __restrict__ out) {
  const int64_t total = n_rows * Co;
  for (int64_t t = (int64_t)blockIdx.x * CV_THREADS + threadIdx.x; t < total; t += (int64_t)gridDim.x * CV_THREADS) {
    const int64_t r = t / Co;
    const int c = (int)(t - r * Co);
    const int j = (int)(r % Wo);
    const int64_t bi = r / Wo;
    const int i = (int)(bi % Ho);
    const int64_t b = bi / Ho;
    out[t] = h[((b * H + (int64_t)s * i) * W + (int64_t)s * j) * C + c];
  }
}

// Inverse of the lower-triangular tap T[c][c''] = w[p][p][c][c''] (c, c'' < n; row stride ld), one
// thread per column by forward substitution. Raises *flag if an entry above the diagonal is not
// zero or a diagonal entry is zero (conditions (ii), (iii) of the lemma).
__global__ void __launch_bounds__(1024)
k_tri_inverse(const float* __restrict__ T, int64_t ld, int n, float* __restrict__ Tinv, int32_t* __restrict__ flag) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  bool bad = (T[(int64_t)j * ld + j] == 0.f);
  for (int c = 0; c < j; ++c) bad = bad || (T[(int64_t)c * ld + j] != 0.f);  // row c < column j must be 0
  if (bad) {
    *flag = 1;
    for (int i = 0; i < n; ++i) Tinv[(int64_t)i * n + j] = (i == j) ? 1.f : 0.f;
    return;
  }
  for (int i = 0; i < j; ++i) Tinv[(int64_t)i * n + j] = 0.f;
  Tinv[(int64_t)j * n + j] = 1.f / T[(int64_t)j * ld + j];
  for (int i = j + 1; i < n; ++i) {
    float acc = 0.f;
    for (int t = j; t < i; ++t) acc += T[(int64_t)i * ld + t] * Tinv[(int64_t)t * n + j];
    Tinv[(int64_t)i * n + j] = -acc / T[(int64_t)i * ld + i];
  }
}

// The same with the columns' partial results in LDS (one wavefront per 64 columns, x[i][lane]): the
// entries of T are the same for every lane (scalar loads), and the running column no longer goes
// through global memory between one row and the next. Needs n * 256 bytes of LDS.
__global__ void __launch_bounds__(64)
k_tri_inverse_lds(const float* __restrict__ T, int64_t ld, int n, float* __restrict__ Tinv, int32_t* __restrict__ flag) {
  extern __shared__ __align__(16) float xs[];  // [n][64]
  const int lane = threadIdx.x;
  const int j = blockIdx.x * 64 + lane;
  const bool live = j < n;
  bool bad = false;
  if (live) {
    bad = (T[(int64_t)j * ld + j] == 0.f);
    for (int c = 0; c < j; ++c) bad = bad || (T[(int64_t)c * ld + j] != 0.f);  // row c < column j must be 0
    if (bad) *flag = 1;
  }
  const int j0 = blockIdx.x * 64;  // the first row in which any column of this wavefront is non-zero
  for (int i = j0; i < n; ++i) {
    float acc = 0.f;
    for (int t = j0; t < i; ++t) acc += T[(int64_t)i * ld + t] * xs[t * 64 + lane];  // xs[t] = 0 above the diagonal
    float v;
    if (i < j) v = 0.f;
    else if (i == j) v = 1.f / T[(int64_t)i * ld + i];
    else v = -acc / T[(int64_t)i * ld + i];
    if (bad) v = (i == j) ? 1.f : 0.f;
    xs[i * 64 + lane] = v;
  }
  if (live) {
    for (int i = 0; i < j0; ++i) Tinv[(int64_t)i * n + j] = 0.f;
    for (int i = j0; i < n; ++i) Tinv[(int64_t)i * n + j] = xs[i * 64 + lane];
  }
}

// Blocked inverse, first step: workgroup b inverts the 64 x 64 diagonal block b of T into the same
// block of Tinv (row stride n) by the substitution above, 64 columns side by side in LDS.
__global__ void __launch_bounds__(64)
k_tri_inverse_diag64(const float* __restrict__ T, int64_t ld, int n, float* __restrict__ Tinv, int32_t* __restrict__ flag) {
  __shared__ float xs[64 * 64];
  const int lane = threadIdx.x;
  const int o = blockIdx.x * 64;
  const float* Tb = T + (int64_t)o * ld + o;
  float* Ib = Tinv + (int64_t)o * n + o;
  const int j = lane;
  const bool bad = (Tb[(int64_t)j * ld + j] == 0.f);
  if (bad) *flag = 1;
  for (int i = 0; i < 64; ++i) {
    float acc = 0.f;
    for (int t = 0; t < i; ++t) acc += Tb[(int64_t)i * ld + t] * xs[t * 64 + lane];
    float v;
    if (i < j) v = 0.f;
    else if (i == j) v = 1.f / Tb[(int64_t)i * ld + i];
    else v = -acc / Tb[(int64_t)i * ld + i];
    if (bad) v = (i == j) ? 1.f : 0.f;
    xs[i * 64 + lane] = v;
  }
  for (int i = 0; i < 64; ++i) Ib[(int64_t)i * n + j] = xs[i * 64 + lane];
}

// Blocked inverse, last step: everything above the diagonal of Tinv is zero (the blocks there served as
// scratch), and T itself must have been zero there (*flag raised otherwise).
__global__ void __launch_bounds__(256)
k_tri_inverse_finish(const float* __restrict__ T, int64_t ld, int n, float* __restrict__ Tinv, int32_t* __restrict__ flag) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)n * n) return;
  const int c = (int)(i / n), cp = (int)(i % n);
  if (c < cp) {
    if (T[(int64_t)c * ld + cp] != 0.f) *flag = 1;
    Tinv[(int64_t)c * n + cp] = 0.f;
  }
}

// T[c][c'] = 0 for c < c' < n (row stride ld): the entries a training step must leave at zero
__global__ void __launch_bounds__(256) k_zero_above_diagonal(float* __restrict__ T, int64_t ld, int n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)n * n) return;
  const int c = (int)(i / n), cp = (int)(i % n);
  if (c < cp) T[(int64_t)c * ld + cp] = 0.f;
}

inline int cv_blocks(int64_t work_items) {
  int64_t b = (work_items + CV_THREADS - 1) / CV_THREADS;
  if (b < 1) b = 1;
  if (b > 256 * 16) b = 256 * 16;
  return (int)b;
}
inline bool al16p(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// rows of `w4` float4 each, from one row stride to another (the fragment store of the 1-D layers: the
// first positions of every block of a cotangent, out of it in Phase II and back into it in Phase III)
__global__ void __launch_bounds__(256)
k_copy_rows(const float* __restrict__ src, int64_t src_ld, float* __restrict__ dst, int64_t dst_ld, int64_t rows, int w4) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= rows * w4) return;
  const int64_t r = i / w4;
  const int c = (int)(i - r * w4);
  *reinterpret_cast<float4*>(dst + r * dst_ld + 4 * c) = *reinterpret_cast<const float4*>(src + r * src_ld + 4 * c);
}

// Weights regrouped for the input-cotangent products. Taps are classed by (ky mod s, kx mod s); class
// (ry, rx) holds, for tap slots ky' < nty, kx' < ntx (ky = ry + s (nty - 1 - ky'), likewise kx), the
// matrix [C_out][C_in] = w[ky][kx]^T, slots in row-major order, classes in (ry, rx) order.
__device__ __forceinline__ int taps_of_class(int k, int s, int r) { return r < k ? (k - r + s - 1) / s : 0; }

__global__ void __launch_bounds__(256)
k_pack_rev_weights(const float* __restrict__ w, int kh, int kw, int s, int Cin, int Cout, float* __restrict__ wrev) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t n = (int64_t)kh * kw * Cin * Cout;
  if (idx >= n) return;
  const int co = (int)(idx % Cout);
  int64_t r = idx / Cout;
  const int ci = (int)(r % Cin);
  r /= Cin;
  const int kx = (int)(r % kw), ky = (int)(r / kw);
  const int ry = ky % s, rx = kx % s;
  const int nty = taps_of_class(kh, s, ry), ntx = taps_of_class(kw, s, rx);
  const int kyp = nty - 1 - ky / s, kxp = ntx - 1 - kx / s;
  int64_t taps_before = 0;  // taps of the classes before (ry, rx)
  for (int a = 0; a < ry; ++a) taps_before += (int64_t)taps_of_class(kh, s, a) * kw;
  for (int b = 0; b < rx; ++b) taps_before += (int64_t)nty * taps_of_class(kw, s, b);
  const int64_t dst = ((taps_before + (int64_t)kyp * ntx + kxp) * Cout + co) * Cin + ci;
  wrev[dst] = w[idx];
}

}  // namespace

hipError_t cv_im2col(const float* x, int H, int W, int C, int Ho, int Wo, int k, int s, int p, int64_t row0,
                     int64_t n_rows, float* patches, hipStream_t stream) {
  if (n_rows <= 0) return hipSuccess;
  const int K = k * k * C;
  if (C % 4 == 0 && al16p(x) && al16p(patches)) {
    hipLaunchKernelGGL(k_im2col<true>, dim3(cv_blocks(n_rows * (K / 4))), dim3(CV_THREADS), 0, stream, x, H, W, C, Ho, Wo, k,
                       s, p, row0, n_rows, patches);
  } else {
    hipLaunchKernelGGL(k_im2col<false>, dim3(cv_blocks(n_rows * K)), dim3(CV_THREADS), 0, stream, x, H, W, C, Ho, Wo, k, s,
                       p, row0, n_rows, patches);
  }
  return hipGetLastError();
}

hipError_t cv_col2im(const float* dpatches, int H, int W, int C, int Ho, int Wo, int k, int s, int p, int64_t img0,
                     int64_t n_img, float* h, hipStream_t stream) {
  if (n_img <= 0) return hipSuccess;
  if (C % 4 == 0 && al16p(dpatches) && al16p(h)) {
    hipLaunchKernelGGL(k_col2im<true>, dim3(cv_blocks(n_img * H * W * (C / 4))), dim3(CV_THREADS), 0, stream, dpatches, H, W,
                       C, Ho, Wo, k, s, p, img0, n_img, h);
  } else {
    hipLaunchKernelGGL(k_col2im<false>, dim3(cv_blocks(n_img * H * W * C)), dim3(CV_THREADS), 0, stream, dpatches, H, W, C,
                       Ho, Wo, k, s, p, img0, n_img, h);
  }
  return hipGetLastError();
}

hipError_t cv_strided_gather(const float* h, int H, int W, int C, int Ho, int Wo, int Co, int s, int64_t n_rows, float* out,
                             hipStream_t stream) {
  if (n_rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_strided_gather, dim3(cv_blocks(n_rows * Co)), dim3(CV_THREADS), 0, stream, h, H, W, C, Ho, Wo, Co, s,
                     n_rows, out);
  return hipGetLastError();
}

hipError_t cv_pack_rev_weights(const float* w, int kh, int kw, int s, int Cin, int Cout, float* wrev, hipStream_t stream) {
  const int64_t n = (int64_t)kh * kw * Cin * Cout;
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_pack_rev_weights, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, w, kh, kw, s, Cin, Cout, wrev);
  return hipGetLastError();
}

hipError_t cv_copy_rows(const float* src, int64_t src_ld, float* dst, int64_t dst_ld, int64_t rows, int width, hipStream_t stream) {
  if (rows <= 0 || width <= 0) return hipSuccess;
  if (width % 4 || src_ld % 4 || dst_ld % 4 || (reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(dst) & 15))
    return hipErrorInvalidValue;
  const int64_t n4 = rows * (width / 4);
  hipLaunchKernelGGL(k_copy_rows, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, stream, src, src_ld, dst, dst_ld, rows, width / 4);
  return hipGetLastError();
}

hipError_t cv_zero_above_diagonal(float* T, int64_t ld, int n, hipStream_t stream) {
  if (n <= 1) return hipSuccess;
  const int64_t total = (int64_t)n * n;
  hipLaunchKernelGGL(k_zero_above_diagonal, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, T, ld, n);
  return hipGetLastError();
}

hipError_t cv_tri_inverse(const float* T, int64_t ld, int n, float* Tinv, int32_t* flag, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  // n = 64 * 2^j, j >= 1: blocked. With T = [A 0; B D], T^{-1} = [A^{-1} 0; -D^{-1} B A^{-1}  D^{-1}]: the 64 x 64
  // diagonal blocks first, then pairs of inverted blocks are joined, doubling the block size each time;
  // X = D^{-1} B is parked in the top right quarter of Tinv, which no diagonal block of any step touches and
  // which the last kernel clears with the rest of the upper triangle.
  if (n >= 128 && n % 64 == 0 && ((n / 64) & (n / 64 - 1)) == 0) {
    const int64_t total = (int64_t)n * n;
    // the joined blocks are read whole: what lies above their diagonals must be zero from the start
    hipLaunchKernelGGL(k_tri_inverse_finish, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, T, ld, n, Tinv, flag);
    hipLaunchKernelGGL(k_tri_inverse_diag64, dim3(n / 64), dim3(64), 0, stream, T, ld, n, Tinv, flag);
    hipError_t e = hipGetLastError();
    for (int m = 64; m < n && e == hipSuccess; m *= 2) {
      for (int o = 0; o < n && e == hipSuccess; o += 2 * m) {
        const float* Ainv = Tinv + (int64_t)o * n + o;
        const float* Dinv = Tinv + (int64_t)(o + m) * n + (o + m);
        const float* B = T + (int64_t)(o + m) * ld + o;
        float* X = Tinv + (int64_t)(o / 2) * n + n / 2;    // pair o / (2 m) gets rows [o / 2, o / 2 + m) of the quarter
        float* Low = Tinv + (int64_t)(o + m) * n + o;
        e = gemm_plain(OP_NN, TILE_AUTO, m, m, m, 1.f, Dinv, n, B, ld, 0.f, X, n, nullptr, stream);
        if (e == hipSuccess) e = gemm_plain(OP_NN, TILE_AUTO, m, m, m, -1.f, X, n, Ainv, n, 0.f, Low, n, nullptr, stream);
      }
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_tri_inverse_finish, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, T, ld, n, Tinv, flag);
    return hipGetLastError();
  }
  const size_t lds = (size_t)n * 64 * sizeof(float);
  if (lds <= 128 * 1024) {
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(k_tri_inverse_lds),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(k_tri_inverse_lds, dim3((n + 63) / 64), dim3(64), lds, stream, T, ld, n, Tinv, flag);
    return hipGetLastError();
  }
  const int threads = n < 1024 ? ((n + 63) / 64) * 64 : 1024;
  hipLaunchKernelGGL(k_tri_inverse, dim3((n + threads - 1) / threads), dim3(threads), 0, stream, T, ld, n, Tinv, flag);
  return hipGetLastError();
}

}  // namespace mw
