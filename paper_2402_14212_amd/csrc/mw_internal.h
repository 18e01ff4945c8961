// Internal host-side interfaces between the translation units of libmoonwalk.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mw {

// tile selectors (same values as MW_TILE_* in the public header)
constexpr int TILE_AUTO = 0, TILE_128 = 1, TILE_64 = 2, TILE_32K4 = 3, TILE_32K8 = 4, TILE_64K2 = 5, TILE_128W8 = 6, TILE_64X128 = 7;
// tiles whose workgroups have eight wavefronts (the others have four)
inline bool tile_has_8_waves(int tile) { return tile == TILE_32K8 || tile == TILE_64K2 || tile == TILE_128W8 || tile == TILE_64X128; }
constexpr int OP_NT = 0, OP_NN = 1, OP_TN = 2;

// Tile choice for an M x N x K product on a 256-CU device. Deterministic in (M, N, K) only, so
// that phase I and phase III compute a layer's pre-activations with the same kernel shape.
int pick_tile(int M, int N, int K);
// tile of a weight-gradient product launched beside a kernel of tile `partner` (TILE_AUTO: alone),
// which is a Phase-III layer kernel (phase3) or backprop's reverse product
int pick_tile_dw(int M, int N, int K, int partner, bool phase3);

// ---- GEMM launchers (gemm_*.hip). All enqueue on `stream` and return the launch status. ----

// C[g] = alpha * op(A[g], B[g]) + beta * D[g], g < n_sets: the same NT or NN product on several operand sets of one
// shape in one launch (gemm_grouped.hip). Pointer tables in device memory; D may be NULL; operands 16-byte aligned,
// row strides multiples of 4 floats.
// + eye * I (eye != 0 needs M == N); bf16 (NN only): operands rounded to bf16 in front of the matrix unit
hipError_t gemm_grouped(int op, int n_sets, int M, int N, int K, float alpha, const float* const* A, int64_t lda,
                        const float* const* B, int64_t ldb, float beta, const float* const* D, float* const* C, int64_t ldc,
                        hipStream_t stream, float eye = 0.f, bool bf16 = false);

// C = alpha * op(A, B) + beta * C + bias (bias indexed by column, may be NULL)
hipError_t gemm_plain(int op, int tile, int M, int N, int K, float alpha, const float* A, int64_t lda,
                      const float* B, int64_t ldb, float beta, float* C, int64_t ldc, const float* bias,
                      hipStream_t stream);

// Xout[M][N] = act(X[M][K] W[N][K]^T + bias); mask (may be NULL) receives the packed signs and
// then requires N % 32 == 0. Zkeep (may be NULL; a debugging aid) receives the pre-activations.
hipError_t gemm_fwd_act(int tile, int M, int N, int K, const float* X, const float* W, const float* bias,
                        float alpha, float* Xout, uint64_t* mask, hipStream_t stream, float* Zkeep = nullptr);

// Phase-II product with the NEXT step's slope folded into the epilogue:
//   h = CTin[M][K] W[K][N];  CT = h .* slope(mask, alpha)  (mask/alpha of the layer whose OUTPUT h is);
//   RAW = h if not NULL; for alpha == 0 the erased entries of h are appended to the fragment store.
struct RevArgs {
  float* CT;
  float* RAW;
  const uint64_t* mask;
  float alpha;
  const uint32_t* offsets;
  float* frag;
  const uint64_t* frag_base;
  uint64_t frag_capacity;
  int32_t* overflow;
};
hipError_t gemm_rev_fused(int tile, int M, int N, int K, const float* CTin, const float* W, const RevArgs& r,
                          hipStream_t stream);
// Hout[M][N] = (H[M][K] .* slope) W[K][N], slope from the stored activation act[M][K] (> 0 ? 1 : alpha)
hipError_t gemm_rev_act(int tile, int M, int N, int K, const float* H, const float* act, float alpha,
                        const float* W, float* Hout, hipStream_t stream);

// dW[M][N] = scale * CTZ[K][M]^T X[K][N];  db[M] = scale * sum_k CTZ[k][M]  (db may be NULL)
hipError_t gemm_dw(int tile, int M, int N, int K, const float* CTZ, const float* X, float scale, float* dW,
                   float* db, hipStream_t stream, float beta = 0.f);
// same with CTZ = Hy .* slope(act), act[K][M] the stored activation of this layer (backprop)
hipError_t gemm_dw_act(int tile, int M, int N, int K, const float* Hy, const float* act, float alpha,
                       const float* X, float scale, float* dW, float* db, hipStream_t stream);

struct VijpArgs {
  const float* X;        // [M][K]   layer input x_{i-1}
  const float* W;        // [N][K]
  const float* bias;     // [N] or NULL
  const float* Hin;      // [M][K]   layer-input cotangent h_{i-1}
  const float* P;        // [N][K]   right inverse
  float alpha;
  const uint64_t* mask;      // packed phase-I signs of this layer
  const uint32_t* offsets;   // ReLU only
  const float* frag;         // ReLU only
  const uint64_t* frag_base; // ReLU only (device scalar)
  uint64_t frag_capacity;
  float* Xout;           // [M][N]
  float* Hout;           // [M][N]
  float* CTZ;            // [M][N]
  unsigned long long* mismatches;  // device counter
};
hipError_t gemm_vijp_dual(int tile, int M, int N, int K, const VijpArgs& a, hipStream_t stream);

// One launch for two independent pieces of the phase-III sweep: layer i's kernel (M x N x K as in
// gemm_vijp_dual) and the weight-gradient product of layer i-1 (gemm_dw's arguments). Either may be
// absent (NULL). Falls back to separate launches when the two cannot share a kernel.
struct DwArgs {
  int M, N, K;          // d_out, d_in, batch
  const float* CTZ;     // [K][M]
  const float* X;       // [K][N]
  float scale;
  float* dW;            // [M][N]
  float* db;            // [M] or NULL
  float beta = 0.f;     // dW = scale * product + beta * dW (same for db): 1 applies an update in place
};
hipError_t gemm_phase3_pair(const VijpArgs* v, int M, int N, int K, const DwArgs* d, hipStream_t stream);

// Phase III for several independent stretches of the network in one launch: n_v layer kernels of one shape
// (M x N x K each, the same alpha) and n_d weight-gradient products of one shape (the same scale and beta; a
// NULL db is skipped), either count may be 0, at most 16 each. Every product gets the bits it gets from
// gemm_phase3_pair. Only for shapes phase3_group_ok accepts and 16-byte aligned operands (else an error,
// nothing launched).
constexpr int MAX_PHASE3_GROUP = 16;
bool phase3_group_ok(int M, int N, int K);
hipError_t gemm_phase3_group(int n_v, const VijpArgs* v, int M, int N, int K, int n_d, const DwArgs* d, hipStream_t stream);

// Backprop's two products of one layer in one launch (both read h .* slope(act)):
//   dW[dout][din] = scale (Hy .* slope)^T Xprev, db = scale * column sums;   Hout[B][din] = (Hy .* slope) W
// Hout == NULL skips the second product (first layer).
struct BpLayerArgs {
  int batch, d_out, d_in;
  const float* Hy;     // [B][d_out]
  const float* act;    // [B][d_out] stored activation of this layer
  float alpha;
  const float* Xprev;  // [B][d_in]
  const float* W;      // [d_out][d_in]
  float scale;
  float* dW;
  float* db;
  float* Hout;         // [B][d_in] or NULL
};
hipError_t gemm_bp_layer(const BpLayerArgs& a, hipStream_t stream);

// ---- elementwise / integer kernels (elementwise.hip) ----
hipError_t ew_bias_act_mask(const float* zin, const float* bias, int64_t rows, int d, float alpha, float* x,
                            uint64_t* mask, hipStream_t stream);
hipError_t ew_mask_from_act(const float* x, int64_t n, uint64_t* mask, hipStream_t stream);
hipError_t ew_rev_scale(const float* h, const uint64_t* mask, int64_t n, float alpha, float* ct_z,
                        hipStream_t stream);
// a two-level scan (two launches); sums: ew_frag_scan_words(n) device words of scratch
size_t ew_frag_scan_words(int64_t n);
hipError_t ew_frag_offsets(const uint64_t* mask, int64_t n, uint32_t* offsets, uint32_t* sums, hipStream_t stream);
// the same scan for several layers in the same two launches; `layers` is a device array, max_n the largest n in it
struct FragLayer {
  const uint64_t* mask;
  uint32_t* offsets;   // [ceil(n / 64) + 1]
  int64_t n;
  uint32_t* sums;      // [ew_frag_scan_words(n)] scratch
};
hipError_t ew_frag_offsets_layers(const FragLayer* layers, int n_layers, int64_t max_n, hipStream_t stream);
// base[i] for the ReLU layers in reverse-pass order: order[j] lists layer slots, counts[slot] points at
// that layer's erased count (last entry of its offsets array)
hipError_t ew_frag_bases(const uint32_t* const* count_ptrs, int n_relu, uint64_t* bases, uint64_t* total,
                         hipStream_t stream);
hipError_t ew_frag_compact(const float* h, const uint64_t* mask, const uint32_t* offsets, int64_t n, float* frag,
                           const uint64_t* base, uint64_t capacity, int32_t* overflow_flag, hipStream_t stream);
hipError_t ew_vijp_epilogue(const float* z, float* ct_z, int64_t rows, int d, float alpha, const uint64_t* mask,
                            const uint32_t* offsets, const float* frag, const uint64_t* base, uint64_t capacity,
                            float* x, float* h_y, unsigned long long* mismatches, hipStream_t stream);
hipError_t ew_colsum(const float* a, int64_t rows, int d, float scale, float* out, hipStream_t stream);
// the same for tall matrices: row ranges summed by separate workgroups into scratch
// (ew_colsum_slices(rows, d, vec) * d floats, at most COLSUM_MAX_SLICES * d), then combined in range order;
// out = scale * sums + beta * out
constexpr int COLSUM_MAX_SLICES = 2048;
int ew_colsum_slices(int64_t rows, int d, bool vec);  // vec: the 128-bit kernel (d % 4 == 0, 16-byte aligned operands)
hipError_t ew_colsum_wide(const float* a, int64_t rows, int d, float scale, float beta, float* out, float* scratch,
                          hipStream_t stream);
// ew_colsum_wide (beta = 0) with the partial sums in an array of the library's own code object (ew_colsum_static_floats()
// floats per GPU) instead of a workspace: allocates nothing. *too_large: the partial sums would not fit, nothing was launched.
size_t ew_colsum_static_floats();
hipError_t ew_colsum_wide_static(const float* a, int64_t rows, int d, float scale, float* out, hipStream_t stream,
                                 bool* too_large);
// out[i] = scale * (sum over the slices of part[.][i], in an order fixed by slices and n) + beta * out[i]; part is [slices][n]
hipError_t ew_reduce_slices(const float* part, int slices, int64_t n, float scale, float beta, float* out, hipStream_t stream);
constexpr int LOSS_BLOCKS = 16384;  // most workgroups (and scratch doubles) the loss reduction uses
// (nonfinite, may be NULL: a device word that receives 1 when the loss is NaN or infinite, else 0)
hipError_t ew_loss_grad(const float* xL, const float* t, int64_t rows, int d, float scale, float* hL, float* loss,
                        double* scratch, hipStream_t stream, uint32_t* nonfinite = nullptr);
hipError_t ew_copy(const float* src, float* dst, int64_t n, hipStream_t stream);
hipError_t ew_fill_u32(uint32_t* p, uint32_t value, int64_t n, hipStream_t stream);
inline hipError_t ew_fill_f32(float* p, float value, int64_t n, hipStream_t stream) {
  uint32_t bits;
  static_assert(sizeof(bits) == sizeof(value), "");
  __builtin_memcpy(&bits, &value, sizeof(bits));
  return ew_fill_u32(reinterpret_cast<uint32_t*>(p), bits, n, stream);
}
// out = h .* (act > 0 ? 1 : alpha)
hipError_t ew_scale_by_act_slope(const float* h, const float* act, int64_t n, float alpha, float* out, hipStream_t stream);
// *out = max(*out, ||E - I||_F) for the n x n matrix E (row stride n); scratch: LOSS_BLOCKS doubles
hipError_t ew_identity_residual(const float* E, int n, double* scratch, float* out, hipStream_t stream);
// the same for n_sets matrices `stride` floats apart, in two launches for all of them (the same scratch)
// (minus_identity = false: ||E||_F itself, for matrices that already hold the residual)
hipError_t ew_identity_residual_sets(const float* E, int64_t stride, int n_sets, int n, double* scratch, float* out,
                                     hipStream_t stream, bool minus_identity = true);
// load-only model of a tiled product (measurement): sink gets (M/tile)*(N/tile)*256 floats
hipError_t ew_operand_stream(const float* A, const float* B, int M, int N, int K, int tile, float* sink,
                             hipStream_t stream);

// ---- convolution helpers (conv_kernels.hip): channels-last activations, [k][k][C][C'] kernels ----
// patches[r - row0][(u k + v) C + c] = x[b, s i' + u - p, s j' + v - p, c] for the patch-matrix rows [row0, row0 + n_rows)
hipError_t cv_im2col(const float* x, int H, int W, int C, int Ho, int Wo, int k, int s, int p, int64_t row0,
                     int64_t n_rows, float* patches, hipStream_t stream);
// h[img0 + b] = transpose of im2col applied to dpatches (rows of the images [img0, img0 + n_img) only), fixed summation order
hipError_t cv_col2im(const float* dpatches, int H, int W, int C, int Ho, int Wo, int k, int s, int p, int64_t img0,
                     int64_t n_img, float* h, hipStream_t stream);
// out[r][c'] = h[b, s i', s j', c'], c' < Co
hipError_t cv_strided_gather(const float* h, int H, int W, int C, int Ho, int Wo, int Co, int s, int64_t n_rows, float* out,
                             hipStream_t stream);
// Tinv = inverse of the lower-triangular n x n matrix T (row stride ld); *flag = 1 if T is not lower-triangular with non-zero diagonal
hipError_t cv_tri_inverse(const float* T, int64_t ld, int n, float* Tinv, int32_t* flag, hipStream_t stream);

// ---- convolution with the patch matrix gathered inside the GEMM (conv_gemm.hip) ----
struct ConvGeom {
  int H, W, C;     // input image, channels-last
  int Ho, Wo;      // output grid
  int kh, kw;      // taps in y and x (a 1-D convolution is a one-row image with kh = 1)
  int s;           // stride, both directions
  int ph, pw;      // padding in y and x
  int taps() const { return kh * kw; }
};
// the gathered kernels need C % 4 == 0, C_out % 32 == 0 and 16-byte aligned operands (x may be NULL: not checked)
bool conv_gather_ok(const ConvGeom& g, int Cout, const float* x, const float* w);
// most images one launch may take (every operand below 2 GiB); 0 if not even one fits
int64_t conv_gather_max_images(const ConvGeom& g, int Cout);
// xout[r][c'] = act(patches(x)[r] . w[:, c'] + b[c']) for the n_img images at x; mask32 (may be NULL) gets
// the sign bits of the same flat index, 32 per word
hipError_t conv_fwd_act(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                        float* xout, uint32_t* mask32, hipStream_t stream);
// Phase III of a layer whose ct_z [rows][Cout] is already in memory: z recomputed from x (the tile of
// conv_fwd_act, hence the same bits), x out, h out = ct_z / slope, sign check against mask32
hipError_t conv_vijp_given(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                           const float* ctz, const uint32_t* mask32, float* xout, float* hout, unsigned long long* mismatches,
                           hipStream_t stream);
// Phase III of a leaky convolutional layer for n_img images: z recomputed from x, ct_z = sub(h_in) Tinv^T,
// x out, h out = ct_z / slope, sign check against mask32. hin_as_read: hin is sub(h_in) itself,
// [rows][Cout], instead of the whole input cotangent [n_img][H][W][C]
hipError_t conv_vijp_layer(const ConvGeom& g, int n_img, const float* x, const float* w, const float* b, float alpha, int Cout,
                           const float* hin, int hin_as_read, const float* Tinv, const uint32_t* mask32, float* xout, float* hout, float* ctz,
                           unsigned long long* mismatches, hipStream_t stream);
// dW[K1][Cout] = scale * patches(x)^T ct_z + beta * dW, the patch rows split into slices whose partial
// products (part: conv_dw_part_floats floats) are added in slice order
constexpr int CONV_DW_MAX_SLICES = 256;
size_t conv_dw_part_floats(const ConvGeom& g, int n_img, int Cout);
hipError_t conv_dw(const ConvGeom& g, int n_img, const float* x, const float* ctz, int Cout, float scale, float beta,
                   float* dW, float* part, hipStream_t stream);

// ct [rows][Cout] = sub(hin) Tinv^T: hin [n_img][H][W][C] at the strided positions, first Cout channels
hipError_t conv_sub_solve(const ConvGeom& g, int n_img, int Cout, const float* hin, const float* Tinv, float* ct, hipStream_t stream);
// the general vijp's sweep over the anti-diagonals of the output grid, in place on ct (which holds sub(h) Tinv^T);
// Asweep: [Cout][((reach + 1)^2 - 1) Cout], slot (ky, kx) = T^{-1} w[p + (reach - ky) s][p + (reach - kx) s][:Cout]
hipError_t conv_vijp_sweep(int Ho, int Wo, int Cout, int n_img, int reach, float* ct, const float* Asweep, hipStream_t stream);
// whether conv_input_cotangent can be used (stride classes fit the task, channels in fours)
bool conv_rev_ok(const ConvGeom& g, int Cout);
// input cotangent of the layer for n_img images from ct_z [n_img][Ho][Wo][Cout]: raw (may be NULL) = h,
// ct (may be NULL; needs C % 32 == 0) = h times the slope the previous layer's sign bits (mask32, flat
// index of the input element) select: 1 or alpha. wrev: weights packed by cv_pack_rev_weights.
hipError_t conv_input_cotangent(const ConvGeom& g, int n_img, int Cout, const float* ctz, const float* wrev, float* raw,
                                float* ct, const uint32_t* mask32, float alpha, hipStream_t stream);
// wrev (kh kw Cin Cout floats) = the per-stride-class transposed taps conv_input_cotangent multiplies with
hipError_t cv_pack_rev_weights(const float* w, int kh, int kw, int s, int Cin, int Cout, float* wrev, hipStream_t stream);
// rows x width floats from src (row stride src_ld) to dst (row stride dst_ld); all three multiples of 4, 16-byte aligned
hipError_t cv_copy_rows(const float* src, int64_t src_ld, float* dst, int64_t dst_ld, int64_t rows, int width, hipStream_t stream);

// T[c][c'] = 0 for c < c' < n
hipError_t cv_zero_above_diagonal(float* T, int64_t ld, int n, hipStream_t stream);

// records the text of a failed HIP call for moonwalk_strerror and returns MW_ERR_HIP (moonwalk_api.hip)
int record_hip_failure(hipError_t e, const char* where);

// ---- right-inverse setup (setup_solve.hip) ----
// P[d_out][d_in] = (W W^T)^{-1} W by blocked Cholesky and two blocked triangular solves.
// work: at least setup_work_floats(d_out, d_in) floats. bad_pivot: device int32, set to 1 if a
// pivot is not positive (W not of full row rank).
size_t setup_work_floats(int d_out, int d_in);
hipError_t setup_right_inverse(const float* W, int d_out, int d_in, float* P, float* work, int32_t* bad_pivot,
                               hipStream_t stream);
// the same for `count` layers of one shape side by side; work: count * setup_work_floats(d_out, d_in) floats,
// W and P: host arrays of device pointers
hipError_t setup_right_inverse_group(int count, const float* const* W, int d_out, int d_in, float* const* P, float* work,
                                     int32_t* bad_pivot, hipStream_t stream);

}  // namespace mw
