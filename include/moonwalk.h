/*
 * libmoonwalk — mixed-mode Moonwalk gradients for dense submersive networks on MI355X (gfx950).
 *
 * C ABI. Every pointer is a DEVICE pointer unless its comment says "host". The library
 * never takes ownership of a caller's buffer and never frees one. All calls enqueue work
 * on the HIP stream they are given (a hipStream_t passed as void*, NULL = default stream)
 * and return without synchronising, except where stated (setup, refresh, status, fetch).
 *
 * Network (row-vector convention, row-major storage):
 *     z_i = x_{i-1} W_i^T + b_i ,  m_i = (z_i > 0) ,  x_i = m_i ? z_i : alpha_i z_i ,  i = 1..L
 *     J   = 0.5 ||x_L - target||_F^2 / B
 * x_i is [B][d_i], W_i is [d_i][d_{i-1}], b_i is [d_i]. Each layer must be a submersion
 * (Definition "Submersion" of the Moonwalk paper): d_i <= d_{i-1} and W_i of full row rank.
 *
 * Return value of every int function: 0 on success, a negative MW_ERR_* code otherwise.
 * No exception crosses this boundary and nothing aborts.
 */
#ifndef MOONWALK_H
#define MOONWALK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MW_OK                    0
#define MW_ERR_INVALID_ARG      (-1)  /* NULL/zero/negative argument, alpha outside [0,1], bad enum   */
#define MW_ERR_NOT_SUBMERSIVE   (-2)  /* d_out > d_in, or W W^T not positive definite (Cholesky pivot) */
#define MW_ERR_OOM              (-3)  /* the allocator callback returned NULL                          */
#define MW_ERR_FRAG_OVERFLOW    (-4)  /* fragment store smaller than the number of erased cotangents   */
#define MW_ERR_HIP              (-5)  /* a HIP call failed; text available from moonwalk_strerror      */
#define MW_ERR_SIGN_MISMATCH    (-6)  /* phase-III recomputed signs differ from the phase-I masks      */
#define MW_ERR_NOT_PLANNED      (-7)  /* entry point called on a handle planned without it             */
#define MW_ERR_TOO_LARGE        (-8)  /* input beyond the fixed scratch of an entry point that allocates nothing */
#define MW_ERR_NONFINITE        (-9)  /* the loss of the last gradient step was NaN or infinite         */

typedef struct mw_handle mw_handle_t;   /* opaque; owned by the library */

/* One dense layer followed by a leaky ReLU (alpha in (0,1]) or a ReLU (alpha == 0). */
typedef struct {
  int32_t d_in, d_out;   /* 1 <= d_out <= d_in                                                    */
  const float* W;        /* device, row-major [d_out][d_in]; caller owns; must outlive the handle */
  const float* b;        /* device [d_out]; NULL means zero bias                                  */
  float alpha;           /* 0 < alpha <= 1: leaky ReLU (submersive); 0: ReLU + fragment store     */
} mw_layer_t;

#define MW_PLAN_MOONWALK 1   /* build P_i and the Moonwalk workspace                 */
#define MW_PLAN_BACKPROP 2   /* build the stored-activation workspace for backprop   */

typedef struct {
  int32_t batch;            /* B, fixed for the handle's lifetime                                         */
  int32_t reseed_interval;  /* K: keep the cotangent of every K-th layer boundary in the reverse pass and
                               restart the forward sweep from it (plain cotangent checkpointing, Overview
                               section). 0 = never: the method exactly as printed. -1 = chosen by the
                               library from the layers' slopes (a seed wherever the predicted error
                               growth prod (alpha + 1/alpha)/2 since the last seed would pass 700).        */
  float   loss_scale;       /* s > 0, a power of two: the output cotangent is multiplied by s and the
                               gradients are divided by s again (exact); guards fp32 under/overflow.      */
  int32_t plan;             /* MW_PLAN_* bits; 0 means MW_PLAN_MOONWALK | MW_PLAN_BACKPROP                 */
  int32_t fuse;             /* 1: bias/activation/mask/cotangent steps fused into the GEMM kernels;
                               0: plain GEMMs plus stand-alone elementwise kernels (same results, bit for bit) */
  double  frag_capacity_factor; /* fragment-store capacity as a fraction of B * sum(d_out over ReLU
                               layers); 1.0 = worst case; <= 0 means 1.0                                   */
  /* Every byte of device memory the library owns comes from dev_alloc and goes back through
     dev_free (both host functions). NULL, NULL = hipMalloc / hipFree. */
  void* (*dev_alloc)(size_t bytes, void* ctx);
  void  (*dev_free)(void* ptr, void* ctx);
  void*   alloc_ctx;
  int32_t segment_length;   /* S > 0: Moonwalk with rematerialisation (Table 1, "Moonwalk + checkpoint"). Phase I
                               keeps the activation of every S-th layer boundary and NO masks; the segments
                               of S layers are then finished one at a time from the top: forward again
                               inside the segment (masks, fragment index), reverse, Phase III. Masks,
                               fragments and their index exist for one segment only; costs one more forward
                               pass. Needs fuse = 1. 0 or >= n_layers: off.                               */
  int32_t debug_keep;       /* 0: nothing extra. 1: a debugging aid for moonwalk_debug_fetch: every layer's Phase-I
                               pre-activations z_i, Phase-II cotangent at its output and Phase-III cotangent at
                               its output are kept in buffers of their own (3 x 4 B d_i bytes per layer, itemised
                               as bytes_debug). The results of the gradient calls do not change by a bit.   */
  int32_t phase3_parallel_segments; /* Phase III side by side. The re-seed points (reseed_interval) cut the network into
                               stretches whose forward sweeps do not depend on each other once the activation at a
                               stretch's first layer is kept as well (Table 1, "Moonwalk + checkpoint": Phase I
                               writes it there on its way, B d_i floats per re-seed point). Up to this many
                               consecutive stretches of one shape are swept in ONE launch per layer position,
                               which fills the chip when one small-batch layer cannot. 1: off (one layer per
                               launch, nothing extra kept). 0: chosen by the library (enough stretches to give
                               every CU a 64 x 64 tile; off where one layer fills the chip already, or with fewer
                               than two stretches). 2..16: at most that many. Each stretch in flight has its own 7
                               rotating buffers of B max d floats. Needs fuse = 1 and segment_length = 0 (else
                               ignored). Gradients, masks and h_0 are the same bit for bit whatever the value.     */
  int32_t phase3_overlap;   /* 1: the grouped sweeps of phase3_parallel_segments are issued on a second stream of
                               the library (default priority), each as soon as Phase II has passed its lowest
                               re-seed point, and share the machine with the rest of Phase II; the caller's stream
                               waits for them at the end of the call, so the call still looks asynchronous on
                               hip_stream alone. 0: everything on hip_stream, Phase III after Phase II.           */
  int32_t refresh_precision; /* moonwalk_refresh_incremental / moonwalk_sgd_step. 0: every product of a Schulz iteration in
                               fp32. 1: the residual R = I - P W^T in fp32 (that difference is where digits are lost),
                               the correction R P that is then added to P with its operands rounded to bf16 (to nearest
                               even) in front of the matrix unit, sums and the addition in fp32: the correction is
                               ||R|| times the size of P, so its 2^-8 relative error is 2^-8 ||R|| of P, and the next
                               iteration (which measures its residual in fp32 again) takes it out; the residual then
                               shrinks like R^2 + 2^-8 R per iteration instead of R^2. About three times faster for the
                               correction product. Layers whose operands are not 16-byte aligned or whose widths are
                               not multiples of four stay in fp32.                                                   */
} mw_config_t;

/* Itemised device bytes held by a handle (closed forms are in the design notes). */
typedef struct {
  uint64_t bytes_P;             /* right inverses, = bytes of all W                                   */
  uint64_t bytes_masks;         /* 1-bit sign masks, 8 * ceil(B d_i / 64) per layer                   */
  uint64_t bytes_fragments;     /* fragment store capacity (ReLU layers)                              */
  uint64_t bytes_frag_index;    /* per-word erased offsets, layer bases                               */
  uint64_t bytes_checkpoints;   /* re-seed cotangents; with segments also the kept activations        */
  uint64_t bytes_mw_scratch;    /* ping-pong activations / cotangents, ct_z, loss partials, flags     */
  uint64_t bytes_bp_activations;/* stored x_1..x_L of the backprop path                               */
  uint64_t bytes_bp_scratch;    /* backprop cotangent ping-pong, loss partials                        */
  uint64_t bytes_live;          /* currently held through dev_alloc                                   */
  uint64_t bytes_peak;          /* high-water mark through dev_alloc, setup scratch included          */
  uint64_t bytes_setup_peak;    /* high-water mark during setup / refresh alone                       */
  uint64_t frag_used;           /* erased cotangents stored by the last moonwalk_grad                 */
  uint64_t sign_mismatches;     /* phase-III signs that differed from the stored masks (must be 0)    */
  int32_t  frag_overflow;       /* 1 if the last moonwalk_grad overflowed the fragment store          */
  int32_t  phase3_group_width;  /* most stretches Phase III sweeps in one launch (cfg.phase3_parallel_segments as planned); 0: one layer per launch */
  uint64_t bytes_debug;         /* cfg.debug_keep: the kept z_i and cotangents                          */
  int32_t  nonfinite_loss;      /* 1 if the loss of the last moonwalk_grad / sgd_step / backprop_grad was NaN or
                                   infinite (inputs, weights or activations out of range): its gradients are void */
  int32_t  reserved;
} mw_memstats_t;

/*
 * moonwalk_setup — create a handle for a fixed network and batch size.
 * Validates the submersion condition (d_out <= d_in; Cholesky of W W^T must succeed), computes
 * the per-layer right inverse P_i = (W_i W_i^T)^{-1} W_i on the device (the (.)^+ of the vijp
 * definition, Notation section; P_i^T is the Moore-Penrose right inverse of the layer Jacobian
 * W_i), and allocates the workspaces named in cfg->plan.
 * layers: host array of n_layers descriptors (copied). Synchronises the stream before returning.
 * Every matrix (d_out x d_in weights, batch x d activations) must be smaller than 2 GiB (the
 * kernels use 31-bit byte offsets): MW_ERR_INVALID_ARG otherwise.
 * On failure *out is NULL and everything allocated so far has been freed.
 */
int moonwalk_setup(mw_handle_t** out, const mw_layer_t* layers, int32_t n_layers,
                   const mw_config_t* cfg, void* hip_stream);

/* Recompute every P_i after the caller changed W in place (Algorithm 1, "Apply g_i").
   Synchronises. Same errors as moonwalk_setup. */
int moonwalk_refresh(mw_handle_t* h, void* hip_stream);

/*
 * moonwalk_refresh_incremental — bring every P_i up to date after a SMALL change of W_i (an
 * optimizer step) without redoing the factorisation. The paper leaves open how the inverse follows
 * the weights (Algorithm 1 applies g_i and goes on); this is this library's answer:
 *   P_0 = (P P^T) W_new            (P P^T = (W_old W_old^T)^{-1}: first-order guess whose rows lie
 *                                   in the row space of W_new, so every iterate below is the
 *                                   minimum-norm right inverse of its own residual equation)
 *                                   (a square layer has one inverse and no row space to stay in: P_0 = P)
 *   P_{k+1} = (2 I - P_k W_new^T) P_k,  k = 0 .. iters-1   (Newton-Schulz: I - P W^T squares each time)
 * Plain GEMMs on the given stream; does not synchronise. iters in 0..16. residual_out (device float
 * or NULL) receives max over layers of ||I - P W^T||_F measured BEFORE the last iteration (after it
 * the residual is about the square of that); -1 with iters = 0. If that figure is not well below 1
 * the change of W was too large: call moonwalk_refresh. Scratch of the largest layer's
 * d_out^2 + d_out d_in floats is allocated on first use (MW_ERR_OOM) and kept.
 */
int moonwalk_refresh_incremental(mw_handle_t* h, int32_t iters, float* residual_out, void* hip_stream);

/*
 * moonwalk_grad — one gradient step of mixed-mode Moonwalk (Overview section, Phases I-III;
 * Algorithm 1 with h_0 from the reverse pass of the Mixed-Mode section).
 *   Phase I   forward; keeps only the packed sign masks m_i (Residual Impact section).
 *   Phase II  reverse for the input cotangent h_0 alone; for ReLU layers the erased entries of
 *             the output cotangent go to the fragment store (Fragmental Gradient Checkpointing).
 *   Phase III forward sweep: recompute z_i, ct_z = h_{i-1} P_i^T (vijp, Eq. h_i), undo the
 *             activation slope or restore fragments, dW_i = ct_z^T x_{i-1}, db_i = sum_b ct_z
 *             (vjp w.r.t. parameters, Eq. g_i).
 * x [B][d_0], target [B][d_L]: read only. grads_out: flat buffer laid out as reported by
 * moonwalk_grad_layout, overwritten (not accumulated). loss_out: one float, may be NULL.
 * Asynchronous. Results are bit-identical run to run.
 */
int moonwalk_grad(mw_handle_t* h, const float* x, const float* target,
                  float* grads_out, float* loss_out, void* hip_stream);

/*
 * moonwalk_sgd_step — one training step in place (Algorithm 1 with "Apply g_i"): the three phases of
 * moonwalk_grad, but each layer's gradient is applied as soon as Phase III has produced it,
 *   W_i -= lr * dW_i,  b_i -= lr * db_i
 * in the weight-gradient product's own epilogue, to the W_i / b_i arrays given at setup (device;
 * they are WRITTEN by this call). No gradient buffer exists at any time. Afterwards, if
 * refresh_iters >= 0, P is refreshed as by moonwalk_refresh_incremental(refresh_iters,
 * residual_out); with refresh_iters < 0 the caller must refresh before the next step.
 * Needs the fused path (cfg.fuse) and MW_PLAN_MOONWALK, else MW_ERR_NOT_PLANNED. loss_out as in
 * moonwalk_grad (loss of the weights BEFORE the update). Does not synchronise.
 */
int moonwalk_sgd_step(mw_handle_t* h, const float* x, const float* target, float lr, int32_t refresh_iters,
                      float* loss_out, float* residual_out, void* hip_stream);

/* backprop_grad — the same gradient by ordinary reverse mode with every activation stored
   (the comparison method of the paper, Fig. 1 right column). Same arguments and layout. */
int backprop_grad(mw_handle_t* h, const float* x, const float* target,
                  float* grads_out, float* loss_out, void* hip_stream);

/* Layout of grads_out: layer i (0-based) has dW_i, row-major [d_out][d_in], at float offset
   dW_off[i] and db_i at db_off[i]. total_floats, dW_off, db_off: host pointers, any may be NULL;
   the arrays have n_layers entries. */
int moonwalk_grad_layout(const mw_handle_t* h, size_t* total_floats, size_t* dW_off, size_t* db_off);

/* Itemised memory and the sticky device-side conditions of the last step. out: host.
   Synchronises the device (reads the flags back). Returns MW_ERR_FRAG_OVERFLOW, MW_ERR_NONFINITE or
   MW_ERR_SIGN_MISMATCH (in this order) if the last step raised one, after filling *out. */
int moonwalk_memory_stats(mw_handle_t* h, mw_memstats_t* out);

/* What moonwalk_debug_fetch can copy to the host (element type, count for layer i):          */
#define MW_FETCH_MASK          1  /* uint64[ceil(B d_i / 64)]  packed signs, bit e%64 of word e/64 */
#define MW_FETCH_FRAG          2  /* float[n0_i]               erased cotangents, ascending index  */
#define MW_FETCH_FRAG_OFFSETS  3  /* uint32[n_words + 1]       erased count before each word; last = n0_i */
#define MW_FETCH_FRAG_BASE     4  /* uint64[1]                 start of layer i in the store        */
#define MW_FETCH_H0            5  /* float[B d_0]              input cotangent (scaled by loss_scale); layer ignored */
#define MW_FETCH_P             6  /* float[d_out d_in]         right inverse                         */
#define MW_FETCH_CHECKPOINT    7  /* float[B d_i]              kept cotangent at the OUTPUT of layer i (error if not kept) */
/* The next three need cfg.debug_keep = 1 (MW_ERR_INVALID_ARG otherwise):                                   */
#define MW_FETCH_Z             8  /* float[B d_i]              z_i = x_{i-1} W_i^T + b_i as Phase I computed it (the mask
                                                               bits are z_i > 0; Residual Impact section)              */
#define MW_FETCH_H             9  /* float[B d_i]              Phase-II cotangent at the OUTPUT of layer i, scaled by
                                                               loss_scale, before the activation slope is applied: the
                                                               tensor whose erased entries are the layer's fragments
                                                               (Fragmental Gradient Checkpointing section)             */
#define MW_FETCH_H_FORWARD    10  /* float[B d_i]              Phase-III cotangent at the OUTPUT of layer i (Eq. h_i:
                                                               the vijp of layer i applied to the cotangent below it)  */
/* Synchronous copy of library state after the last step to host_dst (host, cap bytes).
   layer is 0-based. *n_bytes (host, may be NULL) receives the size. host_dst == NULL with
   cap == 0 is a size query (returns MW_OK); if cap is too small nothing is copied and
   MW_ERR_INVALID_ARG is returned with *n_bytes set. */
int moonwalk_debug_fetch(mw_handle_t* h, int32_t layer, int32_t what, void* host_dst, size_t cap,
                         size_t* n_bytes);

/* ------------------------------------------------------------------------------------------
 * Submersive 2-D convolutional layers (lemma on submersive convolutional layers; the fully
 * parallel 2-D setting of the experiments).
 *
 * Activations are channels-last, [B][H][W][C] fp32; a layer is
 *   z[b,i',j',c'] = sum_{u,v,c} w[u,v,c,c'] x[b, s i'+u-p, s j'+v-p, c] + bias[c'],  x' = leaky_relu(z)
 * with kernel w [k][k][C_in][C_out] (row-major in that order), one stride s and padding p for both
 * spatial dimensions, and the loss J = 0.5 ||x_L - t||^2 / B. Setup checks the lemma's conditions:
 * k > p, s > p, n > s (n' - 1) in both dimensions, C_out <= C_in, and on the device that the tap
 * w[p][p] is channel-triangular (w[p][p][c][c'] = 0 for c < c') with non-zero diagonal
 * (MW_ERR_NOT_SUBMERSIVE otherwise); alpha must be in (0, 1]. For k <= p + s (the fully parallel case)
 * no other output position enters the equation of h[s i', s j', c'] and the vijp of the convolution
 * is, at every output position on its own, the triangular solve
 * T h'[i', j', :] = h[s i', s j', :C_out] with T = w[p][p][:C_out][:C_out]. For wider kernels the
 * equation also holds the earlier positions (i' - a, j' - b), a, b <= (k - 1 - p) / s, through the taps
 * (p + a s, p + b s): those are subtracted in a sweep over the anti-diagonals of the output grid, one
 * launch per diagonal. That sweep needs C_in and C_out to be multiples of 32, MW_CONV_KERNELS_AUTO and
 * MW_CONV_H0_FULL (MW_ERR_INVALID_ARG otherwise), and its re-seed cotangents are kept whole. The
 * library keeps T^{-1} per layer, and for the layers on the gathered kernels a regrouped copy of the
 * taps that BOTH gradient paths use: after changing w call moonwalk_conv_refresh before either
 * moonwalk_conv_grad or backprop_conv_grad (it recomputes both, whatever the plan).
 * The gradient layout is per layer dw [k][k][C_in][C_out] then db [C_out].
 *
 * Fragmental 1-D layers (section on fragmental gradient checkpointing, its appendix and the
 * fragmental vijp algorithm): kind = MW_CONV_FRAGMENTAL_1D. The input is a one-row image
 * ([B][1][N][C], cfg.height = 1), the kernel is [k][C_in][C_out] with k odd, stride 1 and padding
 * (k - 1) / 2, so every layer keeps the length N; C_in and C_out must be multiples of 32,
 * C_out <= C_in, N a multiple of `block`, block >= k - 1 (MW_ERR_INVALID_ARG otherwise). Such a layer
 * is not submersive. The tap w[0] must be channel-triangular (w[0][c][c'] = 0 for c < c') with
 * non-zero diagonal (MW_ERR_NOT_SUBMERSIVE otherwise). Phase II keeps, per layer, the first k - 1
 * positions of every block of the convolution's output cotangent ((k - 1) / block of an activation);
 * Phase III rebuilds the other positions of a block one after the other,
 *   T ct[t, :] = h[t - p, :C_out] - sum_{u = 1}^{k-1} w[u][:C_out]^T-contracted ct[t - u, :],
 * all blocks and samples at once. h_0 is computed whole (MW_CONV_H0_FULL is required).
 * The gradient layout is per layer dw [k][C_in][C_out] then db [C_out].
 * ------------------------------------------------------------------------------------------ */
typedef struct mw_conv_handle mw_conv_handle_t;

#define MW_CONV_KERNELS_AUTO 0
#define MW_CONV_KERNELS_PATCH_MATRIX 1
#define MW_CONV_SUBMERSIVE 0
#define MW_CONV_FRAGMENTAL_1D 1
#define MW_CONV_H0_FULL 0
#define MW_CONV_H0_AS_READ 1

typedef struct {
  int32_t channels_in, channels_out, k, stride, pad;
  const float* w;   /* device, [k][k][channels_in][channels_out]; caller owns; must outlive the handle */
  const float* b;   /* device [channels_out]; NULL means zero bias                                     */
  float alpha;      /* leaky-ReLU slope in (0, 1]                                                      */
  int32_t kind;     /* MW_CONV_SUBMERSIVE (the lemma's layer, 2-D, vijp in closed form) or
                       MW_CONV_FRAGMENTAL_1D (see below); the same for every layer of a chain             */
  int32_t block;    /* MW_CONV_FRAGMENTAL_1D: positions per block of the fragment store                  */
} mw_conv_layer_t;

typedef struct {
  int32_t batch, height, width;  /* input activation [batch][height][width][layers[0].channels_in]      */
  int32_t reseed_interval;       /* as in mw_config_t (>= 0)                                            */
  float   loss_scale;            /* as in mw_config_t                                                   */
  int32_t plan;                  /* MW_PLAN_* bits; 0 = both                                            */
  int32_t kernels;               /* MW_CONV_KERNELS_AUTO: layers with C_in % 4 == 0 and C_out % 32 == 0 run
                                    kernels that gather the patch matrix inside the product (forward, Phase
                                    III, weight gradient); MW_CONV_KERNELS_PATCH_MATRIX: every layer goes
                                    through the patch buffer                                             */
  int32_t input_cotangent;       /* MW_CONV_H0_FULL: Phase II ends with h_0 for every input element (a caller
                                    with layers before this chain continues its own reverse pass from it),
                                    and backprop_conv_grad computes the same h_0 at the end of its sweep;
                                    MW_CONV_H0_AS_READ: only the entries the first layer's vijp reads are
                                    computed and kept, [B][H'][W'][C_out] of layer 0 (the strided positions,
                                    the first C_out channels), and the first layer's reverse product is
                                    skipped                                                              */
  int32_t max_images_per_launch; /* the gathered kernels take the batch in launches of at most this many images
                                    (0 = as many as the 2 GiB limit on a launch's operands allows; < 0:
                                    MW_ERR_INVALID_ARG); the launches are of equal size up to the last one, and
                                    the weight gradient's partial sums are sized for one launch             */
  size_t  patch_bytes;           /* size of the buffer the image chunks' patch matrices are gathered into
                                    (0 = 256 MiB); at least one image's patches are always taken        */
  void* (*dev_alloc)(size_t bytes, void* ctx);
  void  (*dev_free)(void* ptr, void* ctx);
  void*   alloc_ctx;
} mw_conv_config_t;

typedef struct {
  uint64_t bytes_masks;            /* 1-bit sign masks of all layer outputs                              */
  uint64_t bytes_tap_inverses;     /* T^{-1}, C_out^2 floats per layer                                   */
  uint64_t bytes_packed_weights;   /* taps regrouped by stride class for the input-cotangent kernel: one
                                      copy of every layer's weights that takes the gathered kernels      */
  uint64_t bytes_fragments;        /* fragmental layers: the first k - 1 positions of every block of each
                                      layer's ct_z, (k - 1) / block of an activation per layer           */
  uint64_t bytes_checkpoints;      /* re-seed cotangents, each as the next layer's vijp reads it:
                                      [B][H'][W'][C_out] of that layer                                   */
  uint64_t bytes_input_cotangent;  /* h_0: as large as the network input, or as read (see the config)   */
  uint64_t bytes_scratch;          /* ping-pong activations / cotangents, z, ct_z, right-hand sides      */
  uint64_t bytes_patches;          /* the patch buffer (shared by both paths)                            */
  uint64_t bytes_bp_activations;   /* backprop: stored layer outputs                                     */
  uint64_t bytes_bp_scratch;       /* backprop: cotangent ping-pong (when planned without Moonwalk)      */
  uint64_t bytes_live, bytes_peak;
  uint64_t sign_mismatches;        /* Phase-III signs that differed from the stored masks (must be 0)    */
  uint64_t nonfinite_loss;         /* 1 if the loss of the last gradient step was NaN or infinite         */
} mw_conv_memstats_t;

/* Same contracts as the dense entry points of the same names (setup synchronises; grad calls only
   enqueue; gradients are overwritten, bit-identical run to run). x: [B][H][W][C_0]; target: shape of
   the last layer's output. */
int moonwalk_conv_setup(mw_conv_handle_t** out, const mw_conv_layer_t* layers, int32_t n_layers,
                        const mw_conv_config_t* cfg, void* hip_stream);
int moonwalk_conv_refresh(mw_conv_handle_t* h, void* hip_stream);
int moonwalk_conv_grad(mw_conv_handle_t* h, const float* x, const float* target, float* grads_out, float* loss_out,
                       void* hip_stream);
int backprop_conv_grad(mw_conv_handle_t* h, const float* x, const float* target, float* grads_out, float* loss_out,
                       void* hip_stream);
/* One training step in place (Algorithm 1 with "Apply g_i"): the phases of moonwalk_conv_grad, but each
   layer's gradient goes straight onto that layer's own arrays, w_i -= lr dw_i and b_i -= lr db_i (a layer
   given b = NULL has no bias to update), in the reduction that ends the weight-gradient product; the w and
   b arrays given at setup are WRITTEN. The entries the method constrains to zero (above the diagonal of
   the triangular tap, first C_out rows) are then put back to zero: a projected step, the layers stay
   submersive / fragmental as long as no diagonal entry reaches zero. No gradient buffer exists at any
   time. Ends with what moonwalk_conv_refresh does. Every layer must be on the gathered kernels and the
   plan must hold MW_PLAN_MOONWALK (MW_ERR_NOT_PLANNED otherwise). loss_out: the loss BEFORE the update.
   Synchronises (the refresh reads back its check of the taps); returns MW_ERR_NOT_SUBMERSIVE if a diagonal
   entry has become zero. */
int moonwalk_conv_sgd_step(mw_conv_handle_t* h, const float* x, const float* target, float lr, float* loss_out,
                           void* hip_stream);
int moonwalk_conv_grad_layout(const mw_conv_handle_t* h, size_t* total_floats, size_t* dW_off, size_t* db_off);
/* Synchronises; returns MW_ERR_NONFINITE or MW_ERR_SIGN_MISMATCH if the last gradient step raised one, after filling *out. */
int moonwalk_conv_memory_stats(mw_conv_handle_t* h, mw_conv_memstats_t* out);
/* what: MW_FETCH_MASK, MW_FETCH_H0 (whole or as read, see the config), MW_FETCH_P (here: T^{-1},
   float[C_out^2]), MW_FETCH_FRAG (fragmental layers: float[B N / block][k - 1][C_out]) or MW_FETCH_CHECKPOINT (the cotangent kept at the output of `layer`, in the
   [B][H'][W'][C_out] form of layer + 1). */
int moonwalk_conv_fetch(mw_conv_handle_t* h, int32_t layer, int32_t what, void* host_dst, size_t cap, size_t* n_bytes);
void moonwalk_conv_destroy(mw_conv_handle_t* h);

/* Patch gather and its transpose (kernel-level, for the unit tests). Row r = (b H' + i') W' + j' of the
   patch matrix, column (u k + v) C + c. im2col writes rows [row0, row0 + n_rows) to patches
   ([n_rows][k k C]); col2im sums the rows of the images [img0, img0 + n_img) held in dpatches
   ([n_img H' W'][k k C]) into h[img0 ..] ([.][H][W][C]), in a fixed order. */
int mw_conv_im2col(const float* x, int32_t H, int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad, int64_t row0,
                   int64_t n_rows, float* patches, void* hip_stream);
int mw_conv_col2im(const float* dpatches, int32_t H, int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad,
                   int64_t img0, int64_t n_img, float* h, void* hip_stream);

/* The three products that gather the patch matrix inside the MFMA main loop (kernel-level, for the
   unit tests; the convolution of the lemma on submersive convolutional layers, its vjp and its parameter
   vjp, for any kernel kh x kw, stride and paddings, not only the layers Moonwalk accepts). All tensors
   device, channels-last; w is [kh][kw][C_in][C_out]; H', W' = (H + 2 ph - kh) / stride + 1, likewise W'.
   C_in and C_out must be multiples of 32, every tensor below 2 GiB, stride * stride <= 9 for the input
   cotangent (MW_ERR_INVALID_ARG otherwise).
     mw_conv_forward:         xout [B][H'][W'][C_out] = act(conv(x, w) + b) with act = leaky ReLU of slope alpha
                              (alpha = 1: none); b may be NULL; mask (may be NULL) gets the packed signs of z.
     mw_conv_input_cotangent: h [B][H][W][C_in] = vjp of the convolution w.r.t. its input applied to ctz
                              [B][H'][W'][C_out]; work: kh kw C_in C_out floats (regrouped taps).
     mw_conv_weight_grad:     dw [kh][kw][C_in][C_out] = scale * vjp w.r.t. the kernel, db [C_out] = scale * sums of
                              ctz over all positions; work: mw_conv_weight_grad_work_floats(...) floats. */
typedef struct {
  int32_t batch, height, width, channels_in, channels_out, kh, kw, stride, pad_h, pad_w;
} mw_conv_shape_t;
int mw_conv_forward(const mw_conv_shape_t* shape, const float* x, const float* w, const float* b, float alpha, float* xout,
                    uint64_t* mask, void* hip_stream);
int mw_conv_input_cotangent(const mw_conv_shape_t* shape, const float* ctz, const float* w, float* h, float* work,
                            void* hip_stream);
size_t mw_conv_weight_grad_work_floats(const mw_conv_shape_t* shape);
int mw_conv_weight_grad(const mw_conv_shape_t* shape, const float* x, const float* ctz, float scale, float* dw, float* db,
                        float* work, void* hip_stream);

/* Frees every device buffer through dev_free. NULL is allowed. Synchronises the device first. */
void moonwalk_destroy(mw_handle_t* h);

/* Static text for a code; for MW_ERR_HIP the text of the last HIP error seen by this thread. */
const char* moonwalk_strerror(int code);

/* ------------------------------------------------------------------------------------------
 * Kernel-level entry points: the individual device steps, for unit parity tests and roofline
 * measurements. All asynchronous on hip_stream; all pointers device pointers.
 * ---------------------------------------------------------------------------------------- */

#define MW_GEMM_NT 0  /* C[M][N] = alpha * A[M][K] * B[N][K]^T + beta * C   (forward, vijp)      */
#define MW_GEMM_NN 1  /* C[M][N] = alpha * A[M][K] * B[K][N]   + beta * C   (reverse vjp)        */
#define MW_GEMM_TN 2  /* C[M][N] = alpha * A[K][M]^T * B[K][N] + beta * C   (weight gradient)    */
#define MW_TILE_AUTO 0
#define MW_TILE_128  1  /* 128x128 workgroup tile                                   */
#define MW_TILE_64   2  /* 64x64 workgroup tile                                     */
#define MW_TILE_32K4 3  /* 32x32 workgroup tile, K split over four wavefronts        */
#define MW_TILE_32K8 4  /* 32x32 workgroup tile, K split over eight wavefronts       */
#define MW_TILE_64K2 5  /* 64x64 workgroup tile, K split over two groups of four wavefronts */
#define MW_TILE_128W8 6 /* 128x128 workgroup tile, eight wavefronts                     */
#define MW_TILE_64X128 7 /* 64x128 workgroup tile, eight wavefronts                     */
/* fp32 MFMA GEMM with LDS-staged tiles; lda/ldb/ldc are row strides in floats. */
int mw_gemm_f32(int32_t op, int32_t tile, int32_t M, int32_t N, int32_t K, float alpha,
                const float* A, int32_t lda, const float* B, int32_t ldb, float beta,
                float* C, int32_t ldc, void* hip_stream);

/* Phase-I epilogue (mask pack + activation): x[e] = m ? z : alpha z with z = zin[e] + bias[e % d],
   mask bit e = (z > 0). n = rows * d elements; mask has ceil(n/64) words. bias may be NULL.
   zin and x may alias. */
int mw_bias_act_mask(const float* zin, const float* bias, int64_t rows, int32_t d, float alpha,
                     float* x, uint64_t* mask, void* hip_stream);

/* Phase-II scaling: ct_z[e] = h[e] * (m[e] ? 1 : alpha). h and ct_z may alias. */
int mw_rev_scale(const float* h, const uint64_t* mask, int64_t n, float alpha, float* ct_z,
                 void* hip_stream);

/* Erased-element index of a mask: offsets[w] = number of zero bits among elements < 64 w,
   offsets[n_words] = n0 (uint32[n_words + 1]). Deterministic integer scan in two levels (two launches: the
   erased counts of chunks of 2048 mask words, then the offsets); every mask word is read twice whatever n is.
   work: mw_frag_offsets_work_words(n) device words of scratch (one per chunk). */
size_t mw_frag_offsets_work_words(int64_t n);
int mw_frag_offsets(const uint64_t* mask, int64_t n, uint32_t* offsets, uint32_t* work, void* hip_stream);

/* Stream compaction of the erased cotangents: frag[offsets[e/64] + rank of e within its word] =
   h[e] for every e with mask bit 0, ascending e. capacity in floats; on overflow nothing past
   capacity is written and *overflow_flag (device int32, may be NULL) is set to 1. */
int mw_frag_compact(const float* h, const uint64_t* mask, const uint32_t* offsets, int64_t n,
                    float* frag, uint64_t capacity, int32_t* overflow_flag, void* hip_stream);

/* Phase-III epilogue. z, ct_z: [rows][d] pre-activation (bias already added) and affine-vijp
   result. Writes x = f(z) and the layer-output cotangent h_y.
   alpha > 0: m = (z > 0), h_y = m ? ct_z : ct_z / alpha (as a multiplication by fp32 1/alpha).
   alpha == 0: m = stored mask; ct_z is zeroed in place where m == 0 and h_y = m ? ct_z :
   frag[offsets[e/64] + rank]. mask/offsets/frag are required only for alpha == 0. */
int mw_vijp_epilogue(const float* z, float* ct_z, int64_t rows, int32_t d, float alpha,
                     const uint64_t* mask, const uint32_t* offsets, const float* frag,
                     float* x, float* h_y, void* hip_stream);

/* Column sums: out[j] = scale * sum_r a[r][j], fixed summation order. */
int mw_colsum(const float* a, int64_t rows, int32_t d, float scale, float* out, void* hip_stream);
/* The same for tall matrices (the bias gradient of a convolutional layer: rows = B H' W'): the rows are cut
   into ranges summed by separate workgroups (128-bit non-temporal loads when d % 4 == 0 and a, work are
   16-byte aligned), and the ranges' sums are added in range order. work: mw_colsum_work_floats(d) device
   floats. Fixed summation order, another one than mw_colsum's. */
size_t mw_colsum_work_floats(int32_t d);
int mw_colsum_wide(const float* a, int64_t rows, int32_t d, float scale, float* out, float* work, void* hip_stream);

/* mw_colsum_wide for callers that cannot allocate and have no workspace to pass: code under HIP graph
   capture, tight serving loops, harnesses that forbid hipMalloc. Same result as mw_colsum_wide with a
   256-byte aligned workspace, bit for bit (same kernels, same row ranges, same summation order). The
   row-range partial sums go to a fixed array inside the library's code object, mw_colsum_noalloc_max_floats()
   floats (4 MiB) on every GPU the library is loaded on, held until the process ends; the call makes no
   hipMalloc / hipFree and calls no allocating routine. It needs (number of row ranges) * d floats of
   that array: always enough for d <= 4096, and for any d up to the array's size when rows is small
   enough for one range; beyond it MW_ERR_TOO_LARGE is returned and nothing is launched. All calls
   on one GPU share the array, which keeps the last call's contents (nothing needs clearing: every
   slot a call reads it has written first): calls that overlap on one GPU, from different streams or
   threads, race; order them. Asynchronous on hip_stream like the others. */
size_t mw_colsum_noalloc_max_floats(void);
int mw_colsum_wide_noalloc(const float* a, int64_t rows, int32_t d, float scale, float* out, void* hip_stream);

/* Loss step: h_L = scale (x_L - t) / rows and *loss = 0.5 ||x_L - t||_F^2 / rows (fixed-order
   reduction; partial sums in double). loss may be NULL. scratch: device doubles,
   at least mw_loss_scratch_doubles() of them. */
int mw_loss_grad(const float* xL, const float* t, int64_t rows, int32_t d, float scale,
                 float* hL, float* loss, double* scratch, void* hip_stream);
size_t mw_loss_scratch_doubles(void);

#ifdef __cplusplus
}
#endif
#endif /* MOONWALK_H */
