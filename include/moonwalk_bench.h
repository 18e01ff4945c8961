/*
 * libmoonwalk, measurement aids. Nothing here is part of the method: these entry points exist so that
 * a benchmark can time one class of the library's kernels alone, and compare the machine's copy and
 * operand-fill rates with what the kernels reach. They live in the same shared library as the entry
 * points of moonwalk.h and follow the same conventions (device pointers, a hipStream_t passed as
 * void*, 0 or a negative MW_ERR_* code).
 */
#ifndef MOONWALK_BENCH_H
#define MOONWALK_BENCH_H

#include "moonwalk.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid: run the gradient drivers with only ONE class of kernel launches enabled, so
   that a caller can time that class alone between two events on its stream (the launches then run
   back to back over the handle's real buffers, layer after layer, with the real shapes and cold
   weights; the numbers they produce are meaningless). Classes: the Phase-I forward GEMM, the
   Phase-II reverse GEMM, the Phase-III layer kernel alone (recompute + vijp + epilogue), the
   weight-gradient GEMM alone, every elementwise/integer kernel, and the Phase-III launches as the
   step really issues them (layer i's kernel and layer i-1's weight gradient in one launch). */
#define MW_KCLASS_FWD    0
#define MW_KCLASS_REV    1
#define MW_KCLASS_VIJP   2
#define MW_KCLASS_DW     3
#define MW_KCLASS_EW     4
#define MW_KCLASS_PHASE3 5
#define MW_KCLASS_COUNT  6
/* kclass = -1 restores normal operation. Does not synchronise. */
int moonwalk_profile_filter(mw_handle_t* h, int32_t kclass);
/* Number of launches of the class made by the last moonwalk_grad / backprop_grad call. launches: host. */
int moonwalk_profile_launches(const mw_handle_t* h, int32_t kclass, uint64_t* launches);

/* Plain device-to-device copy kernel of n floats (bandwidth yardstick for the profiles). */
int mw_copy_f32(const float* src, float* dst, int64_t n, void* hip_stream);

/* Load-only model of a tiled NT product (measurement aid, computes nothing): one workgroup per
   tile x tile output tile of an M x N product reads its two operand row panels, A[M][K] and
   B[N][K] (device, row stride K, 16-byte aligned), the way the GEMM kernels do, and writes one
   checksum per thread to sink (device, at least (M/tile)*(N/tile)*256 floats). Its run time gives
   the rate at which the CUs can pull operand panels through their L1 caches, the bound of the
   small-batch products. The kernel is launched `repeats` (>= 1) times back to back, so that a
   caller timing the call is not bound by its own launch rate. tile is 16, 32 or 64; M and N must
   be multiples of tile, K of 256. MW_ERR_INVALID_ARG otherwise. */
int mw_probe_operand_stream(int32_t M, int32_t N, int32_t K, int32_t tile, const float* A, const float* B,
                            float* sink, int32_t repeats, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MOONWALK_BENCH_H */
