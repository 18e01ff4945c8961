"""Mixed-mode Moonwalk gradients for dense submersive networks on MI355X.

Thin Python binding over the C-ABI library `libmoonwalk.so` (HIP, gfx950). Every step of the
method runs in the library's kernels; torch only provides device memory and the stream.
There is no CPU fallback: without the built library, or without a GPU, calls raise.
"""
from .binding import (ConvMoonwalkNet, conv_im2col, conv_col2im, conv_forward, conv_input_cotangent, conv_weight_grad, MoonwalkError, MoonwalkNet, GradResult, load_library, library_path,
                      gemm_f32, bias_act_mask, rev_scale, frag_offsets, frag_compact,
                      vijp_epilogue, colsum, colsum_wide, colsum_wide_noalloc, loss_grad, copy_f32, probe_operand_stream,
                      GEMM_NT, GEMM_NN, GEMM_TN, TILE_AUTO, TILE_128, TILE_64, TILE_32K4, TILE_32K8, TILE_64K2, TILE_128W8, TILE_64X128,
                      PLAN_MOONWALK, PLAN_BACKPROP, CONV_KERNELS_AUTO, CONV_KERNELS_PATCH_MATRIX, CONV_H0_FULL, CONV_H0_AS_READ, CONV_SUBMERSIVE, CONV_FRAGMENTAL_1D, EXPORTED_SYMBOLS)

__all__ = ["ConvMoonwalkNet", "conv_im2col", "conv_col2im", "conv_forward", "conv_input_cotangent", "conv_weight_grad", "MoonwalkError", "MoonwalkNet", "GradResult", "load_library", "library_path",
           "gemm_f32", "bias_act_mask", "rev_scale", "frag_offsets", "frag_compact",
           "vijp_epilogue", "colsum", "colsum_wide", "colsum_wide_noalloc", "loss_grad", "copy_f32", "probe_operand_stream",
           "GEMM_NT", "GEMM_NN", "GEMM_TN", "TILE_AUTO", "TILE_128", "TILE_64", "TILE_32K4", "TILE_32K8", "TILE_64K2", "TILE_128W8", "TILE_64X128",
           "PLAN_MOONWALK", "PLAN_BACKPROP", "CONV_KERNELS_AUTO", "CONV_KERNELS_PATCH_MATRIX", "CONV_H0_FULL", "CONV_H0_AS_READ", "CONV_SUBMERSIVE", "CONV_FRAGMENTAL_1D", "EXPORTED_SYMBOLS"]
