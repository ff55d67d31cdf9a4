// Tile variants of the bf16 MFMA GEMM: X(index, BM, BN, BK, WM, WN, direct).  direct = 1: the kernel
// whose global loads go straight into LDS (both operands K-contiguous only).  Each variant is compiled
// in its own translation unit (gemm_variant.hip with -DL2L_VARIANT=index) so that the build runs in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include "common.h"

#define L2L_GEMM_VARIANTS(X) \
  X(0, 128, 128, 64, 64, 64, 0) \
  X(1, 128, 64, 64, 64, 32, 0) \
  X(2, 256, 128, 64, 64, 64, 0) \
  X(3, 256, 256, 64, 128, 64, 0) \
  X(4, 256, 256, 64, 64, 128, 0) \
  X(5, 128, 256, 64, 64, 64, 0) \
  X(6, 256, 256, 64, 128, 64, 1) \
  X(7, 128, 128, 64, 64, 64, 1) \
  X(8, 256, 128, 64, 64, 64, 1)

constexpr int kNumGemmVariants = 9;

// launches variant `index` (layouts and output type taken from the arguments)
#define L2L_DECLARE(i, bm, bn, bk, wm, wn, d)                                                      \
  void l2l_launch_mfma_v##i(const GemmArgs& g, hipStream_t s, int splits, bool out_f32); /* bf16 */ \
  void l2l_launch_mfma_h##i(const GemmArgs& g, hipStream_t s, int splits, bool out_f32); /* fp16 */
L2L_GEMM_VARIANTS(L2L_DECLARE)
#undef L2L_DECLARE
