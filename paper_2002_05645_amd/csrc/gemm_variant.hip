// One tile variant of the 16-bit MFMA GEMM (selected with -DL2L_VARIANT=<index>): all four operand
// layouts, 16-bit and fp32 outputs.
#include "gemm.h"
#include "gemm_variants.h"

#ifndef L2L_VARIANT
#error "compile with -DL2L_VARIANT=<index>"
#endif

namespace {

template <int BM, int BN, int BK, int WM, int WN, bool AKC, bool BKC, typename TC, typename E>
void launch_one(const GemmArgs& g, hipStream_t s, int splits) {
  constexpr int LDS = 2 * (TileLds<BM, BK>::BYTES + TileLds<BN, BK>::BYTES);
  static_assert(LDS <= 160 * 1024, "tile does not fit the 160 KB LDS");
  auto kern = gemm_mfma_kernel<BM, BN, BK, WM, WN, AKC, BKC, TC, E>;
  static const bool once = [&] {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    return true;
  }();
  (void)once;
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  dim3 grid(tiles, splits, g.nbatch), block((BM / WM) * (BN / WN) * 64);
  hipLaunchKernelGGL(kern, grid, block, LDS, s, g);
}

template <int BM, int BN, int BK, int WM, int WN, typename TC, typename E>
void launch_layout(const GemmArgs& g, hipStream_t s, int splits) {
  if (g.a_kc && g.b_kc) launch_one<BM, BN, BK, WM, WN, true, true, TC, E>(g, s, splits);
  else if (g.a_kc && !g.b_kc) launch_one<BM, BN, BK, WM, WN, true, false, TC, E>(g, s, splits);
  else if (!g.a_kc && g.b_kc) launch_one<BM, BN, BK, WM, WN, false, true, TC, E>(g, s, splits);
  else launch_one<BM, BN, BK, WM, WN, false, false, TC, E>(g, s, splits);
}

}  // namespace

template <int BM, int BN, int WM, int WN, bool AKC, bool BKC, typename TC, typename E, int EPI = -1>
void launch_direct_one(const GemmArgs& g, hipStream_t s, int splits) {
  constexpr int LDS = dlds_lds_bytes<BM, BN, WM, WN>();
  static_assert(LDS <= 160 * 1024, "tile does not fit the 160 KB LDS");
  auto kern = gemm_mfma_dlds_kernel<BM, BN, WM, WN, AKC, BKC, TC, E, EPI>;
  static const bool once = [&] {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    return true;
  }();
  (void)once;
  const int num_cus = g.resident / 8 * 8;   // a multiple of the 8 XCDs keeps each resident workgroup's tiles on its own XCD's range
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  // more tiles than CUs: one resident workgroup per CU walks the tile order (the kernel's loop)
  const int gx = (num_cus > 0 && splits == 1 && g.nbatch == 1 && tiles > num_cus) ? num_cus : tiles;
  dim3 grid(gx, splits, g.nbatch), block((BM / WM) * (BN / WN) * 64);
  hipLaunchKernelGGL(kern, grid, block, LDS, s, g);
}

// the direct-to-LDS kernel is built for the two layout pairs that carry the layer's work: both operands
// K-contiguous (forward with transposed weights, dX) and both K-strided (dW)
template <int BM, int BN, int WM, int WN, typename TC, typename E>
void launch_direct(const GemmArgs& g, hipStream_t s, int splits) {
  // The 256 x 256 tile with 16-bit output and both operands K-contiguous carries the layer's forward, recompute and
  // dX GEMMs: their eight epilogues get kernels with the flags compiled in (a third off the epilogue's time); any
  // other combination runs the kernel that reads the flags at run time.
  if constexpr (BM == 256 && BN == 256 && sizeof(TC) == 2) {
    if (g.a_kc && g.b_kc && g.alpha == 1.0f) {
      switch (g.epi) {
#define L2L_EPI_CASE(e) case (e): launch_direct_one<BM, BN, WM, WN, true, true, TC, E, (e)>(g, s, splits); return;
        L2L_EPI_CASE(0)
        L2L_EPI_CASE(EPI_BIAS)
        L2L_EPI_CASE(EPI_BIAS | EPI_RESID)
        L2L_EPI_CASE(EPI_BIAS | EPI_GELU)
        L2L_EPI_CASE(EPI_BIAS | EPI_GELU | EPI_KEEPGRAD)
        L2L_EPI_CASE(EPI_MULAUX)
        L2L_EPI_CASE(EPI_MULAUX | EPI_COLSUM)
        L2L_EPI_CASE(EPI_RESID)
#undef L2L_EPI_CASE
        default: break;
      }
    }
  }
  if (g.a_kc && g.b_kc) launch_direct_one<BM, BN, WM, WN, true, true, TC, E>(g, s, splits);
  else if (g.a_kc) launch_direct_one<BM, BN, WM, WN, true, false, TC, E>(g, s, splits);
  else launch_direct_one<BM, BN, WM, WN, false, false, TC, E>(g, s, splits);
}

struct TileCfg { int bm, bn, bk, wm, wn, direct; };
#define L2L_ROW(i, bm, bn, bk, wm, wn, d) {bm, bn, bk, wm, wn, d},
constexpr TileCfg kCfg[] = {L2L_GEMM_VARIANTS(L2L_ROW)};
#undef L2L_ROW
constexpr TileCfg kThis = kCfg[L2L_VARIANT];

#define L2L_CAT2(a, b) a##b
#define L2L_CAT(a, b) L2L_CAT2(a, b)
// The element type of the 16-bit operands is fixed per translation unit (-DL2L_ELEM_FP16 selects IEEE half, default
// bfloat16), so that each format's kernels sit in a code object of their own.
#ifdef L2L_ELEM_FP16
typedef fp16 Elem;
#define L2L_LAUNCH_NAME L2L_CAT(l2l_launch_mfma_h, L2L_VARIANT)
#else
typedef bf16 Elem;
#define L2L_LAUNCH_NAME L2L_CAT(l2l_launch_mfma_v, L2L_VARIANT)
#endif

void L2L_LAUNCH_NAME(const GemmArgs& g, hipStream_t s, int splits, bool out_f32) {
  if constexpr (kThis.direct) {   // callers pick these variants for every layout pair but (A K-strided, B K-contiguous)
    if (out_f32) launch_direct<kThis.bm, kThis.bn, kThis.wm, kThis.wn, float, Elem>(g, s, splits);
    else launch_direct<kThis.bm, kThis.bn, kThis.wm, kThis.wn, Elem, Elem>(g, s, 1);
  } else {
    if (out_f32) launch_layout<kThis.bm, kThis.bn, kThis.bk, kThis.wm, kThis.wn, float, Elem>(g, s, splits);
    else launch_layout<kThis.bm, kThis.bn, kThis.bk, kThis.wm, kThis.wn, Elem, Elem>(g, s, 1);
  }
}
