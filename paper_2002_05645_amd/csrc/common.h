// Shared device helpers for the L2L kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef _Float16 fp16;
typedef __attribute__((ext_vector_type(8))) _Float16 fp16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define WAVE 64

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return (float)x; }
__device__ __forceinline__ float to_f32(fp16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { return (bf16)x; }  // round to nearest even
template <> __device__ __forceinline__ fp16 from_f32<fp16>(float x) { return (fp16)x; }  // round to nearest even, overflow to inf

// Reductions over the 64 lanes of a wave (every lane active; every lane gets the result).  Within a row of 16 lanes the
// partners come through DPP operands of the add itself (quad permutes, then the mirror of a half row, then of the row);
// the four rows' results are read out as scalars.  No step goes through the LDS crossbar, whose round trip a chain of
// six dependent shuffles would pay six times over.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float lane_value(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);   // row_half_mirror
  v += dpp_move<0x140>(v);   // row_mirror
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v));
  v = fmaxf(v, dpp_move<0x4E>(v));
  v = fmaxf(v, dpp_move<0x141>(v));
  v = fmaxf(v, dpp_move<0x140>(v));
  return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}

// ---- 8-wide vector access ------------------------------------------------------------------------
__device__ __forceinline__ void load8(const float* p, float v[8]) {
  const f32x4 a = *(const f32x4*)p, b = *(const f32x4*)(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16* p, float v[8]) {
  const bf16x8 a = *(const bf16x8*)p;
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (float)a[i];
}
__device__ __forceinline__ void load8(const fp16* p, float v[8]) {
  const fp16x8 a = *(const fp16x8*)p;
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (float)a[i];
}
__device__ __forceinline__ void store8(float* p, const float v[8]) {
  *(f32x4*)p = f32x4{v[0], v[1], v[2], v[3]};
  *(f32x4*)(p + 4) = f32x4{v[4], v[5], v[6], v[7]};
}
__device__ __forceinline__ void store8(bf16* p, const float v[8]) {
  bf16x8 a;
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = (bf16)v[i];
  *(bf16x8*)p = a;
}

__device__ __forceinline__ void store8(fp16* p, const float v[8]) {
  fp16x8 a;
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = (fp16)v[i];
  *(fp16x8*)p = a;
}

// 8 x 16-bit values already in registers (as loaded with one 16-byte access) to fp32
template <typename E>
__device__ __forceinline__ void unpack8(u32x4 raw, float v[8]) {
  typedef __attribute__((ext_vector_type(8))) E e8;
  const e8 a = __builtin_bit_cast(e8, raw);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (float)a[i];
}

// One 32x32x16 MFMA step on 16-bit operands of element type E (fragments are carried as 8 x 16 bits).
template <typename E>
__device__ __forceinline__ f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c) {
  if constexpr (sizeof(E) == 2 && __is_same(E, fp16)) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(fp16x8, a), __builtin_bit_cast(fp16x8, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
}

// GELU in its exact (erf) form and its derivative.
__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  return 0.5f * (1.0f + erff(u * 0.70710678118654752f)) + u * __expf(-0.5f * u * u) * 0.39894228040143268f;
}

// Cheaper forms for the bf16 path, whose results are rounded to bf16 (relative step 2^-8) anyway: no
// transcendental instructions, one odd polynomial each, fitted (minimax, in s = u / a) to the exact
// functions on [-a, a] with the value at s = 1 pinned to the limit (P(1) = Q(1) = 1/2); outside, u is
// clamped to the interval, so the tails are 0 and 1 to fp32 rounding (the true functions are within the
// fit's error of those limits there).
//   Phi(u) = 1/2 (1 + erf(u / sqrt 2)) = 1/2 + s P(s^2),  a = 4,   |error| < 4e-5
//   gelu'(u) = Phi(u) + u phi(u)      = 1/2 + s Q(s^2),  a = 4.5, |error| < 2e-4 (fp32 rounding of Q included)
__device__ __forceinline__ float gelu_fast_f(float u) {
  const float s = __builtin_amdgcn_fmed3f(u, -4.0f, 4.0f) * 0.25f;
  const float t = s * s;
  float p = -1.372012435e+00f;
  p = fmaf(p, t, 7.008298544e+00f);
  p = fmaf(p, t, -1.555825966e+01f);
  p = fmaf(p, t, 1.997211423e+01f);
  p = fmaf(p, t, -1.672855746e+01f);
  p = fmaf(p, t, 9.811292493e+00f);
  p = fmaf(p, t, -4.228097766e+00f);
  p = fmaf(p, t, 1.595222051e+00f);
  return u * fmaf(p, s, 0.5f);
}
__device__ __forceinline__ float gelu_grad_fast_f(float u) {
  const float s = __builtin_amdgcn_fmed3f(u, -4.5f, 4.5f) * (1.0f / 4.5f);
  const float t = s * s;
  float p = -6.218507148e+01f;
  p = fmaf(p, t, 3.462898774e+02f);
  p = fmaf(p, t, -8.493878126e+02f);
  p = fmaf(p, t, 1.214708786e+03f);
  p = fmaf(p, t, -1.132123153e+03f);
  p = fmaf(p, t, 7.287199075e+02f);
  p = fmaf(p, t, -3.336748434e+02f);
  p = fmaf(p, t, 1.087429044e+02f);
  p = fmaf(p, t, -2.418076579e+01f);
  p = fmaf(p, t, 3.590171402e+00f);
  return fmaf(p, s, 0.5f);
}

// GELU and its derivative from one evaluation of Phi: gelu(u) = u Phi(u), gelu'(u) = Phi(u) + u phi(u) with the
// density phi(u) = exp(-u^2 / 2) / sqrt(2 pi) from the hardware's exponential (one transcendental instruction
// instead of the second polynomial; |error| of gelu' = that of Phi, < 4e-5).  For the forward GEMM of a recompute
// pass, which has u in registers and can leave gelu'(u) behind for the backward pass.
__device__ __forceinline__ void gelu_and_grad_fast_f(float u, float& gelu, float& grad) {
  const float s = __builtin_amdgcn_fmed3f(u, -4.0f, 4.0f) * 0.25f;
  const float t = s * s;
  float p = -1.372012435e+00f;
  p = fmaf(p, t, 7.008298544e+00f);
  p = fmaf(p, t, -1.555825966e+01f);
  p = fmaf(p, t, 1.997211423e+01f);
  p = fmaf(p, t, -1.672855746e+01f);
  p = fmaf(p, t, 9.811292493e+00f);
  p = fmaf(p, t, -4.228097766e+00f);
  p = fmaf(p, t, 1.595222051e+00f);
  const float cdf = fmaf(p, s, 0.5f);
  gelu = u * cdf;
  // exp(-u^2 / 2) = 2^(-u^2 log2(e) / 2); beyond |u| = 13 the argument is clamped (the density is 0 to fp32 there)
  const float e = __builtin_amdgcn_exp2f(fmaxf(u * u * -0.72134752044448170f, -126.0f));
  grad = fmaf(u * e, 0.39894228040143268f, cdf);
}

// GELU of the 16-bit epilogues: the polynomial forms.  Their absolute errors (4e-5 and 2e-4) are below half a unit
// in the last place of bf16 everywhere and of fp16 (2.4e-4 relative) wherever the result exceeds 0.2 and 0.8; below
// that they stay under one unit.
template <typename E> __device__ __forceinline__ float gelu_epi(float u) { return gelu_fast_f(u); }
template <typename E> __device__ __forceinline__ float gelu_grad_epi(float u) { return gelu_grad_fast_f(u); }
template <typename E> __device__ __forceinline__ void gelu_and_grad_epi(float u, float& g, float& d) { gelu_and_grad_fast_f(u, g, d); }

// Epilogue flags of the GEMM kernels.
// EPI_COLSUM: also leave the column sums of the stored values in GemmArgs::colsum (a bias gradient that would
// otherwise cost a pass over the output); the direct-to-LDS kernel's 16-byte epilogue path only.
// EPI_KEEPGRAD (with EPI_GELU and aux_out): aux_out receives gelu'(u) instead of the pre-activation u.
// EPI_MULAUX: the result is multiplied by aux element-wise (aux = gelu'(u) kept by such a forward GEMM).
enum { EPI_BIAS = 1, EPI_GELU = 2, EPI_GELUGRAD = 4, EPI_RESID = 8, EPI_ACCUM = 16, EPI_COLSUM = 32, EPI_KEEPGRAD = 64, EPI_MULAUX = 128 };

// One GEMM launch: C[M,N] = epi(alpha * sum_k A(m,k) B(k,n)), optionally batched over z.
struct GemmArgs {
  const void* A;
  const void* B;
  void* C;
  int M, N, K;
  int a_kc, b_kc;         // 1: operand stored with K contiguous ([M,K] / [N,K]); 0: [K,M] / [K,N]
  long long lda, ldb, ldc;  // row strides in elements
  int nbatch, zdiv;       // z -> (z / zdiv, z % zdiv)
  long long a_zo, a_zi, b_zo, b_zi, c_zo, c_zi;  // batch offsets in elements
  float alpha;
  int epi;
  const void* bias;       // [N]
  const void* resid;      // [M,N], row stride ldr
  long long ldr;
  const void* aux;        // EPI_GELUGRAD: pre-activation [M,N], row stride ldaux; EPI_MULAUX: the factor
  void* aux_out;          // EPI_GELU: where to keep the pre-activation, or with EPI_KEEPGRAD gelu' of it (or null)
  long long ldaux;
  const int* m_dev;       // optional device-side bound on M (rows beyond it are not computed)
  const int* k_dev;       // optional device-side bound on K
  long long split_stride; // direct-to-LDS kernel with K split over grid.y: 0 = the splits add into C with atomics; otherwise
                          // split s stores its partial result at C + s * split_stride (elements) and the caller adds them up
  int resident;           // direct-to-LDS kernel: > 0 = launch at most this many workgroups (one per compute unit) and let
                          // each walk its share of the tile order; 0 = one workgroup per tile
  float* colsum;          // EPI_COLSUM: fp32 [ceil(M / WM)][N] (WM = rows of a wave's tile): row r receives the column sums
                          // of the values stored to rows r WM .. r WM + WM - 1 of C (plain stores; the caller adds the rows up)
};

// Whether a launch takes the epilogue's 16-byte path (8 columns per lane); the kernels test it per launch, the host
// tests it before it asks for EPI_COLSUM, which only that path provides.  C: the output of the batch entry.
__host__ __device__ inline bool gemm_vec_ok(const GemmArgs& g, int epi, const void* C) {
  const auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  return (g.N % 8 == 0) && (g.ldc % 8 == 0) && al16(C) && (!(epi & EPI_BIAS) || al16(g.bias)) &&
         (!(epi & EPI_RESID) || (g.ldr % 8 == 0 && al16(g.resid))) &&
         (!(epi & (EPI_GELUGRAD | EPI_MULAUX)) || (g.ldaux % 8 == 0 && al16(g.aux))) &&
         (!((epi & EPI_GELU) && g.aux_out) || (g.ldaux % 8 == 0 && al16(g.aux_out))) &&
         (!(epi & EPI_COLSUM) || al16(g.colsum));
}
