// Shared device helpers for the L2L kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define WAVE 64

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { return (bf16)x; }  // round to nearest even

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
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

// GELU in its exact (erf) form and its derivative.
__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  return 0.5f * (1.0f + erff(u * 0.70710678118654752f)) + u * __expf(-0.5f * u * u) * 0.39894228040143268f;
}

// Cheaper forms for the bf16 path, whose results are rounded to bf16 anyway: erf by the rational
// approximation erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p x), x >= 0 (Abramowitz and
// Stegun 7.1.26, absolute error below 1.5e-7).  phi_out receives exp(-u^2 / 2), which the derivative needs.
__device__ __forceinline__ float erf_as(float x, float& e) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  e = __expf(-ax * ax);
  const float r = 1.0f - p * t * e;
  return copysignf(r, x);
}
__device__ __forceinline__ float gelu_fast_f(float u) {
  float e;
  return 0.5f * u * (1.0f + erf_as(u * 0.70710678118654752f, e));
}
__device__ __forceinline__ float gelu_grad_fast_f(float u) {
  float e;
  const float cdf = 0.5f * (1.0f + erf_as(u * 0.70710678118654752f, e));
  return fmaf(u * e, 0.39894228040143268f, cdf);
}

// Epilogue flags of the GEMM kernels.
enum { EPI_BIAS = 1, EPI_GELU = 2, EPI_GELUGRAD = 4, EPI_RESID = 8, EPI_ACCUM = 16 };

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
  const void* aux;        // EPI_GELUGRAD: pre-activation [M,N], row stride ldaux
  void* aux_out;          // EPI_GELU: where to keep the pre-activation (or null)
  long long ldaux;
  const int* m_dev;       // optional device-side bound on M (rows beyond it are not computed)
  const int* k_dev;       // optional device-side bound on K
};
