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

// GELU in its exact (erf) form and its derivative.
__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  return 0.5f * (1.0f + erff(u * 0.70710678118654752f)) + u * __expf(-0.5f * u * u) * 0.39894228040143268f;
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
