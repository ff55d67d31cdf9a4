// Fused attention for the 16-bit paths (element type E = bf16 or fp16), head width d = 64, sequence length a
// multiple of 32 up to 128: scores, softmax and context (forward) and all five attention gradients (backward)
// of one (sequence, head) pair in one workgroup, without the S x S matrices ever leaving the chip.  Longer
// sequences (multiples of 32) go through the chunked kernels at the end of this file.
//
// Everything is computed "transposed": the MFMA tiles are S^T = K Q^T (keys along the accumulator's
// register axis, queries along its lane axis), so that a softmax row lives in the registers of one
// lane pair and row reductions are register adds plus one cross-lane exchange.  The 32x32x16 MFMA's
// accumulator gives lane l the column l % 32 and, per register r, the row 8 (r / 4) + 4 (l / 32) + r % 4;
// eight consecutive registers therefore hold, for one query, exactly the eight keys that the same
// lane must supply as the B operand of the next product over keys (the contraction index may be
// permuted freely as long as both operands agree), so P and dS feed O^T = V^T P^T and
// dQ^T = K^T dS^T straight from registers.  Operands that are needed with the contraction index
// strided in memory (V^T, K^T, and everything contracted over queries) come out of their natural
// [row][64] LDS image through ds_read_b64_tr_b16.
//
// LDS images are [row][64] 16-bit elements (128-byte rows) with the 16-byte chunk c of row r at slot
// c ^ ((r >> 1) & 7): conflict-free for 16-byte fragment reads, two-way for the transpose reads (a layout that
// spreads the four rows of a transposing read over all banks, slot c ^ (2 (r % 4) + (r / 4) % 2), measured the same).
#pragma once
#include "gemm.h"

namespace attn {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

// Orders a wave's own LDS traffic for the compiler (LDS executes a wave's accesses in order; a wave that exchanges data
// between its lanes through a region nobody else touches needs no barrier)
__device__ __forceinline__ void wave_lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// rows [0, S) of a [S][64] slice with row pitch `ld` elements, straight into LDS (1 KiB = 8 rows per instruction)
__device__ __forceinline__ void load_rows(__amdgpu_buffer_rsrc_t rs, uint32_t ld, int S, char* dst, int wave, int nwaves, int lane) {
  for (int blk = wave; blk < S / 8; blk += nwaves) {
    const int row = blk * 8 + (lane >> 3);
    const int c = swz(row, lane & 7);
    const uint32_t off = ((uint32_t)row * ld + (uint32_t)c * 8) * 2u;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)(dst + blk * 1024), 16, (int)off, 0, 0, 0);
  }
}

// rows 32 w .. 32 w + 31 of the slice, into the same rows of the image (four instructions)
__device__ __forceinline__ void load_rows_own(__amdgpu_buffer_rsrc_t rs, uint32_t ld, char* dst, int wave, int lane) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int blk = wave * 4 + i, row = blk * 8 + (lane >> 3);
    const int c = swz(row, lane & 7);
    const uint32_t off = ((uint32_t)row * ld + (uint32_t)c * 8) * 2u;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)(dst + blk * 1024), 16, (int)off, 0, 0, 0);
  }
}

// at most n (1..4) vector-memory loads of this wave still outstanding (nothing is scheduled across the wait: the
// callers count the loads they have issued)
__device__ __forceinline__ void wait_vm_upto(int n) {
  __builtin_amdgcn_sched_barrier(0);
  if (n >= 4) __builtin_amdgcn_s_waitcnt(0x0F74);
  else if (n == 3) __builtin_amdgcn_s_waitcnt(0x0F73);
  else if (n == 2) __builtin_amdgcn_s_waitcnt(0x0F72);
  else __builtin_amdgcn_s_waitcnt(0x0F71);
  __builtin_amdgcn_sched_barrier(0);
}
__device__ __forceinline__ void wait_lds0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// fragment with rows as the M/N index: 8 consecutive columns (k = 16 step + 8 (lane / 32) ..) of row `row`
__device__ __forceinline__ bf16x8 frag_rows(const char* img, int row, int step, int lane) {
  return *(const bf16x8*)(img + row * 128 + swz(row, step * 2 + (lane >> 5)) * 16);
}

// four consecutive rows (the contraction index) of column col0 + 16 ((lane / 16) & 1) + lane % 16
__device__ __forceinline__ s16x4 tr_read(const char* img, int row0, int col0, int lane) {
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const int i16 = lane & 15, R = i16 >> 2, Q = i16 & 3;
  const int row = row0 + R, col = col0 + 16 * ((lane >> 4) & 1) + Q * 4;
  const char* p = img + row * 128 + swz(row, col >> 3) * 16 + (col & 7) * 2;
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(__attribute__((address_space(3))) char*)p);
}

// A-operand fragment for a product over keys whose B operand comes from accumulator registers 8 s .. 8 s + 7 of
// key block kb: the keys are kb*32 + 16 s + 4 (lane / 32) + {0..3} and those + 8; column tile = 32 t
__device__ __forceinline__ bf16x8 frag_keys_T(const char* img, int kb, int s, int t, int lane) {
  const int base = kb * 32 + 16 * s + 4 * (lane >> 5);
  const s16x4 lo = tr_read(img, base, t * 32, lane), hi = tr_read(img, base + 8, t * 32, lane);
  const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// fragments travel as 8 x 16 bits (bf16x8) whatever the element type; only conversions and the MFMA look at E
template <typename E>
struct Vec { typedef __attribute__((ext_vector_type(8))) E x8; typedef __attribute__((ext_vector_type(4))) E x4; };

template <typename E>
__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int r0) {
  typename Vec<E>::x8 v;
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = from_f32<E>(a[r0 + i]);
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ float xor32_max(float v) { return fmaxf(v, __shfl_xor(v, 32, 64)); }
__device__ __forceinline__ float xor32_sum(float v) { return v + __shfl_xor(v, 32, 64); }

// store a transposed 2 x (32 x 32) accumulator pair (rows = 64 columns of the output, lane = output row) as
// out[(row0 + lane % 32) * ld + 8 blk + 4 (lane / 32) + {0..3} (+32 for the second tile)], scaled
template <typename E>
__device__ __forceinline__ void store_T(const f32x16 (&acc)[2], E* out, long long ld, int lane, float scale) {
  E* p = out + (long long)(lane & 31) * ld + 4 * (lane >> 5);
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      typename Vec<E>::x4 v;
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = from_f32<E>(acc[t][blk * 4 + i] * scale);
      *(typename Vec<E>::x4*)(p + t * 32 + blk * 8) = v;
    }
}

// Accumulators on their way out through LDS, so that global memory sees whole rows (a direct store puts 32 rows x 16
// bytes into every instruction): `stage` is a region that only this wave touches.
// NT = 2: 32 rows of 64 columns (128-byte rows, slot c ^ (r & 7)); NT = 1: 32 rows of 32 columns (64-byte rows in a
// 2 KiB region, slot c ^ ((r >> 1) & 3))
template <int NT> __device__ __forceinline__ int stage_swz(int r) { return NT == 2 ? (r & 7) : ((r >> 1) & 3); }

template <typename E, int NT>
__device__ __forceinline__ void stage_T(const f32x16 (&acc)[NT], char* stage, int lane, float scale) {
  const int q = lane & 31;
  char* p = stage + q * (NT * 64) + 8 * (lane >> 5);
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      typename Vec<E>::x4 v;
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = from_f32<E>(acc[t][blk * 4 + i] * scale);
      *(typename Vec<E>::x4*)(p + (((t * 4 + blk) ^ stage_swz<NT>(q)) * 16)) = v;
    }
}

// rows 0..31 of the staged image (4 NT lanes per row, 16 / NT rows per instruction) to out[row * ld + ..];
// colsum (or null, NT = 2 only): this wave's 64 column sums of what it stores, taken in fp32 from the rounded values
template <typename E, int NT>
__device__ __forceinline__ void store_staged(const char* stage, E* out, long long ld, int lane, float* colsum = nullptr) {
  constexpr int LPR = 4 * NT, RPI = 64 / LPR;   // lanes per row, rows per instruction
  const int c = lane & (LPR - 1);
  float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 32 / RPI; ++i) {
    const int r = i * RPI + lane / LPR;
    const bf16x8 v = *(const bf16x8*)(stage + r * (NT * 64) + ((c ^ stage_swz<NT>(r)) * 16));
    *(bf16x8*)(out + (long long)r * ld + c * 8) = v;
    if (NT == 2 && colsum) {
      const typename Vec<E>::x8 e = __builtin_bit_cast(typename Vec<E>::x8, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) cs[j] += to_f32(e[j]);
    }
  }
  if (NT == 2 && colsum) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      cs[j] += __shfl_xor(cs[j], 8, 64);
      cs[j] += __shfl_xor(cs[j], 16, 64);
      cs[j] += __shfl_xor(cs[j], 32, 64);
    }
    if (lane < 8) {
      *(float4*)(colsum + c * 8) = float4{cs[0], cs[1], cs[2], cs[3]};
      *(float4*)(colsum + c * 8 + 4) = float4{cs[4], cs[5], cs[6], cs[7]};
    }
  }
}

constexpr int SMAX = 128;   // longest sequence the fused kernels take
constexpr int NKB = SMAX / 32;

// Forward: out[b*S + q, h*64 ..] = softmax_rows(Q K^T * alpha) V for one (b, h) per workgroup; wave w owns queries
// 32 w .. 32 w + 31.  qkv: [rows, 3H] with Q | K | V column groups.
template <typename E>
__global__ __launch_bounds__(256) void attn_fwd_kernel(const E* qkv, E* out, int S, int H, int A, float alpha) {
  __shared__ __attribute__((aligned(1024))) char lds[2 * SMAX * 128];
  char* Ks = lds;
  char* Vs = lds + SMAX * 128;
  const int b = blockIdx.x / A, h = blockIdx.x % A;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long ld = 3LL * H;
  const E* base = qkv + (long long)b * S * ld + h * 64;
  const uint32_t bytes = (uint32_t)(((long long)(S - 1) * ld + 64) * 2);
  const int nkb = S / 32;
  const bool active = wave < nkb;
  // Wave w's 32 queries pass through rows 32 w .. of the image of V, which are its own until it has asked for those
  // rows of V itself (whole 128-byte rows from memory, like K and V; fragments read straight from memory would put
  // 32 rows x 32 bytes into every load).  Loads return in order: once only the nkb loads of K are outstanding, Q is in.
  if (active) load_rows_own(make_rsrc(base, bytes), (uint32_t)ld, Vs, wave, lane);
  load_rows(make_rsrc(base + H, bytes), (uint32_t)ld, S, Ks, wave, 4, lane);
  bf16x8 qf[4];
  if (active) {
    wait_vm_upto(nkb);
    wave_lds_order();
#pragma unroll
    for (int st = 0; st < 4; ++st) qf[st] = frag_rows(Vs, wave * 32 + (lane & 31), st, lane);
    wait_lds0();   // the fragments are in registers before the loads of V may write over them
    wave_lds_order();
    load_rows_own(make_rsrc(base + 2 * H, bytes), (uint32_t)ld, Vs, wave, lane);
    wait_vm_upto(4);   // K is in (this wave's part), V on its way
  } else {
    wait_vm0();
  }
  __syncthreads();

  f32x16 st_[NKB];
  float m = -INFINITY;
  if (active) {
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      if (kb < nkb) {
        f32x16 a = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4)
          a = mfma_32x32x16<E>(frag_rows(Ks, kb * 32 + (lane & 31), s4, lane), qf[s4], a);
#pragma unroll
        for (int r = 0; r < 16; ++r) { a[r] *= alpha; m = fmaxf(m, a[r]); }
        st_[kb] = a;
      }
    }
  }
  wait_vm0();
  __syncthreads();   // V is in; nobody reads the image of K any more: rows 32 w .. of it are wave w's way out for its context rows
  if (!active) return;
  m = xor32_max(m);
  float sum = 0.f;
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
    if (kb < nkb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) { st_[kb][r] = __expf(st_[kb][r] - m); sum += st_[kb][r]; }
    }
  sum = xor32_sum(sum);
  const float inv = 1.0f / sum;

  f32x16 o[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) o[t] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
    if (kb < nkb) {
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8 pf = pack8<E>(st_[kb], 8 * s2);
#pragma unroll
        for (int t = 0; t < 2; ++t) o[t] = mfma_32x32x16<E>(frag_keys_T(Vs, kb, s2, t, lane), pf, o[t]);
      }
    }
  char* stage = Ks + wave * 4096;
  stage_T<E, 2>(o, stage, lane, inv);
  wave_lds_order();
  store_staged<E, 2>(stage, out + ((long long)b * S + wave * 32) * H + h * 64, H, lane);
}


// ---- backward ------------------------------------------------------------------------------------------
// image of P or dS for products over queries, one half of the keys at a time: [q][64] 16-bit elements, 128-byte rows,
// the 32-byte group holding keys 16 p .. 16 p + 15 of row q at group slot p ^ (q & 3) (so that four consecutive
// query rows hit different banks)
__device__ __forceinline__ int pq_addr(int q, int key) { return q * 128 + (((key >> 4) ^ (q & 3)) * 32) + (key & 15) * 2; }

// key block kb2 (0 or 1) of the half
template <typename E>
__device__ __forceinline__ void pq_store(char* img, const f32x16& a, int q, int kb2, int lane) {
#pragma unroll
  for (int blk = 0; blk < 4; ++blk) {
    typename Vec<E>::x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = from_f32<E>(a[blk * 4 + i]);
    *(typename Vec<E>::x4*)(img + pq_addr(q, kb2 * 32 + 8 * blk + 4 * (lane >> 5))) = v;
  }
}

// B-operand fragment over queries 16 s + 8 (lane / 32) .. + 7 for key column 32 kb2 + lane % 32 of the half
__device__ __forceinline__ bf16x8 pq_frag(const char* img, int s, int kb2, int lane) {
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const int i16 = lane & 15, R = i16 >> 2, Q = i16 & 3;
  const int q0 = 16 * s + 8 * (lane >> 5) + R, key = 32 * kb2 + 16 * ((lane >> 4) & 1) + Q * 4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(__attribute__((address_space(3))) char*)(img + pq_addr(q0, key)));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(__attribute__((address_space(3))) char*)(img + pq_addr(q0 + 4, key)));
  const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// A-operand fragment over queries 16 s + 8 (lane / 32) .. + 7 for column 32 t + lane % 32 of a [q][64] image
__device__ __forceinline__ bf16x8 frag_queries_T(const char* img, int s, int t, int lane) {
  const int q0 = 16 * s + 8 * (lane >> 5);
  const s16x4 lo = tr_read(img, q0, t * 32, lane), hi = tr_read(img, q0 + 4, t * 32, lane);
  const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// 64 KB: two workgroups fit a CU, so that one's loads and stores run under the other's MFMAs
constexpr int BWD_LDS = 4 * SMAX * 128;

// Backward for one (b, h) per workgroup.  dout: [rows, H] gradient of the context; dqkv: [rows, 3H] receives
// dQ | dK | dV.  Phase 1 (wave w = queries 32 w ..): recompute P, dP = dO V^T, dS = P (dP - rowsum(P dP)),
// dQ = alpha dS K; P and dS stay in registers.  Phase 2, once per half of the keys (0..63, 64..127): the waves park
// that half of P and dS in LDS, over the images of K and V, which nobody needs any more, and then wave w takes key
// block w % 2 of the half and columns 32 (w / 2) .. of the head: dV = P^T dO, dK = alpha dS^T Q.
// dq_colsum (or null): fp32 [rows / 32][H]; row (b S + 32 w) / 32 receives the column sums of the 32 rows of dQ that wave
// w stores (the Q part of the QKV bias gradient, which the caller adds up over the rows).
// Two waves per SIMD (two workgroups per CU) is what the 64 KB of LDS allow and what the registers are held to.
template <typename E>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_bwd_kernel(const E* qkv, const E* dout, E* dqkv, float* dq_colsum, int S, int H, int A, float alpha) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  char* Ks = lds;
  char* Vs = lds + SMAX * 128;
  char* Qs = lds + 2 * SMAX * 128;
  char* Os = lds + 3 * SMAX * 128;
  char* Ps = Ks;   // phase 2
  char* Ds = Vs;
  const int b = blockIdx.x / A, h = blockIdx.x % A;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long ld = 3LL * H;
  const E* base = qkv + (long long)b * S * ld + h * 64;
  const uint32_t bytes = (uint32_t)(((long long)(S - 1) * ld + 64) * 2);
  load_rows(make_rsrc(base, bytes), (uint32_t)ld, S, Qs, wave, 4, lane);
  load_rows(make_rsrc(base + H, bytes), (uint32_t)ld, S, Ks, wave, 4, lane);
  load_rows(make_rsrc(base + 2 * H, bytes), (uint32_t)ld, S, Vs, wave, 4, lane);
  const E* dob = dout + (long long)b * S * H + h * 64;
  load_rows(make_rsrc(dob, (uint32_t)(((long long)(S - 1) * H + 64) * 2)), (uint32_t)H, S, Os, wave, 4, lane);
  const int nkb = S / 32;
  const bool active = wave < nkb;
  wait_vm0();
  __syncthreads();

  E* dqkv_b = dqkv + (long long)b * S * ld + h * 64;
  const int qrow = wave * 32 + (lane & 31);
  f32x16 p_[NKB], ds_[NKB], dq[2];
  if (active) {
    bf16x8 qf[4], of[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) { qf[s4] = frag_rows(Qs, qrow, s4, lane); of[s4] = frag_rows(Os, qrow, s4, lane); }
    float m = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
      if (kb < nkb) {
        f32x16 a = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 d = a;
        const int krow = kb * 32 + (lane & 31);
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          a = mfma_32x32x16<E>(frag_rows(Ks, krow, s4, lane), qf[s4], a);
          d = mfma_32x32x16<E>(frag_rows(Vs, krow, s4, lane), of[s4], d);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) { a[r] *= alpha; m = fmaxf(m, a[r]); }
        p_[kb] = a;
        ds_[kb] = d;
      }
    m = xor32_max(m);
    float sum = 0.f;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
      if (kb < nkb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) { p_[kb][r] = __expf(p_[kb][r] - m); sum += p_[kb][r]; }
      }
    const float inv = 1.0f / xor32_sum(sum);
    float dsum = 0.f;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
      if (kb < nkb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) { p_[kb][r] *= inv; dsum += p_[kb][r] * ds_[kb][r]; }
      }
    dsum = xor32_sum(dsum);
#pragma unroll
    for (int t = 0; t < 2; ++t) dq[t] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
      if (kb < nkb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) ds_[kb][r] = p_[kb][r] * (ds_[kb][r] - dsum);   // dP -> dS
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 df = pack8<E>(ds_[kb], 8 * s2);
#pragma unroll
          for (int t = 0; t < 2; ++t) dq[t] = mfma_32x32x16<E>(frag_keys_T(Ks, kb, s2, t, lane), df, dq[t]);
        }
      }
  }
  // phase 2: keys 64 half .. 64 half + 63.  Results leave through LDS (whole rows for global memory): rows 32 w .. of
  // the images of P and dS belong to wave w alone between the two barriers below, so they serve as its way out first,
  // for dQ (first half) or for the previous half's dV and dK
  f32x16 dv[1], dk[1];
  E* dkv_out = nullptr;
  char* stage = Ps + wave * 4096;
  const auto flush_dkv = [&]() {
    stage_T<E, 1>(dv, stage, lane, 1.0f);
    stage_T<E, 1>(dk, stage + 2048, lane, alpha);
    wave_lds_order();
    store_staged<E, 1>(stage, dkv_out + 2 * H, ld, lane);
    store_staged<E, 1>(stage + 2048, dkv_out + H, ld, lane);
    wave_lds_order();
  };
#pragma unroll
  for (int half = 0; half < NKB / 2; ++half) {
    if (2 * half >= nkb) break;
    __syncthreads();   // K and V (first half) or the previous half's P and dS are no longer read
    if (half == 0 && active) {
      stage_T<E, 2>(dq, stage, lane, alpha);
      wave_lds_order();
      store_staged<E, 2>(stage, dqkv_b + (long long)wave * 32 * ld, ld, lane,
                         dq_colsum ? dq_colsum + ((long long)(b * nkb + wave) * H + h * 64) : nullptr);
      wave_lds_order();
    }
    if (half > 0 && dkv_out) flush_dkv();
    if (active) {
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
        if (2 * half + kb2 < nkb) {
          pq_store<E>(Ps, p_[2 * half + kb2], qrow, kb2, lane);
          pq_store<E>(Ds, ds_[2 * half + kb2], qrow, kb2, lane);
        }
    }
    __syncthreads();
    const int kb2 = wave & 1, t = wave >> 1, kb = 2 * half + kb2;
    dkv_out = nullptr;
    if (kb < nkb) {
      dv[0] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      dk[0] = dv[0];
      for (int s = 0; s < S / 16; ++s) {
        const bf16x8 pf = pq_frag(Ps, s, kb2, lane), df = pq_frag(Ds, s, kb2, lane);
        dv[0] = mfma_32x32x16<E>(frag_queries_T(Os, s, t, lane), pf, dv[0]);
        dk[0] = mfma_32x32x16<E>(frag_queries_T(Qs, s, t, lane), df, dk[0]);
      }
      dkv_out = dqkv_b + (long long)kb * 32 * ld + t * 32;
    }
  }
  __syncthreads();   // the last half's P and dS are no longer read
  if (dkv_out) flush_dkv();
}

// ---- long sequences: S a multiple of 32 beyond SMAX -----------------------------------------------------
// A workgroup owns 128 queries (forward, dQ) or 128 keys (dK, dV) of one (sequence, head) pair and walks the other
// index in chunks of 128 rows that pass through LDS.  When S is not a multiple of 128 the last chunk is short: its
// missing 32-row blocks are skipped, and the waves whose own 32 rows lie beyond S only help with the loads (RAGGED
// instantiations; with S a multiple of 128 none of these tests is compiled in).  The forward pass keeps a running row maximum and row sum and
// rescales its context accumulators when the maximum moves; it leaves lse = max + log(sum) per query row, from which
// the backward kernels get P = exp(alpha S - lse) without a reduction.  rowsum(P dP) is taken as rowsum(dO O)
// (the same number: sum_k P_k dO . V_k = dO . O), computed by the dQ kernel from the stored context and passed on.
constexpr int CH = 128;

// (Each of the three kernels below states the least number of waves per SIMD it is to be compiled for: left alone, the
// compiler has settled on fewer, with more registers per wave and a third more time per launch.)
template <typename E, bool RAGGED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(RAGGED ? 2 : 3)))
void attn_fwd_long_kernel(const E* qkv, E* out, float* lse, int S, int H, int A, float alpha) {
  __shared__ __attribute__((aligned(1024))) char lds[2 * CH * 128];
  char* Ks = lds;
  char* Vs = lds + CH * 128;
  const int nch = (S + CH - 1) / CH;
  const int qb = blockIdx.x % nch, bh = blockIdx.x / nch, b = bh / A, h = bh % A;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long ld = 3LL * H;
  const E* base = qkv + (long long)b * S * ld + h * 64;
  const int q = qb * CH + wave * 32 + (lane & 31);
  const bool active = !RAGGED || qb * CH + wave * 32 < S;   // (per wave)
  bf16x8 qf[4];
  if (active) {
    const E* qrow = base + (long long)q * ld + (lane >> 5) * 8;
#pragma unroll
    for (int st = 0; st < 4; ++st) qf[st] = *(const bf16x8*)(qrow + st * 16);
  }
  float m = -INFINITY, sum = 0.f;
  f32x16 o[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) o[t] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int kc = 0; kc < nch; ++kc) {
    const int rows = RAGGED ? min(CH, S - kc * CH) : CH, nkb = rows / 32;   // this chunk's keys
    const uint32_t bytes = (uint32_t)(((long long)(rows - 1) * ld + 64) * 2);
    if (kc) __syncthreads();   // every wave has left the previous chunk
    load_rows(make_rsrc(base + H + (long long)kc * CH * ld, bytes), (uint32_t)ld, rows, Ks, wave, 4, lane);
    load_rows(make_rsrc(base + 2 * H + (long long)kc * CH * ld, bytes), (uint32_t)ld, rows, Vs, wave, 4, lane);
    wait_vm0();
    __syncthreads();
    if (!active) continue;
    f32x16 st_[CH / 32];
    float cm = m;
#pragma unroll
    for (int kb = 0; kb < CH / 32; ++kb)
      if (kb < nkb) {
        f32x16 a = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) a = mfma_32x32x16<E>(frag_rows(Ks, kb * 32 + (lane & 31), s4, lane), qf[s4], a);
#pragma unroll
        for (int r = 0; r < 16; ++r) { a[r] *= alpha; cm = fmaxf(cm, a[r]); }
        st_[kb] = a;
      }
    cm = xor32_max(cm);
    const float rescale = __expf(m - cm);   // 0 on the first chunk
    m = cm;
    float cs = 0.f;
#pragma unroll
    for (int kb = 0; kb < CH / 32; ++kb)
      if (kb < nkb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) { st_[kb][r] = __expf(st_[kb][r] - m); cs += st_[kb][r]; }
      }
    sum = sum * rescale + xor32_sum(cs);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[t][r] *= rescale;
#pragma unroll
    for (int kb = 0; kb < CH / 32; ++kb)
      if (kb < nkb) {
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 pf = pack8<E>(st_[kb], 8 * s2);
#pragma unroll
          for (int t = 0; t < 2; ++t) o[t] = mfma_32x32x16<E>(frag_keys_T(Vs, kb, s2, t, lane), pf, o[t]);
        }
      }
  }
  if (!active) return;
  store_T(o, out + ((long long)b * S + qb * CH + wave * 32) * H + h * 64, H, lane, 1.0f / sum);
  if (lse && lane < 32) lse[(long long)bh * S + q] = m + __logf(sum);
}

// dQ = alpha dS K for 128 queries per workgroup; also leaves dsum[row] = rowsum(dO O) for the dK / dV kernel.
// ctx: [rows, H], the forward pass's output.
template <typename E, bool RAGGED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3)))
void attn_bwd_dq_long_kernel(const E* qkv, const E* dout, const E* ctx, const float* lse,
                                                               float* dsum, E* dqkv, int S, int H, int A, float alpha) {
  __shared__ __attribute__((aligned(1024))) char lds[2 * CH * 128];
  char* Ks = lds;
  char* Vs = lds + CH * 128;
  const int nch = (S + CH - 1) / CH;
  const int qb = blockIdx.x % nch, bh = blockIdx.x / nch, b = bh / A, h = bh % A;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long ld = 3LL * H;
  const E* base = qkv + (long long)b * S * ld + h * 64;
  const int q = qb * CH + wave * 32 + (lane & 31);
  const bool active = !RAGGED || qb * CH + wave * 32 < S;   // (per wave)
  bf16x8 qf[4], of[4];
  float D = 0.f;
  if (active) {
    const E* qrow = base + (long long)q * ld + (lane >> 5) * 8;
    const long long orow = ((long long)b * S + q) * H + h * 64 + (lane >> 5) * 8;
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      qf[st] = *(const bf16x8*)(qrow + st * 16);
      of[st] = *(const bf16x8*)(dout + orow + st * 16);
      const typename Vec<E>::x8 gv = __builtin_bit_cast(typename Vec<E>::x8, of[st]);
      const typename Vec<E>::x8 cv = *(const typename Vec<E>::x8*)(ctx + orow + st * 16);
#pragma unroll
      for (int i = 0; i < 8; ++i) D += to_f32(gv[i]) * to_f32(cv[i]);
    }
  }
  D = xor32_sum(D);
  const long long srow = (long long)bh * S + q;
  const float L = active ? lse[srow] : 0.f;
  if (active && lane < 32) dsum[srow] = D;
  f32x16 dq[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) dq[t] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int kc = 0; kc < nch; ++kc) {
    const int rows = RAGGED ? min(CH, S - kc * CH) : CH, nkb = rows / 32;   // this chunk's keys
    const uint32_t bytes = (uint32_t)(((long long)(rows - 1) * ld + 64) * 2);
    if (kc) __syncthreads();
    load_rows(make_rsrc(base + H + (long long)kc * CH * ld, bytes), (uint32_t)ld, rows, Ks, wave, 4, lane);
    load_rows(make_rsrc(base + 2 * H + (long long)kc * CH * ld, bytes), (uint32_t)ld, rows, Vs, wave, 4, lane);
    wait_vm0();
    __syncthreads();
    if (!active) continue;
#pragma unroll
    for (int kb = 0; kb < CH / 32; ++kb)
      if (kb < nkb) {
        f32x16 a = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 d = a;
        const int krow = kb * 32 + (lane & 31);
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          a = mfma_32x32x16<E>(frag_rows(Ks, krow, s4, lane), qf[s4], a);
          d = mfma_32x32x16<E>(frag_rows(Vs, krow, s4, lane), of[s4], d);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) d[r] = __expf(a[r] * alpha - L) * (d[r] - D);   // dP -> dS
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 df = pack8<E>(d, 8 * s2);
#pragma unroll
          for (int t = 0; t < 2; ++t) dq[t] = mfma_32x32x16<E>(frag_keys_T(Ks, kb, s2, t, lane), df, dq[t]);
        }
      }
  }
  if (!active) return;
  store_T(dq, dqkv + ((long long)b * S + qb * CH + wave * 32) * ld + h * 64, ld, lane, alpha);
}

// dV = P^T dO and dK = alpha dS^T Q for 128 keys per workgroup (wave w: keys 32 w .., held as B-operand fragments of
// K and V), over all queries in chunks of 128 that pass through LDS as images of Q and dO.  Here the tiles are
// S = Q K^T with the queries along the register axis and the keys along the lanes, so P and dS leave the accumulators
// as the B operands of the products over queries, and a wave needs nobody else's P or dS.
template <typename E, bool RAGGED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void attn_bwd_dkv_long_kernel(const E* qkv, const E* dout, const float* lse, const float* dsum,
                                                                E* dqkv, int S, int H, int A, float alpha) {
  __shared__ __attribute__((aligned(1024))) char lds[2 * CH * 128];
  __shared__ __attribute__((aligned(16))) float Ls[CH], Dsm[CH];
  char* Qs = lds;
  char* Os = lds + CH * 128;
  const int nch = (S + CH - 1) / CH;
  const int kc = blockIdx.x % nch, bh = blockIdx.x / nch, b = bh / A, h = bh % A;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long ld = 3LL * H;
  const E* base = qkv + (long long)b * S * ld + h * 64;
  const E* dob = dout + (long long)b * S * H + h * 64;
  const bool active = !RAGGED || kc * CH + wave * 32 < S;   // (per wave)
  bf16x8 kf[4], vf[4];
  if (active) {
    const E* krow = base + H + (long long)(kc * CH + wave * 32 + (lane & 31)) * ld + (lane >> 5) * 8;
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      kf[st] = *(const bf16x8*)(krow + st * 16);
      vf[st] = *(const bf16x8*)(krow + H + st * 16);
    }
  }
  f32x16 dv[2], dk[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    dv[t] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    dk[t] = dv[t];
  }
  for (int qc = 0; qc < nch; ++qc) {
    const int rows = RAGGED ? min(CH, S - qc * CH) : CH, nqb = rows / 32;   // this chunk's queries
    const uint32_t bytes = (uint32_t)(((long long)(rows - 1) * ld + 64) * 2);
    const uint32_t obytes = (uint32_t)(((long long)(rows - 1) * H + 64) * 2);
    if (qc) __syncthreads();   // every wave has left the previous chunk
    load_rows(make_rsrc(base + (long long)qc * CH * ld, bytes), (uint32_t)ld, rows, Qs, wave, 4, lane);
    load_rows(make_rsrc(dob + (long long)qc * CH * H, obytes), (uint32_t)H, rows, Os, wave, 4, lane);
    if (tid < rows) {
      const long long srow = (long long)bh * S + qc * CH + tid;
      Ls[tid] = lse[srow];
      Dsm[tid] = dsum[srow];
    }
    wait_vm0();
    __syncthreads();
    if (!active) continue;
#pragma unroll
    for (int qb = 0; qb < CH / 32; ++qb) {
      if (qb >= nqb) break;
      f32x16 a = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      f32x16 d = a;
      const int qrow = qb * 32 + (lane & 31);
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        a = mfma_32x32x16<E>(frag_rows(Qs, qrow, s4, lane), kf[s4], a);
        d = mfma_32x32x16<E>(frag_rows(Os, qrow, s4, lane), vf[s4], d);
      }
      // register r of this lane belongs to query 32 qb + 8 (r / 4) + 4 (lane / 32) + r % 4
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        const f32x4 L4 = *(const f32x4*)(Ls + qb * 32 + 8 * blk + 4 * (lane >> 5));
        const f32x4 D4 = *(const f32x4*)(Dsm + qb * 32 + 8 * blk + 4 * (lane >> 5));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float p = __expf(a[4 * blk + i] * alpha - L4[i]);
          a[4 * blk + i] = p;
          d[4 * blk + i] = p * (d[4 * blk + i] - D4[i]);
        }
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8 pf = pack8<E>(a, 8 * s2), df = pack8<E>(d, 8 * s2);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          dv[t] = mfma_32x32x16<E>(frag_keys_T(Os, qb, s2, t, lane), pf, dv[t]);
          dk[t] = mfma_32x32x16<E>(frag_keys_T(Qs, qb, s2, t, lane), df, dk[t]);
        }
      }
    }
  }
  if (!active) return;
  E* out = dqkv + ((long long)b * S + kc * CH + wave * 32) * ld + h * 64;
  store_T(dv, out + 2 * H, ld, lane, 1.0f);
  store_T(dk, out + H, ld, lane, alpha);
}

}  // namespace attn
