// GEMM kernels of the L2L layer: a plain strided kernel (any dtype, any shape; the fp32 path and
// the fallback) and the bf16 MFMA kernel (LDS-staged 32x32x16 tiles, fp32 accumulate) with fused
// bias / GELU / GELU-gradient / residual / accumulate epilogues.
#pragma once
#include "common.h"

// ------------------------------------------------------------------------------------------------
// Epilogue shared by both kernels.  v = alpha * acc already applied by the caller.
template <typename T, typename TC>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, TC* C, long long m, long long n, float v) {
  if (g.epi & EPI_BIAS) v += to_f32(((const T*)g.bias)[n]);
  if (g.epi & EPI_GELU) {
    if (g.aux_out) ((T*)g.aux_out)[m * g.ldaux + n] = from_f32<T>(v);
    v = gelu_f(v);
  }
  if (g.epi & EPI_GELUGRAD) v *= gelu_grad_f(to_f32(((const T*)g.aux)[m * g.ldaux + n]));
  if (g.epi & EPI_RESID) v += to_f32(((const T*)g.resid)[m * g.ldr + n]);
  TC* c = C + m * g.ldc + n;
  if (g.epi & EPI_ACCUM) v += to_f32(*c);
  *c = from_f32<TC>(v);
}

// ------------------------------------------------------------------------------------------------
// Plain kernel: 64x64 tile, 256 threads, 4x4 outputs per thread, fp32 FMA.
template <typename T, typename TC>
__global__ __launch_bounds__(256) void gemm_plain_kernel(GemmArgs g) {
  constexpr int TS = 64, KS = 16;
  __shared__ float As[KS][TS + 1];
  __shared__ float Bs[KS][TS + 1];
  const int z = blockIdx.z, zo = z / g.zdiv, zi = z % g.zdiv;
  const T* A = (const T*)g.A + zo * g.a_zo + zi * g.a_zi;
  const T* B = (const T*)g.B + zo * g.b_zo + zi * g.b_zi;
  TC* C = (TC*)g.C + zo * g.c_zo + zi * g.c_zi;
  int M = g.M, K = g.K;
  if (g.m_dev) M = min(M, *g.m_dev);
  if (g.k_dev) K = min(K, *g.k_dev);
  const int N = g.N;
  const int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
  if (m0 >= M) return;
  const long long sam = g.a_kc ? g.lda : 1, sak = g.a_kc ? 1 : g.lda;
  const long long sbk = g.b_kc ? 1 : g.ldb, sbn = g.b_kc ? g.ldb : 1;
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += KS) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;
      int mm, kk;
      if (g.a_kc) { kk = e % KS; mm = e / KS; } else { mm = e % TS; kk = e / TS; }
      float v = 0.f;
      if (m0 + mm < M && k0 + kk < K) v = to_f32(A[(long long)(m0 + mm) * sam + (long long)(k0 + kk) * sak]);
      As[kk][mm] = v;
      int nn;
      if (g.b_kc) { kk = e % KS; nn = e / KS; } else { nn = e % TS; kk = e / TS; }
      v = 0.f;
      if (n0 + nn < N && k0 + kk < K) v = to_f32(B[(long long)(k0 + kk) * sbk + (long long)(n0 + nn) * sbn]);
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) gemm_epilogue<T, TC>(g, C, m, n, g.alpha * acc[i][j]);
    }
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel.
//
// Block tile BM x BN, K step BK, waves arranged (BM/WM) x (BN/WN), each wave owning WM x WN outputs
// as (WM/32) x (WN/32) accumulators of v_mfma_f32_32x32x16_bf16.  An operand whose K index is
// contiguous in memory is kept in LDS as [row][BK+8] bf16 and read back as one 16-byte fragment
// (8 consecutive k).  An operand whose K index is the strided one ([K,M] or [K,N] in memory) is
// loaded as two 16-byte row chunks for k and k+1, interleaved into (k,k+1) pairs per column and
// kept as [BK/2][cols+8] dwords; a fragment is then four dword reads.  Both give the same k order,
// so every combination of layouts feeds the same MFMA -- no transposed copies of weights or
// activations exist in memory.  LDS is double buffered; the next tile's global loads are issued
// before the current tile's MFMAs.
//
// Bounds: a 16-byte chunk is loaded iff its first element is inside the operand's extent, so row
// pitches must cover the extent rounded up to 8 elements and ragged K needs zero padding in the
// K-contiguous operand.  Stores are masked exactly.
template <int ROWS, int BK, bool KC>
struct TileLds {
  // bytes of one stage
  static constexpr int PITCH = KC ? (BK + 8) : (ROWS + 8);            // bf16 elems (KC) or dwords (!KC)
  static constexpr int BYTES = KC ? ROWS * PITCH * 2 : (BK / 2) * PITCH * 4;
};

template <int ROWS, int BK, bool KC, int NT>
struct TileLoader {
  static constexpr int UNITS = KC ? ROWS * (BK / 8) : (BK / 2) * (ROWS / 8);
  static constexpr int PER = (UNITS + NT - 1) / NT;
  static constexpr int REGS = KC ? PER : 2 * PER;
  u32x4 r[REGS];

  // base: operand pointer already offset to (row0, k = 0); ld: row stride; rows_left: extent - row0
  __device__ __forceinline__ void load(const bf16* base, long long ld, int rows_left, int k0, int K, int tid) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int u = tid + i * NT;
      if (KC) {
        const int row = u / (BK / 8), kc = u % (BK / 8);
        const int k = k0 + kc * 8;
        u32x4 v = {0, 0, 0, 0};
        if ((UNITS % NT == 0 || u < UNITS) && row < rows_left && k < K)
          v = *(const u32x4*)(base + (long long)row * ld + k);
        r[i] = v;
      } else {
        const int kp = u / (ROWS / 8), cc = u % (ROWS / 8);
        const int k = k0 + 2 * kp, col = cc * 8;
        u32x4 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
        if ((UNITS % NT == 0 || u < UNITS) && col < rows_left) {
          if (k < K) lo = *(const u32x4*)(base + (long long)k * ld + col);
          if (k + 1 < K) hi = *(const u32x4*)(base + (long long)(k + 1) * ld + col);
        }
        r[2 * i] = lo;
        r[2 * i + 1] = hi;
      }
    }
  }

  __device__ __forceinline__ void store(char* lds, int tid) const {
    constexpr int PITCH = TileLds<ROWS, BK, KC>::PITCH;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int u = tid + i * NT;
      if (UNITS % NT != 0 && u >= UNITS) continue;
      if (KC) {
        const int row = u / (BK / 8), kc = u % (BK / 8);
        *(u32x4*)(lds + (row * PITCH + kc * 8) * 2) = r[i];
      } else {
        const int kp = u / (ROWS / 8), cc = u % (ROWS / 8);
        const u32x4 lo = r[2 * i], hi = r[2 * i + 1];
        u32x4 p0, p1;  // dword j = (k element j, k+1 element j)
        p0.x = __builtin_amdgcn_perm(hi.x, lo.x, 0x05040100u);
        p0.y = __builtin_amdgcn_perm(hi.x, lo.x, 0x07060302u);
        p0.z = __builtin_amdgcn_perm(hi.y, lo.y, 0x05040100u);
        p0.w = __builtin_amdgcn_perm(hi.y, lo.y, 0x07060302u);
        p1.x = __builtin_amdgcn_perm(hi.z, lo.z, 0x05040100u);
        p1.y = __builtin_amdgcn_perm(hi.z, lo.z, 0x07060302u);
        p1.z = __builtin_amdgcn_perm(hi.w, lo.w, 0x05040100u);
        p1.w = __builtin_amdgcn_perm(hi.w, lo.w, 0x07060302u);
        char* p = lds + (kp * PITCH + cc * 8) * 4;
        *(u32x4*)p = p0;
        *(u32x4*)(p + 16) = p1;
      }
    }
  }
};

// Fragment (8 k-values for one row/column) of k16-step kk out of a staged tile.
template <int ROWS, int BK, bool KC>
__device__ __forceinline__ bf16x8 read_frag(const char* lds, int row, int kk, int lane) {
  constexpr int PITCH = TileLds<ROWS, BK, KC>::PITCH;
  const int g = lane >> 5;
  if (KC) {
    return *(const bf16x8*)(lds + (row * PITCH + kk * 16 + g * 8) * 2);
  } else {
    const uint32_t* p = (const uint32_t*)lds + (kk * 8 + g * 4) * PITCH + row;
    u32x4 v;
    v.x = p[0];
    v.y = p[PITCH];
    v.z = p[2 * PITCH];
    v.w = p[3 * PITCH];
    return __builtin_bit_cast(bf16x8, v);
  }
}

template <int BM, int BN, int BK, int WM, int WN, bool AKC, bool BKC, typename TC>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_mfma_kernel(GemmArgs g) {
  constexpr int NWM = BM / WM, NWN = BN / WN, NT = NWM * NWN * 64;
  constexpr int FM = WM / 32, FN = WN / 32;
  using LA = TileLds<BM, BK, AKC>;
  using LB = TileLds<BN, BK, BKC>;
  constexpr int STAGE = LA::BYTES + LB::BYTES;
  __shared__ __attribute__((aligned(16))) char lds[2 * STAGE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / NWN, wn = wave % NWN;

  int M = g.M, K = g.K;
  if (g.m_dev) M = min(M, *g.m_dev);
  if (g.k_dev) K = min(K, *g.k_dev);
  const int N = g.N;

  // tile mapping: consecutive workgroups go to different XCDs, so give each XCD (id % 8) a
  // contiguous range of tiles, N fastest, so that one XCD's L2 sees the same A panel repeatedly.
  const int tiles_n = (N + BN - 1) / BN, tiles_m = (g.M + BM - 1) / BM;
  const int total = tiles_m * tiles_n;
  int id = blockIdx.x;
  {
    const int per = total / 8, rem_start = per * 8;
    if (id < rem_start) id = (id % 8) * per + id / 8;
  }
  const int tm = id / tiles_n, tn = id % tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;
  if (m0 >= M) return;

  const int z = blockIdx.z, zo = z / g.zdiv, zi = z % g.zdiv;
  const bf16* A = (const bf16*)g.A + zo * g.a_zo + zi * g.a_zi + (AKC ? (long long)m0 * g.lda : (long long)m0);
  const bf16* B = (const bf16*)g.B + zo * g.b_zo + zi * g.b_zi + (BKC ? (long long)n0 * g.ldb : (long long)n0);
  TC* C = (TC*)g.C + zo * g.c_zo + zi * g.c_zi;

  TileLoader<BM, BK, AKC, NT> la;
  TileLoader<BN, BK, BKC, NT> lb;
  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (K + BK - 1) / BK;
  la.load(A, g.lda, M - m0, 0, K, tid);
  lb.load(B, g.ldb, N - n0, 0, K, tid);
  la.store(lds, tid);
  lb.store(lds + LA::BYTES, tid);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const char* cur = lds + (kt & 1) * STAGE;
    char* nxt = lds + ((kt + 1) & 1) * STAGE;
    const bool more = kt + 1 < nk;
    if (more) {
      la.load(A, g.lda, M - m0, (kt + 1) * BK, K, tid);
      lb.load(B, g.ldb, N - n0, (kt + 1) * BK, K, tid);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[FM], bfr[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) af[i] = read_frag<BM, BK, AKC>(cur, wm * WM + i * 32 + (lane & 31), kk, lane);
#pragma unroll
      for (int j = 0; j < FN; ++j)
        bfr[j] = read_frag<BN, BK, BKC>(cur + LA::BYTES, wn * WN + j * 32 + (lane & 31), kk, lane);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      la.store(nxt, tid);
      lb.store(nxt + LA::BYTES, tid);
    }
    __syncthreads();
  }

  // accumulator layout of the 32x32 MFMA: lane -> column (lane % 32); register r -> row
  // 8*(r/4) + 4*(lane/32) + r%4.
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int n = n0 + wn * WN + j * 32 + (lane & 31);
      if (n >= N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < M) gemm_epilogue<bf16, TC>(g, C, m, n, g.alpha * acc[i][j][r]);
      }
    }
}
