// GEMM kernels of the L2L layer: a plain strided kernel (any dtype, any shape; the fp32 path and
// the fallback) and the bf16 MFMA kernel (LDS-staged 32x32x16 tiles, fp32 accumulate) with fused
// bias / GELU / GELU-gradient / residual / accumulate epilogues.
#pragma once
#include "common.h"
#include <type_traits>

// compile-time loop: f(integral_constant<int, I>) for I in [0, N) -- keeps register arrays indexed by constants
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// ------------------------------------------------------------------------------------------------
// Epilogue shared by both kernels.  v = alpha * acc already applied by the caller.
template <typename T, typename TC>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, TC* C, long long m, long long n, float v) {
  if (g.epi & EPI_BIAS) v += to_f32(((const T*)g.bias)[n]);
  if (g.epi & EPI_GELU) {
    if (g.aux_out) ((T*)g.aux_out)[m * g.ldaux + n] = from_f32<T>((g.epi & EPI_KEEPGRAD) ? gelu_grad_f(v) : v);
    v = gelu_f(v);
  }
  if (g.epi & EPI_GELUGRAD) v *= gelu_grad_f(to_f32(((const T*)g.aux)[m * g.ldaux + n]));
  if (g.epi & EPI_MULAUX) v *= to_f32(((const T*)g.aux)[m * g.ldaux + n]);
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
// loaded as 8 x 8 blocks (eight 16-byte row chunks per thread), transposed in registers and stored
// in that same LDS image, so every combination of layouts feeds the same MFMA from 16-byte LDS
// reads (the only LDS read width that reaches 256 B/clk on this chip) -- no transposed copies of
// weights or activations exist in memory.  LDS is double buffered; the next tile's global loads are issued
// before the current tile's MFMAs.
//
// Global loads are buffer loads: the descriptor's byte range ends where the operand's valid rows end,
// so rows past M / N / K come back as zeros from the hardware without a branch; a 16-byte chunk of a
// K-contiguous operand whose first element is past K is sent out of range explicitly.  Row pitches
// must therefore cover the extent rounded up to 8 elements, and ragged K needs zero padding in the
// K-contiguous operand.  Columns past M / N only feed outputs that are never stored.
//
// Epilogue: each wave parks one 32-row strip of its accumulators in LDS (fp32), reads it back row
// major and applies bias / GELU / residual on 8 consecutive columns at a time with 16-byte global
// accesses; a scalar path covers unaligned outputs.  Stores are masked exactly.
// Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (id % 8), each with its own 4 MB
// L2, so an XCD is given a contiguous range of the tile order; the order itself walks strips of up to 8
// tile rows, M fastest, so that the ~32 tiles an XCD works on at a time are a near-square patch: few
// A panels and few B panels, each shared by many resident tiles.
__device__ __forceinline__ void tile_of_block(int id, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int total = tiles_m * tiles_n;
  const int per = total / 8;
  if (id < per * 8) id = (id % 8) * per + id / 8;
  const int GM = min(8, tiles_m);
  const int group = GM * tiles_n, grp = id / group, first = grp * GM;
  const int gm = min(GM, tiles_m - first), in = id - grp * group;
  tm = first + in % gm;
  tn = in / gm;
}

typedef __attribute__((ext_vector_type(4))) int i32x4;
constexpr uint32_t BUF_OOB = 0x80000000u;  // beyond any descriptor range used here (operands are < 2 GiB)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
}

// LDS image of one operand tile, the same for both memory layouts: [row][BK + 8] bf16 (row = output
// row for A, output column for B), so a fragment is always one 16-byte read.
template <int ROWS, int BK>
struct TileLds {
  static constexpr int PITCH = BK + 8;              // bf16 elements; 16 bytes of padding per row
  static constexpr int BYTES = ROWS * PITCH * 2;    // one stage
};

// Byte range of an operand tile seen from its first element: rows_left rows (KC) or K rows (!KC).
template <bool KC>
__device__ __forceinline__ uint32_t tile_bytes(long long ld, int rows_left, int K) {
  const long long k8 = (K + 7) & ~7, r8 = (rows_left + 7) & ~7;
  const long long e = KC ? (long long)(rows_left - 1) * ld + k8 : (long long)(K - 1) * ld + r8;
  return (uint32_t)(e * 2);
}

// Global -> registers -> LDS for one operand tile.
//  KC  (memory [rows, K]):   a unit is one 16-byte chunk (8 k of one row), copied as is.
//  !KC (memory [K, rows]):   a unit is an 8(k) x 8(rows) block: eight 16-byte loads (one per k), transposed
//                            in registers with byte permutes, stored as eight 16-byte chunks (one per row).
//                            Lanes of a wave take 8 row-blocks x 8 k-blocks, so that each load instruction
//                            reads 128-byte row segments and each store instruction covers all LDS banks.
template <int ROWS, int BK, bool KC, int NT>
struct TileLoader {
  static constexpr int PITCH = TileLds<ROWS, BK>::PITCH;
  static constexpr int UNITS = KC ? ROWS * (BK / 8) : (ROWS / 8) * (BK / 8);
  static constexpr int PER = (UNITS + NT - 1) / NT;
  static constexpr int REGS = KC ? PER : 8 * PER;
  static_assert(KC || (BK / 8 == 8 && (ROWS / 8) % 8 == 0), "transposing loader wants BK = 64 and rows in blocks of 64");
  u32x4 r[REGS];

  // unit -> (row block, k block) for the transposing loader
  static __device__ __forceinline__ void unit_pos(int u, int& rb, int& kb) {
    const int w = u >> 6, l = u & 63;          // 64 units per wave: 8 row blocks x 8 k blocks
    rb = w * 8 + (l >> 3);   // 16 consecutive lanes = 2 row blocks x 8 k blocks: their 16-byte stores hit all banks
    kb = l & 7;
  }

  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rs, uint32_t ld, int k0, int K, int tid) {
    static_for<0, PER>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      const int u = tid + i * NT;
      const bool live = UNITS % NT == 0 || u < UNITS;
      if constexpr (KC) {
        const int row = u / (BK / 8), kc = u % (BK / 8);
        const int k = k0 + kc * 8;
        uint32_t off = ((uint32_t)row * ld + (uint32_t)k) * 2u;
        if (k >= K || !live) off = BUF_OOB;
        r[i] = buf_load16(rs, off);
      } else {
        int rb, kb;
        unit_pos(u, rb, kb);
        // rows k >= K fall past the descriptor's range and read as zero
        uint32_t off = ((uint32_t)(k0 + kb * 8) * ld + (uint32_t)(rb * 8)) * 2u;
        static_for<0, 8>([&](auto kc) {
          constexpr int kq = decltype(kc)::value;
          r[8 * i + kq] = buf_load16(rs, live ? off + (uint32_t)kq * ld * 2u : BUF_OOB);
        });
      }
    });
  }

  __device__ __forceinline__ void store(char* lds, int tid) const {
    static_for<0, PER>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      const int u = tid + i * NT;
      if (UNITS % NT == 0 || u < UNITS) {
        if constexpr (KC) {
          const int row = u / (BK / 8), kc = u % (BK / 8);
          *(u32x4*)(lds + (row * PITCH + kc * 8) * 2) = r[i];
        } else {
          int rb, kb;
          unit_pos(u, rb, kb);
          char* p = lds + ((rb * 8) * PITCH + kb * 8) * 2;
          // out row j, dword d = (k = 2d, k = 2d + 1) of input column j: halves of dword j/2 of r[2d], r[2d+1]
          static_for<0, 8>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            constexpr uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
            u32x4 o;
            o.x = __builtin_amdgcn_perm(r[8 * i + 1][j >> 1], r[8 * i + 0][j >> 1], sel);
            o.y = __builtin_amdgcn_perm(r[8 * i + 3][j >> 1], r[8 * i + 2][j >> 1], sel);
            o.z = __builtin_amdgcn_perm(r[8 * i + 5][j >> 1], r[8 * i + 4][j >> 1], sel);
            o.w = __builtin_amdgcn_perm(r[8 * i + 7][j >> 1], r[8 * i + 6][j >> 1], sel);
            *(u32x4*)(p + j * PITCH * 2) = o;
          });
        }
      }
    });
  }
};

// Fragment (8 consecutive k of one row / column) of k16-step kk out of a staged tile.
template <int ROWS, int BK>
__device__ __forceinline__ bf16x8 read_frag(const char* lds, int row, int kk, int lane) {
  return *(const bf16x8*)(lds + (row * TileLds<ROWS, BK>::PITCH + kk * 16 + (lane >> 5) * 8) * 2);
}

// Split-K partial sums go into the (pre-zeroed or already accumulating) fp32 output with hardware atomics.
__device__ __forceinline__ void gemm_epilogue_atomic(const GemmArgs& g, float* C, long long m, long long n, float v) {
  unsafeAtomicAdd(C + m * g.ldc + n, v);
}

// 8 consecutive outputs of one row: v[] = alpha * acc on entry.
template <typename E, typename TC>
__device__ __forceinline__ void epilogue8(const GemmArgs& g, TC* C, long long m, long long n, float v[8], bool atomic) {
  float t[8];
  if (g.epi & EPI_BIAS) {
    load8((const E*)g.bias + n, t);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] += t[i];
  }
  if (g.epi & EPI_GELU) {
    if (g.aux_out && (g.epi & EPI_KEEPGRAD)) {
#pragma unroll
      for (int i = 0; i < 8; ++i) gelu_and_grad_epi<E>(v[i], v[i], t[i]);
      store8((E*)g.aux_out + m * g.ldaux + n, t);
    } else {
      if (g.aux_out) store8((E*)g.aux_out + m * g.ldaux + n, v);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = gelu_epi<E>(v[i]);
    }
  }
  if (g.epi & EPI_GELUGRAD) {
    load8((const E*)g.aux + m * g.ldaux + n, t);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= gelu_grad_epi<E>(t[i]);
  }
  if (g.epi & EPI_MULAUX) {
    load8((const E*)g.aux + m * g.ldaux + n, t);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= t[i];
  }
  if (g.epi & EPI_RESID) {
    load8((const E*)g.resid + m * g.ldr + n, t);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] += t[i];
  }
  TC* c = C + m * g.ldc + n;
  if constexpr (sizeof(TC) == 4) {
    if (atomic) {
#pragma unroll
      for (int i = 0; i < 8; ++i) unsafeAtomicAdd((float*)c + i, v[i]);
      return;
    }
  }
  if (g.epi & EPI_ACCUM) {
    load8(c, t);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] += t[i];
  }
  store8(c, v);
}

template <int BM, int BN, int BK, int WM, int WN, bool AKC, bool BKC, typename TC, typename E = bf16>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_mfma_kernel(GemmArgs g) {
  constexpr int NWM = BM / WM, NWN = BN / WN, NT = NWM * NWN * 64;
  constexpr int FM = WM / 32, FN = WN / 32, KK = BK / 16;
  using LA = TileLds<BM, BK>;
  using LB = TileLds<BN, BK>;
  constexpr int STAGE = LA::BYTES + LB::BYTES;
  constexpr int EP_PITCH = WN + 4;                       // floats
  constexpr int EP_BYTES = 32 * EP_PITCH * 4;            // one wave's strip
  static_assert(NWM * NWN * EP_BYTES <= 2 * STAGE, "epilogue strips must fit the staging buffers");
  extern __shared__ __attribute__((aligned(16))) char lds[];  // 2 * STAGE bytes

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / NWN, wn = wave % NWN;

  int M = g.M, K = g.K;
  if (g.m_dev) M = min(M, *g.m_dev);
  if (g.k_dev) K = min(K, *g.k_dev);
  const int N = g.N;

  const int tiles_n = (N + BN - 1) / BN, tiles_m = (g.M + BM - 1) / BM;
  int tm, tn;
  tile_of_block(blockIdx.x, tiles_m, tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;
  if (m0 >= M) return;

  // split-K: blockIdx.y owns k-tiles [kt0, kt1)
  const int nk_all = (K + BK - 1) / BK;
  const int per_split = (nk_all + gridDim.y - 1) / gridDim.y;
  const int kt0 = blockIdx.y * per_split, kt1 = min(nk_all, kt0 + per_split);
  if (kt0 >= kt1) return;

  const int z = blockIdx.z, zo = z / g.zdiv, zi = z % g.zdiv;
  const bf16* A = (const bf16*)g.A + zo * g.a_zo + zi * g.a_zi + (AKC ? (long long)m0 * g.lda : (long long)m0);
  const bf16* B = (const bf16*)g.B + zo * g.b_zo + zi * g.b_zi + (BKC ? (long long)n0 * g.ldb : (long long)n0);
  TC* C = (TC*)g.C + zo * g.c_zo + zi * g.c_zi;
  const __amdgpu_buffer_rsrc_t ra = make_rsrc(A, tile_bytes<AKC>(g.lda, M - m0, K));
  const __amdgpu_buffer_rsrc_t rb = make_rsrc(B, tile_bytes<BKC>(g.ldb, N - n0, K));
  const uint32_t lda = (uint32_t)g.lda, ldb = (uint32_t)g.ldb;

  TileLoader<BM, BK, AKC, NT> la;
  TileLoader<BN, BK, BKC, NT> lb;
  f32x16 acc[FM * FN];
  static_for<0, FM * FN>([&](auto t) {
    constexpr int T = decltype(t)::value;
    acc[T] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  });

  la.load(ra, lda, kt0 * BK, K, tid);
  lb.load(rb, ldb, kt0 * BK, K, tid);
  la.store(lds, tid);
  lb.store(lds + LA::BYTES, tid);
  __syncthreads();

  const int arow = wm * WM + (lane & 31), brow = wn * WN + (lane & 31);
  for (int kt = kt0; kt < kt1; ++kt) {
    const char* cur = lds + ((kt - kt0) & 1) * STAGE;
    char* nxt = lds + ((kt - kt0 + 1) & 1) * STAGE;
    // next tile into registers while this one is multiplied; unconditional, so that the loop has no
    // branch: past the last tile this fetches rows beyond K (zeros) or the next split's tile, unused.
    // (Keeping two tiles in flight was measured and bought nothing: load latency is not the limiter.)
    la.load(ra, lda, (kt + 1) * BK, K, tid);
    lb.load(rb, ldb, (kt + 1) * BK, K, tid);
    // fragments of step kk+1 are fetched from LDS while the MFMAs of step kk run
    bf16x8 af[2 * FM], bfr[2 * FN];
    static_for<0, FM>([&](auto i) { af[i] = read_frag<BM, BK>(cur, arow + i * 32, 0, lane); });
    static_for<0, FN>([&](auto j) { bfr[j] = read_frag<BN, BK>(cur + LA::BYTES, brow + j * 32, 0, lane); });
    static_for<0, KK>([&](auto kkc) {
      constexpr int kk = decltype(kkc)::value;
      constexpr int cs = (kk & 1), ns = ((kk + 1) & 1);
      if constexpr (kk + 1 < KK) {
        static_for<0, FM>([&](auto i) { af[ns * FM + i] = read_frag<BM, BK>(cur, arow + i * 32, kk + 1, lane); });
        static_for<0, FN>(
            [&](auto j) { bfr[ns * FN + j] = read_frag<BN, BK>(cur + LA::BYTES, brow + j * 32, kk + 1, lane); });
      }
      static_for<0, FM * FN>([&](auto t) {
        constexpr int T = decltype(t)::value;
        constexpr int i = T / FN, j = T % FN;
        acc[T] = mfma_32x32x16<E>(af[cs * FM + i], bfr[cs * FN + j], acc[T]);
      });
      __builtin_amdgcn_sched_barrier(0);  // keep at most two fragment sets live
    });
    la.store(nxt, tid);
    lb.store(nxt + LA::BYTES, tid);
    __syncthreads();
  }

  // ---- epilogue ---------------------------------------------------------------------------------
  // accumulator layout of the 32x32 MFMA: lane -> column (lane % 32); register r -> row
  // 8*(r/4) + 4*(lane/32) + r%4.  One 32 x WN strip at a time goes through this wave's LDS region.
  const bool atomic = gridDim.y > 1;
  float* strip = (float*)(lds + wave * EP_BYTES);
  const auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  const bool vec_ok = (N % 8 == 0) && (g.ldc % 8 == 0) && al16(C) &&
                      (!(g.epi & EPI_BIAS) || al16(g.bias)) &&
                      (!(g.epi & EPI_RESID) || (g.ldr % 8 == 0 && al16(g.resid))) &&
                      (!(g.epi & (EPI_GELUGRAD | EPI_MULAUX)) || (g.ldaux % 8 == 0 && al16(g.aux))) &&
                      (!((g.epi & EPI_GELU) && g.aux_out) || (g.ldaux % 8 == 0 && al16(g.aux_out)));
  static_for<0, FM>([&](auto ic) {
    constexpr int i = decltype(ic)::value;
    __builtin_amdgcn_sched_barrier(0);  // one strip's accumulators at a time leave the accumulation registers
    static_for<0, FN>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      static_for<0, 16>([&](auto rc) {
        constexpr int r = decltype(rc)::value;
        strip[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * EP_PITCH + j * 32 + (lane & 31)] = g.alpha * acc[i * FN + j][r];
      });
    });
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int mrow0 = m0 + wm * WM + i * 32, ncol0 = n0 + wn * WN;
    if (vec_ok && !atomic) {   // atomics go lane-per-column so that one instruction touches two cache lines
#pragma unroll 1
      for (int u = lane; u < 32 * (WN / 8); u += 64) {
        const int row = u / (WN / 8), c8 = (u % (WN / 8)) * 8;
        const int m = mrow0 + row, n = ncol0 + c8;
        if (m < M && n < N) {
          float v[8];
          load8(strip + row * EP_PITCH + c8, v);
          epilogue8<E, TC>(g, C, m, n, v, atomic);
        }
      }
    } else {
#pragma unroll 1
      for (int u = lane; u < 32 * WN; u += 64) {
        const int row = u / WN, col = u % WN;
        const int m = mrow0 + row, n = ncol0 + col;
        if (m < M && n < N) {
          const float v = strip[row * EP_PITCH + col];
          if constexpr (sizeof(TC) == 4) {
            if (atomic) { gemm_epilogue_atomic(g, (float*)C, m, n, v); continue; }
          }
          gemm_epilogue<E, TC>(g, C, m, n, v);
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  });
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel whose global loads are written straight into LDS.
//
// Same tiling and epilogue as gemm_mfma_kernel, but the tiles never pass through registers: each
// wave issues buffer loads with the LDS modifier, one instruction filling 1 KiB of the stage; no
// staging registers, no LDS store instructions, no byte permutes.  The LDS side of such a load is
// fixed (lane l writes bytes [16 l, 16 l + 16) of the instruction's 1 KiB), so the bank-conflict
// avoiding swizzle is applied on the global side: which 16-byte chunk a lane fetches.
//
//  K-contiguous operand (memory [rows, K]): LDS image [row][64] bf16, 128 bytes per row, no padding;
//    chunk c of row r sits at chunk slot c ^ ((r >> 1) & 7); a fragment is one 16-byte read and the 16
//    rows a quarter-wave reads land on 16 different bank groups.
//  K-strided operand (memory [K, rows]): LDS image [k][rows] as in memory; chunk c of k-row k sits at
//    slot c ^ ((k & 3) << 2), i.e. the 64-byte blocks of a k-row are permuted within groups of four.
//    A fragment (8 consecutive k of one column) is two ds_read_b64_tr_b16: within 16 lanes, lane
//    4 R + Q supplies the address of 4 consecutive columns of k-row R, and lane i receives column i of
//    those 4 k-rows.  A k-row is a multiple of 256 bytes, so unswizzled the 4 k-rows of a read would sit
//    on the same banks; with the swizzle the 32 lanes of a half-wave (4 k-rows x 64 bytes) cover all
//    64 banks once.
template <int ROWS, int NT, bool KC>
struct DirectLoader {
  static constexpr int BK = 64;
  static constexpr int BYTES = ROWS * BK * 2;              // one stage
  static constexpr int NBLK = BYTES / 1024;                // 1 KiB blocks, one load instruction each
  static constexpr int PER = NBLK / (NT / 64);
  static_assert(PER * (NT / 64) == NBLK, "blocks must split evenly over the waves");
  static constexpr int ROWB = ROWS * 2;                    // !KC: bytes per k-row
  static constexpr int CPR = ROWS / 8;                     // !KC: chunks per k-row
  static_assert(KC || (CPR <= 64 && 64 % CPR == 0), "a k-row must fit one load instruction");

  __device__ __forceinline__ static void load(__amdgpu_buffer_rsrc_t rs, uint32_t ld, int k0, int K, char* stage, int wave,
                                              int lane) {
    load_part<0, PER>(rs, ld, k0, K, stage, wave, lane);
  }
  // blocks [I0, I1) of this wave's PER blocks
  template <int I0, int I1>
  __device__ __forceinline__ static void load_part(__amdgpu_buffer_rsrc_t rs, uint32_t ld, int k0, int K, char* stage,
                                                   int wave, int lane) {
    static_for<(I0 < PER ? I0 : PER), (I1 < PER ? I1 : PER)>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      const int blk = i * (NT / 64) + wave;
      uint32_t off;
      if constexpr (KC) {
        const int row = blk * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        const int k = k0 + c * 8;
        off = ((uint32_t)row * ld + (uint32_t)k) * 2u;
        if (k >= K) off = BUF_OOB;
      } else {
        const int k = blk * (64 / CPR) + lane / CPR;        // k-row inside the tile
        const int c = (lane % CPR) ^ ((k & 3) << 2);
        off = ((uint32_t)(k0 + k) * ld + (uint32_t)(c * 8)) * 2u;   // k0 + k >= K is past the descriptor: zeros
      }
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)(stage + blk * 1024), 16, (int)off,
                                               0, 0, 0);
    });
  }
};

// Per-lane part of a fragment's LDS address; the k16-step and the 32-row fragment index add constants.
template <int ROWS, bool KC>
struct FragAddr {
  int base[4];   // KC: [0] only.  !KC: one per 32-column fragment of the wave's tile
  int koff[4];   // KC: chunk offset of each k16-step (swizzled)
  __device__ __forceinline__ void init(int row0, int lane) {   // row0: first row / column of this wave's tile
    if constexpr (KC) {
      const int r = lane & 31, gsel = lane >> 5, sw = (r >> 1) & 7;
      base[0] = (row0 + r) * 128;
      base[1] = base[2] = base[3] = 0;
      static_for<0, 4>([&](auto kc) { koff[kc] = (((decltype(kc)::value * 2) | gsel) ^ sw) * 16; });
    } else {
      const int i16 = lane & 15, q16 = lane >> 4;
      const int R = i16 >> 2, Q = i16 & 3, colhalf = q16 & 1, gsel = q16 >> 1;
      // fragment f starts at 64-byte block (row0 / 32 + f) of the k-row; the swizzle XORs the block index with R
      const int common = (gsel * 8 + R) * (ROWS * 2) + colhalf * 32 + Q * 8;
      static_for<0, 4>([&](auto f) { base[f] = common + (((row0 / 32 + decltype(f)::value) ^ R) * 64); });
      static_for<0, 4>([&](auto kc) { koff[kc] = decltype(kc)::value * 16 * (ROWS * 2); });
    }
  }
  // fragment f (32 rows / columns each) of k16-step kk
  template <int F, int KKI>
  __device__ __forceinline__ bf16x8 read(const char* tile) const {
    if constexpr (KC) {
      return *(const bf16x8*)(tile + base[0] + F * 4096 + koff[KKI]);
    } else {
      typedef __attribute__((ext_vector_type(4))) short s16x4;
      typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
      static_assert(F < 4, "a wave's tile holds at most four fragments per operand");
      const char* p = tile + base[F] + koff[KKI];
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(__attribute__((address_space(3))) char*)p);
      const s16x4 hi =
          __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(__attribute__((address_space(3))) char*)(p + 4 * (ROWS * 2)));
      typedef __attribute__((ext_vector_type(8))) short s16x8;
      const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, v);
    }
  }
};

// wait until this wave's LDS-directed loads have landed (vmcnt(0); other counters untouched)
__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }
// ... and until every LDS read this wave issued has returned (vmcnt(0) lgkmcnt(0))
__device__ __forceinline__ void wait_vm0_lds0() { __builtin_amdgcn_s_waitcnt(0x0070); }

// dynamic LDS of gemm_mfma_dlds_kernel: two stages; the epilogue's strips (one of 32 x (WN + 4) floats per wave) sit
// behind the first stage, which by then is receiving the next tile
template <int BM, int BN, int WM, int WN>
constexpr int dlds_lds_bytes() {
  constexpr int stage = (BM + BN) * 128, strips = (BM / WM) * (BN / WN) * 32 * (WN + 4) * 4;
  return stage + (stage > strips ? stage : strips);
}

// EPI >= 0: the epilogue flags are this compile-time constant (the launcher guarantees g.epi == EPI), which takes
// the flag tests and the code of the unused operations out of the unrolled epilogue; EPI < 0: flags read from g.epi.
template <int BM, int BN, int WM, int WN, bool AKC, bool BKC, typename TC, typename E = bf16, int EPI = -1>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_mfma_dlds_kernel(GemmArgs g) {
  constexpr int BK = 64;
  const int epi = EPI >= 0 ? EPI : g.epi;
  const float alpha = EPI >= 0 ? 1.0f : g.alpha;   // the launcher sends only alpha = 1 to the kernels with compiled-in flags
  constexpr int NWM = BM / WM, NWN = BN / WN, NT = NWM * NWN * 64;
  constexpr int FM = WM / 32, FN = WN / 32, KK = BK / 16;
  static_assert(WM % 64 == 0 && WN % 64 == 0, "wave tiles start on multiples of 64 rows / columns");
  using DA = DirectLoader<BM, NT, AKC>;
  using DB = DirectLoader<BN, NT, BKC>;
  constexpr int STAGE = DA::BYTES + DB::BYTES;
  constexpr int EP_PITCH = WN + 4;
  constexpr int EP_BYTES = 32 * EP_PITCH * 4;
  extern __shared__ __attribute__((aligned(1024))) char lds[];  // dlds_lds_bytes<BM, BN, WM, WN>()

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / NWN, wn = wave % NWN;

  int M = g.M, K = g.K;
  if (g.m_dev) M = min(M, *g.m_dev);
  if (g.k_dev) K = min(K, *g.k_dev);
  const int N = g.N;

  const int tiles_n = (N + BN - 1) / BN, tiles_m = (g.M + BM - 1) / BM;
  const int nk_all = (K + BK - 1) / BK;
  const int per_split = (nk_all + gridDim.y - 1) / gridDim.y;
  const int kt0 = blockIdx.y * per_split, kt1 = min(nk_all, kt0 + per_split);
  if (kt0 >= kt1) return;

  // A workgroup takes tiles blockIdx.x, blockIdx.x + gridDim.x, ...: launched with one workgroup per tile it runs
  // once, launched with one workgroup per CU it stays resident and walks its share of the tile order, which
  // saves the dispatch of a 512-thread, 128 KB workgroup per tile.
  const int z = blockIdx.z, zo = z / g.zdiv, zi = z % g.zdiv;
  const uint32_t lda = (uint32_t)g.lda, ldb = (uint32_t)g.ldb;
  // buffer descriptors of the operand panels of the tile at (m0, n0)
  const auto panels = [&](int m0, int n0, __amdgpu_buffer_rsrc_t& ra, __amdgpu_buffer_rsrc_t& rb) {
    const bf16* A = (const bf16*)g.A + zo * g.a_zo + zi * g.a_zi + (AKC ? (long long)m0 * g.lda : (long long)m0);
    const bf16* B = (const bf16*)g.B + zo * g.b_zo + zi * g.b_zi + (BKC ? (long long)n0 * g.ldb : (long long)n0);
    ra = make_rsrc(A, tile_bytes<AKC>(g.lda, M - m0, K));
    rb = make_rsrc(B, tile_bytes<BKC>(g.ldb, N - n0, K));
  };
  int staged_vb = -1;   // the tile whose first k-tile is already on its way into stage 0 (issued under the previous epilogue)
  for (int vb = blockIdx.x; vb < tiles_m * tiles_n; vb += gridDim.x) {
  int tm, tn;
  tile_of_block(vb, tiles_m, tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;
  if (m0 >= M) continue;

  TC* C = (TC*)g.C + zo * g.c_zo + zi * g.c_zi + (long long)blockIdx.y * g.split_stride;
  __amdgpu_buffer_rsrc_t ra, rb;
  panels(m0, n0, ra, rb);

  f32x16 acc[FM * FN];
  static_for<0, FM * FN>([&](auto t) {
    constexpr int T = decltype(t)::value;
    acc[T] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  });

  // A wave's loads of a tile (PER blocks of A, then PER blocks of B) are not issued in one burst: the memory
  // pipeline of a CU takes them at about 30 bytes per clock, a wave that issues into a full queue stands still, MFMAs
  // included, and the other waves then wait for it at the barrier.  The loads of tile t + 2 are spread over the
  // window in which their stage is free: LS0 of them right after the barrier (last k16-step of tile t), then up to
  // LS1, LS2, LS3 in total by the first three k16-steps of tile t + 1; the barrier of tile t + 1 needs them landed.
  constexpr int NLD = DA::PER + DB::PER;
  // Measured (256 x 256 tile, 8 loads per wave): K-contiguous x K-contiguous gains 6-8 % with 2 + 3 + 3 + 0 against all
  // 8 at once (per k-tile: 3250 -> 2700 clocks, of which load issue 920 -> 90 and barrier wait 620 -> 310);
  // K-strided operands, whose fragment reads already load the LDS pipe more, do best with the burst.
  constexpr int SPLIT0 = (AKC && BKC) ? 2 : (AKC || BKC) ? 4 : 8, SPLIT1 = (AKC && BKC) ? 5 : 8, SPLIT2 = 8;   // cumulative eighths
  constexpr int LS0 = (NLD * SPLIT0 + 7) / 8, LS1 = (NLD * SPLIT1 + 7) / 8, LS2 = (NLD * SPLIT2 + 7) / 8;
  const auto load_ab = [&](auto i0c, auto i1c, int kbase, char* stage) {
    constexpr int I0 = decltype(i0c)::value, I1 = decltype(i1c)::value;
    DA::template load_part<I0, I1>(ra, lda, kbase, K, stage, wave, lane);
    DB::template load_part<(I0 > DA::PER ? I0 - DA::PER : 0), (I1 > DA::PER ? I1 - DA::PER : 0)>(rb, ldb, kbase, K, stage + DA::BYTES, wave, lane);
  };
  FragAddr<BM, AKC> fa;
  FragAddr<BN, BKC> fb;
  fa.init(wm * WM, lane);
  fb.init(wn * WN, lane);

  // Two LDS stages.  The loads of tile t + 1 are issued once every wave has read the last fragments
  // of tile t - 1 out of that stage, which is at the barrier before the last k16-step of tile t - 1;
  // that same barrier publishes tile t.  The barrier therefore sits between MFMA groups, and the
  // first fragments of the next tile are read while the last MFMAs of this one run.  Past the last
  // tile the loads fetch rows beyond K (zeros) or the next split's tile, neither of which is used.
  if (staged_vb != vb) {
    DA::load(ra, lda, kt0 * BK, K, lds, wave, lane);
    DB::load(rb, ldb, kt0 * BK, K, lds + DA::BYTES, wave, lane);
  }
  wait_vm0();
  __syncthreads();   // stage 0 is complete, and every wave has left the previous tile's strips, which lie over stage 1
  load_ab(std::integral_constant<int, 0>{}, std::integral_constant<int, LS0>{}, (kt0 + 1) * BK, lds + STAGE);

  bf16x8 af[2 * FM], bfr[2 * FN];
  static_for<0, FM>([&](auto i) { af[i] = fa.template read<decltype(i)::value, 0>(lds); });
  static_for<0, FN>([&](auto j) { bfr[j] = fb.template read<decltype(j)::value, 0>(lds + DA::BYTES); });

  for (int kt = kt0; kt < kt1; ++kt) {
    char* cur = lds + ((kt - kt0) & 1) * STAGE;
    const char* nxt = lds + ((kt - kt0 + 1) & 1) * STAGE;
    static_for<0, KK>([&](auto kkc) {
      constexpr int kk = decltype(kkc)::value;
      constexpr int cs = (kk & 1), ns = ((kk + 1) & 1);
      if constexpr (kk + 1 < KK) {
        // the rest of tile kt + 1's loads (its stage was released at the previous barrier)
        constexpr int P0 = kk == 0 ? LS0 : kk == 1 ? LS1 : LS2, P1 = kk == 0 ? LS1 : kk == 1 ? LS2 : NLD;
        if constexpr (P1 > P0) load_ab(std::integral_constant<int, P0>{}, std::integral_constant<int, P1>{}, (kt + 1) * BK, (char*)nxt);
        static_for<0, FM>([&](auto i) { af[ns * FM + i] = fa.template read<decltype(i)::value, kk + 1>(cur); });
        static_for<0, FN>([&](auto j) { bfr[ns * FN + j] = fb.template read<decltype(j)::value, kk + 1>(cur + DA::BYTES); });
      } else {
        // every fragment of this tile is in registers and this wave's part of the next tile has landed
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        load_ab(std::integral_constant<int, 0>{}, std::integral_constant<int, LS0>{}, (kt + 2) * BK, cur);
        static_for<0, FM>([&](auto i) { af[ns * FM + i] = fa.template read<decltype(i)::value, 0>(nxt); });
        static_for<0, FN>([&](auto j) { bfr[ns * FN + j] = fb.template read<decltype(j)::value, 0>(nxt + DA::BYTES); });
      }
      __builtin_amdgcn_sched_barrier(0);   // fragment reads first: the MFMAs below cover their latency
      static_for<0, FM * FN>([&](auto t) {
        constexpr int T = decltype(t)::value;
        constexpr int i = T / FN, j = T % FN;
        acc[T] = mfma_32x32x16<E>(af[cs * FM + i], bfr[cs * FN + j], acc[T]);
      });
      __builtin_amdgcn_sched_barrier(0);
    });
  }
  // the loads still in flight target the staging buffers the epilogue is about to reuse
  wait_vm0();
  __syncthreads();

  // ---- epilogue (as in gemm_mfma_kernel) ----------------------------------------------------------
  const bool atomic = gridDim.y > 1 && g.split_stride == 0;
  float* strip = (float*)(lds + STAGE + wave * EP_BYTES);   // behind stage 0, which the next tile is about to use
  const bool vec_ok = gemm_vec_ok(g, epi, C);
  // vector path: 8-column chunk and row-in-pass of this lane, its bias values, and the first pass's prefetch
  constexpr int CPR = WN / 8, RPP = 64 / CPR, PASSES = 32 / RPP;
  const int c8 = (lane % CPR) * 8, prow = lane / CPR;
  const int ncol = n0 + wn * WN + c8;
  float bias8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float csum8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // EPI_COLSUM: this lane's share of its 8 columns' sums
  // one 16-byte operand per pass is prefetched: the residual, or the pre-activation of GELU' (no epilogue of the
  // layer uses both; a launch that did would take the residual from memory in the pass itself)
  const bool pre_aux = (epi & (EPI_GELUGRAD | EPI_MULAUX)) != 0, pre_res = !pre_aux && (epi & EPI_RESID);
  // A residual / kept-activation chunk is requested PD - 1 passes before the pass that uses it.  A pass takes a
  // few hundred nanoseconds, a load from memory comes back after about one microsecond: requested one pass ahead
  // every pass waited (measured: 11 us per 256 x 256 tile on top of a store-only epilogue, three passes ahead 6 us;
  // four passes ahead would cost the first spilled registers).
#ifndef L2L_EPI_DEPTH
#define L2L_EPI_DEPTH 4
#endif
  constexpr int PD = L2L_EPI_DEPTH;
  u32x4 pre[PD];
  // row offsets: the lane's own part (row prow of a pass, its 8 columns) once per tile; the pass's first row is the
  // same for the whole wave, so its product with the row stride is scalar work
  const long long pre_ld = pre_aux ? g.ldaux : g.ldr;
  const E* pre_lane = (pre_aux ? (const E*)g.aux : (const E*)g.resid) + (long long)prow * pre_ld + ncol;
  TC* c_lane = C + (long long)prow * g.ldc + ncol;
  const auto fetch = [&](int fi, int fp, u32x4& d) {
    const int mu = m0 + wm * WM + fi * 32 + fp * RPP;   // wave-uniform
    if (mu + prow < M && ncol < N) {
      if (pre_aux || pre_res) d = *(const u32x4*)(pre_lane + (long long)mu * pre_ld);
    }
  };
  if (vec_ok && !atomic) {
    if ((epi & EPI_BIAS) && ncol < N) load8((const E*)g.bias + ncol, bias8);
    static_for<0, PD - 1>([&](auto qc) {
      constexpr int q = decltype(qc)::value;
      if constexpr (q < FM * PASSES) fetch(q / PASSES, q % PASSES, pre[q]);
    });
  }
  // The first k-tile of this workgroup's next tile goes into stage 0 now, under the epilogue (issued after the
  // epilogue's own first loads: loads return in order, and the passes must not wait for 64 KB of operands).
  {
    const int vbn = vb + gridDim.x;
    if (vbn < tiles_m * tiles_n) {
      int tmn, tnn;
      tile_of_block(vbn, tiles_m, tiles_n, tmn, tnn);
      if (tmn * BM < M) {
        __amdgpu_buffer_rsrc_t ran, rbn;
        panels(tmn * BM, tnn * BN, ran, rbn);
        DA::load(ran, lda, kt0 * BK, K, lds, wave, lane);
        DB::load(rbn, ldb, kt0 * BK, K, lds + DA::BYTES, wave, lane);
        staged_vb = vbn;
      }
    }
  }
  static_for<0, FM>([&](auto ic) {
    constexpr int i = decltype(ic)::value;
    __builtin_amdgcn_sched_barrier(0);
    // register rr of a lane: row 8 (rr / 4) + 4 (lane / 32) + rr % 4, column lane % 32.  One base address per group
    // of four registers keeps the offsets of its stores within the range of the two-address LDS store.
    static_for<0, 4>([&](auto gc) {
      constexpr int g4 = decltype(gc)::value;
      int so = (8 * g4 + 4 * (lane >> 5)) * EP_PITCH + (lane & 31);
      asm volatile("" : "+v"(so));   // opaque, or the four bases are folded back into one with large offsets
      static_for<0, FN>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        static_for<0, 4>([&](auto rc) {
          constexpr int r4 = decltype(rc)::value;
          strip[so + r4 * EP_PITCH + j * 32] = alpha * acc[i * FN + j][4 * g4 + r4];
        });
      });
    });
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int mrow0 = m0 + wm * WM + i * 32, ncol0 = n0 + wn * WN;
    if (vec_ok && !atomic) {
      // a lane keeps its 8 columns through the tile: bias8 was loaded once, and the residual / kept-activation
      // values of a pass were requested PD - 1 passes earlier (pre[])
      static_for<0, PASSES>([&](auto pc) {
        constexpr int p = decltype(pc)::value, idx = i * PASSES + p;
        if constexpr (idx + PD - 1 < FM * PASSES) fetch((idx + PD - 1) / PASSES, (idx + PD - 1) % PASSES, pre[(idx + PD - 1) % PD]);
        const int row = p * RPP + prow;
        const int m = mrow0 + row;
        if (m < M && ncol < N) {
          float v[8], tt[8];
          load8(strip + row * EP_PITCH + c8, v);
          if (epi & EPI_BIAS) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += bias8[e];
          }
          if (epi & EPI_GELU) {
            if ((epi & EPI_KEEPGRAD) && g.aux_out) {
#pragma unroll
              for (int e = 0; e < 8; ++e) gelu_and_grad_epi<E>(v[e], v[e], tt[e]);
              store8((E*)g.aux_out + (long long)m * g.ldaux + ncol, tt);
            } else {
              if (g.aux_out) store8((E*)g.aux_out + (long long)m * g.ldaux + ncol, v);
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] = gelu_epi<E>(v[e]);
            }
          }
          if (pre_aux) {
            unpack8<E>(pre[idx % PD], tt);
            if (epi & EPI_MULAUX) {
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] *= tt[e];
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_epi<E>(tt[e]);
            }
          }
          if (epi & EPI_RESID) {
            if (pre_res) unpack8<E>(pre[idx % PD], tt);
            else load8((const E*)g.resid + (long long)m * g.ldr + ncol, tt);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += tt[e];
          }
          TC* cp = c_lane + (long long)(mrow0 + p * RPP) * g.ldc;
          if (epi & EPI_ACCUM) {
            load8(cp, tt);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += tt[e];
          }
          store8(cp, v);
          if (epi & EPI_COLSUM) {
#pragma unroll
            for (int e = 0; e < 8; ++e) csum8[e] += v[e];
          }
        }
      });
    } else {
#pragma unroll 1
      for (int u = lane; u < 32 * WN; u += 64) {
        const int row = u / WN, col = u % WN;
        const int m = mrow0 + row, n = ncol0 + col;
        if (m < M && n < N) {
          const float v = strip[row * EP_PITCH + col];
          if constexpr (sizeof(TC) == 4) {
            if (atomic) { gemm_epilogue_atomic(g, (float*)C, m, n, v); continue; }
          }
          gemm_epilogue<E, TC>(g, C, m, n, v);   // (EPI_COLSUM is not served here: the host asks for it only when vec_ok holds)
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  });
  if ((epi & EPI_COLSUM) && vec_ok && !atomic) {
    // lanes l, l + CPR, l + 2 CPR, ... hold the same 8 columns (different rows): fold them; the wave's 8 x CPR sums go
    // to its own row of the partial-sum matrix (atomics on the few lines of one [N] vector would queue up at L2)
#pragma unroll
    for (int o = CPR; o < 64; o <<= 1) {
#pragma unroll
      for (int e = 0; e < 8; ++e) csum8[e] += __shfl_xor(csum8[e], o, WAVE);
    }
    // (a wave whose rows all lie past M has nothing to report, and the partial-sum matrix has no row for it)
    if (lane < CPR && ncol < N && m0 + wm * WM < M) store8(g.colsum + (long long)((m0 + wm * WM) / WM) * N + ncol, csum8);
  }
  }   // (the next tile's first barrier comes before anything is loaded over the strips)
}
