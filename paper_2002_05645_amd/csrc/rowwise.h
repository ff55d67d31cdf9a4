// Memory-bound kernels of the L2L layer: LayerNorm forward/backward, row softmax forward/backward,
// column sums (bias / gain gradients), embedding gather / scatter, cross-entropy.
// One wavefront owns one row; reductions use wavefront shuffles; statistics are fp32.
#pragma once
#include "common.h"
#include "gemm.h"

// Row sources: a plain row, or the embedding sum E[tok] + Ppos[s] formed on the fly.
template <typename T>
struct PlainRow {
  const T* p;
  __device__ __forceinline__ void operator()(int j, float v[8]) const { load8(p + j, v); }
};
template <typename T>
struct EmbedRow {
  const T* e;
  const T* pos;
  __device__ __forceinline__ void operator()(int j, float v[8]) const {
    float a[8], b[8];
    load8(e + j, a);
    load8(pos + j, b);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = a[i] + b[i];
  }
};

// mean and 1/sqrt(biased variance + eps) of one row, two passes (the second re-reads through cache).
template <typename Row>
__device__ __forceinline__ void row_stats(const Row& row, int n, float eps, int lane, float& mean, float& rstd) {
  float s = 0.f;
  for (int j = lane * 8; j < n; j += WAVE * 8) {
    float v[8];
    row(j, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) s += v[i];
  }
  mean = wave_sum(s) / n;
  float q = 0.f;
  for (int j = lane * 8; j < n; j += WAVE * 8) {
    float v[8];
    row(j, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) q += (v[i] - mean) * (v[i] - mean);
  }
  rstd = rsqrtf(wave_sum(q) / n + eps);
}

template <typename T, typename Row>
__device__ __forceinline__ void ln_write(const Row& row, int n, int lane, float mean, float rstd, const T* gamma,
                                         const T* beta, T* y) {
  for (int j = lane * 8; j < n; j += WAVE * 8) {
    float v[8], g[8], b[8];
    row(j, v);
    load8(gamma + j, g);
    load8(beta + j, b);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = g[i] * ((v[i] - mean) * rstd) + b[i];
    store8(y + j, v);
  }
}

// y = LN(x); optionally keeps mean / rstd per row.
template <typename T>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* x, const T* gamma, const T* beta, T* y, float* mean_out,
                                                     float* rstd_out, int rows, int n, float eps) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  PlainRow<T> row{x + (long long)r * n};
  float mean, rstd;
  row_stats(row, n, eps, lane, mean, rstd);
  ln_write<T>(row, n, lane, mean, rstd, gamma, beta, y + (long long)r * n);
  if (lane == 0 && mean_out) { mean_out[r] = mean; rstd_out[r] = rstd; }
}

// x0 = LN_e(E[tok] + Ppos[s]) per token row; keeps mean / rstd for the backward pass.
template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const int32_t* tokens, const T* E, const T* pos, const T* gamma,
                                                        const T* beta, T* y, float* mean_out, float* rstd_out, int rows,
                                                        int S, int n, float eps, int V, int32_t* bad_ids) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  // an id outside the vocabulary is reported through the flag and clamped, never followed out of the table
  int tok = tokens[r];
  if (tok < 0 || tok >= V) {
    if (lane == 0) atomicOr(bad_ids, 1);
    tok = min(max(tok, 0), V - 1);
  }
  EmbedRow<T> row{E + (long long)tok * n, pos + (long long)(r % S) * n};
  float mean, rstd;
  row_stats(row, n, eps, lane, mean, rstd);
  ln_write<T>(row, n, lane, mean, rstd, gamma, beta, y + (long long)r * n);
  if (lane == 0) { mean_out[r] = mean; rstd_out[r] = rstd; }
}

// dr = rstd * (g - mean(g) - xhat * mean(g * xhat)), g = dy * gamma.
template <typename T, typename Row, typename Sink>
__device__ __forceinline__ void ln_bwd_row(const Row& row, int n, int lane, float mean, float rstd, const T* gamma,
                                           const T* dy, Sink sink) {
  float c1 = 0.f, c2 = 0.f;
  for (int j = lane * 8; j < n; j += WAVE * 8) {
    float v[8], g[8], d[8];
    row(j, v);
    load8(gamma + j, g);
    load8(dy + j, d);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float gg = d[i] * g[i];
      c1 += gg;
      c2 += gg * ((v[i] - mean) * rstd);
    }
  }
  c1 = wave_sum(c1) / n;
  c2 = wave_sum(c2) / n;
  for (int j = lane * 8; j < n; j += WAVE * 8) {
    float v[8], g[8], d[8];
    row(j, v);
    load8(gamma + j, g);
    load8(dy + j, d);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = rstd * (d[i] * g[i] - c1 - ((v[i] - mean) * rstd) * c2);
    sink(j, v);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void ln_bwd_dx_kernel(const T* dy, const T* x, const float* mean, const float* rstd,
                                                        const T* gamma, T* dx, int rows, int n) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  PlainRow<T> row{x + (long long)r * n};
  T* out = dx + (long long)r * n;
  ln_bwd_row<T>(row, n, lane, mean[r], rstd[r], gamma, dy + (long long)r * n,
             [out](int j, const float v[8]) { store8(out + j, v); });
}

// LayerNorm backward with its three column reductions in the same pass: dx as above, and
//   dgamma[j] += sum_r dy[r,j] xhat[r,j],  dbeta[j] += sum_r dy[r,j],  dbias[j] += sum_r dx[r,j]
// (dbias: the bias of the linear layer whose output, plus a residual, this LayerNorm normalises).  A block
// takes LNF_ROWS rows, a wave one row at a time; a lane owns columns lane * 8 + 512 k, k < NCH, keeps
// the row's values in registers between the two passes and the column sums in registers across rows;
// the four waves' sums are combined in LDS and leave as one fp32 atomic per column and block.
constexpr int LNF_ROWS = 64;   // measured best of 16 .. 128 at 32768 x 1024: fewer rows mean more atomics, more mean fewer waves
// FROMY: `x` holds the LayerNorm's OUTPUT y = gamma xhat + beta instead of its input, `rstd` the statistics kept by the
// forward pass, and xhat is taken back out of y as (y - beta) / gamma; the input itself is then not needed (the
// backward pass of the layer's last LayerNorm, whose output is the stashed boundary activation: the GEMM in front
// of it need not be recomputed).  The caller makes sure that no |gamma| is tiny.
//
// RING > 0 (16-bit rows, every one of the NCH column groups in use): rows come in through LDS.  Each wave owns RING
// slots of [x | dy][NCH KiB] and keeps the loads of its next RING - 1 rows in flight as direct-to-LDS loads, which need
// no registers to land in: with rows requested into registers one ahead, a CU has 32 to 48 KB on their way, half of what
// the memory system needs to stay busy.  The slots sit where the column sums are combined once the rows are done.
// A wave's vector-memory operations complete in the order issued, so "row i is in" is a count of the operations
// issued after its request: the later requests' loads and the stores of dx in between (the row statistics are
// fetched up front for that reason: no other vector-memory operation may sit in the loop).
template <int N>
__device__ __forceinline__ void wait_vm_le() {   // at most N vector-memory operations of this wave outstanding
  static_assert(N >= 0 && N < 64, "vmcnt has six bits");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

template <typename T, int NCH, bool FROMY = false, int RING = 0>
__global__ __launch_bounds__(256) void ln_bwd_fused_kernel(const T* dy, const T* x, const float* mean, const float* rstd,
                                                           const T* gamma, T* dx, float* dgamma, float* dbeta,
                                                           float* dbias, int rows, int n, float eps, const T* beta) {
  // mean == nullptr: the row statistics are computed here, from the row already held in registers (same two
  // passes as the forward kernel), which spares a forward-statistics kernel where nothing else needs its output
  extern __shared__ float lnf_red[];   // [4 waves][3][NCH * 512]
  constexpr int NC = NCH * 512;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float sg[NCH][8], sb[NCH][8], sx[NCH][8], gam[NCH][8];
  float bet[FROMY ? NCH : 1][8], ginv[FROMY ? NCH : 1][8];
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const int j = lane * 8 + k * 512;
#pragma unroll
    for (int i = 0; i < 8; ++i) sg[k][i] = sb[k][i] = sx[k][i] = gam[k][i] = 0.f;
    if (j < n) load8(gamma + j, gam[k]);
    if constexpr (FROMY) {
#pragma unroll
      for (int i = 0; i < 8; ++i) bet[k][i] = 0.f;
      if (j < n) load8(beta + j, bet[k]);
#pragma unroll
      for (int i = 0; i < 8; ++i) ginv[k][i] = 1.0f / gam[k][i];
    }
  }
  const int r0 = blockIdx.x * LNF_ROWS, r1 = min(rows, r0 + LNF_ROWS);
  // 16-bit rows without the ring: the wave's next row is requested (as packed 16-byte words) before the current one is
  // worked on, so that its two reductions and its store run under the loads
  constexpr bool RINGED = RING > 0;
  constexpr bool AHEAD = sizeof(T) == 2 && !RINGED;
  static_assert(!RINGED || sizeof(T) == 2, "the ring takes 16-bit rows");
  u32x4 xr[NCH], dr[NCH];
  const auto request = [&](int r) {
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const int j = lane * 8 + k * 512;
      if (j < n && r < r1) {
        xr[k] = *(const u32x4*)(x + (long long)r * n + j);
        dr[k] = *(const u32x4*)(dy + (long long)r * n + j);
      }
    }
  };
  constexpr int SLOT = 2 * NCH * 1024;   // bytes of one ring slot
  char* ring = (char*)lnf_red + w * (RINGED ? RING : 0) * SLOT;
  const int nblk = r1 - r0;
  __amdgpu_buffer_rsrc_t rx, rd;
  float st_mu = 0.f, st_rs = 0.f;   // lane i: the statistics of this wave's i-th row
  if constexpr (RINGED) {
    rx = make_rsrc(x + (long long)r0 * n, (uint32_t)nblk * (uint32_t)n * 2u);
    rd = make_rsrc(dy + (long long)r0 * n, (uint32_t)nblk * (uint32_t)n * 2u);
    const int rl = r0 + w + 4 * lane;
    if (lane < LNF_ROWS / 4 && rl < r1) {
      if (rstd) st_rs = rstd[rl];
      if (!FROMY && mean) st_mu = mean[rl];
    }
  }
  // the wave's i-th row into slot i % RING; past the block's last row the last row again, so that every request is 2 NCH loads
  const auto request_ring = [&](int i) {
    const uint32_t rr = (uint32_t)min(w + 4 * i, nblk - 1);
    char* dst = ring + (i % (RINGED ? RING : 1)) * SLOT;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const uint32_t off = (rr * (uint32_t)n + (uint32_t)(k * 512 + lane * 8)) * 2u;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void*)(dst + k * 1024), 16, (int)off, 0, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rd, (__attribute__((address_space(3))) void*)(dst + (NCH + k) * 1024), 16, (int)off, 0, 0, 0);
    }
  };
  if constexpr (AHEAD) request(r0 + w);
  if constexpr (RINGED) {
#pragma unroll
    for (int i = 0; i < RING - 1; ++i) request_ring(i);
  }
  int it = 0;
  for (int r = r0 + w; r < r1; r += 4, ++it) {
    float xh[NCH][8], d[NCH][8];
    if constexpr (RINGED) {
      // (the count below takes the previous rows' stores as issued: nothing may be moved across this point)
      asm volatile("" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      request_ring(it + RING - 1);
      // issued since row `it` was asked for: RING - 1 requests, and the stores (NCH each) of the rows worked on since
      if (it < RING - 1) wait_vm_le<(RING - 1) * 2 * NCH>();
      else wait_vm_le<(RING - 1) * 3 * NCH>();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const char* src = ring + (it % (RINGED ? RING : 1)) * SLOT + lane * 16;
#pragma unroll
      for (int k = 0; k < NCH; ++k) {
        xr[k] = *(const u32x4*)(src + k * 1024);
        dr[k] = *(const u32x4*)(src + (NCH + k) * 1024);
      }
    }
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const int j = lane * 8 + k * 512;
      if (j < n) {
        if constexpr (AHEAD || RINGED) {
          unpack8<T>(xr[k], xh[k]);
          unpack8<T>(dr[k], d[k]);
        } else {
          load8(x + (long long)r * n + j, xh[k]);
          load8(dy + (long long)r * n + j, d[k]);
        }
      }
    }
    if constexpr (AHEAD) request(r + 4);
    float mu = 0.f, rs;
    if constexpr (RINGED && FROMY) {
      rs = __shfl(st_rs, it, 64);
    } else if constexpr (FROMY) {
      rs = rstd[r];
    } else if (mean) {
      if constexpr (RINGED) {
        mu = __shfl(st_mu, it, 64);
        rs = __shfl(st_rs, it, 64);
      } else {
        mu = mean[r];
        rs = rstd[r];
      }
    } else {
      float s = 0.f, q = 0.f;
#pragma unroll
      for (int k = 0; k < NCH; ++k)
        if (lane * 8 + k * 512 < n) {
#pragma unroll
          for (int i = 0; i < 8; ++i) s += xh[k][i];
        }
      mu = wave_sum(s) / n;
#pragma unroll
      for (int k = 0; k < NCH; ++k)
        if (lane * 8 + k * 512 < n) {
#pragma unroll
          for (int i = 0; i < 8; ++i) q += (xh[k][i] - mu) * (xh[k][i] - mu);
        }
      rs = rsqrtf(wave_sum(q) / n + eps);
    }
    float c1 = 0.f, c2 = 0.f;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const int j = lane * 8 + k * 512;
      if (j < n) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          if constexpr (FROMY) xh[k][i] = (xh[k][i] - bet[k][i]) * ginv[k][i];
          else xh[k][i] = (xh[k][i] - mu) * rs;
          const float gg = d[k][i] * gam[k][i];
          c1 += gg;
          c2 += gg * xh[k][i];
        }
      }
    }
    c1 = wave_sum(c1) / n;
    c2 = wave_sum(c2) / n;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const int j = lane * 8 + k * 512;
      if (j < n) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          v[i] = rs * (d[k][i] * gam[k][i] - c1 - xh[k][i] * c2);
          sg[k][i] += d[k][i] * xh[k][i];
          sb[k][i] += d[k][i];
          sx[k][i] += v[i];
        }
        store8(dx + (long long)r * n + j, v);
      }
    }
  }
  if constexpr (RINGED) {   // the slots become the place where the column sums meet: every wave is done with its own first
    wait_vm_le<0>();
    __syncthreads();
  }
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    float* p = lnf_red + (w * 3) * NC + k * 512 + lane * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      p[i] = sg[k][i];
      p[NC + i] = sb[k][i];
      p[2 * NC + i] = sx[k][i];
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 3 * NC; idx += 256) {
    const int which = idx / NC, col = idx % NC;
    if (col < n) {
      const float s = lnf_red[idx] + lnf_red[3 * NC + idx] + lnf_red[6 * NC + idx] + lnf_red[9 * NC + idx];
      atomicAdd((which == 0 ? dgamma : which == 1 ? dbeta : dbias) + col, s);
    }
  }
}

// Embedding backward: dr through LN_e, scatter-added (fp32 atomics) into dE[tok] and dPpos[s].
// A block takes one position s of EMB_SEQS consecutive sequences (a wave one row at a time), so that the
// rows' contributions to dPpos[s] meet in LDS first and leave as one global atomic per column and block;
// the token rows are scattered, their atomics go to memory directly.  Dynamic LDS: n floats, 5 n if `turned`.
constexpr int EMB_SEQS = 16;
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_kernel(const int32_t* tokens, const T* E, const T* pos, const T* gamma,
                                                        const T* dy, const float* mean, const float* rstd, float* dE,
                                                        float* dpos, int rows, int S, int n, bool turned, int V) {
  extern __shared__ float pos_acc[];   // n floats, then (turned) one row of n floats per wave
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int s = blockIdx.x % S, grp = blockIdx.x / S;
  const int nseq = rows / S;
  for (int j = threadIdx.x; j < n; j += 256) pos_acc[j] = 0.f;
  __syncthreads();
  const int q1 = min(nseq, (grp + 1) * EMB_SEQS);
  float* tw = pos_acc + (long long)(1 + w) * n;
  for (int q = grp * EMB_SEQS + w; q < q1; q += 4) {
    const int r = q * S + s;
    const long long tok = min(max(tokens[r], 0), V - 1);   // (clamped as in the forward kernel, which reports it)
    EmbedRow<T> row{E + tok * n, pos + (long long)s * n};
    float* de = dE + tok * n;
    if (turned) {
      // a lane computes 8 consecutive columns; the atomics go out with consecutive lanes on consecutive columns
      // (whole cache lines per instruction in memory, no bank conflicts in LDS), so the row turns through LDS first
      ln_bwd_row<T>(row, n, lane, mean[r], rstd[r], gamma, dy + (long long)r * n, [tw](int j, const float v[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) tw[j + i] = v[i];
      });
      __builtin_amdgcn_wave_barrier();
      for (int col = lane; col < n; col += WAVE) {
        const float x = tw[col];
        atomicAdd(de + col, x);
        atomicAdd(pos_acc + col, x);
      }
      __builtin_amdgcn_wave_barrier();
    } else {
      ln_bwd_row<T>(row, n, lane, mean[r], rstd[r], gamma, dy + (long long)r * n, [de](int j, const float v[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          atomicAdd(de + j + i, v[i]);
          atomicAdd(pos_acc + j + i, v[i]);
        }
      });
    }
  }
  __syncthreads();
  float* dp = dpos + (long long)s * n;
  for (int j = threadIdx.x; j < n; j += 256) atomicAdd(dp + j, pos_acc[j]);
}

// ---- column reductions -----------------------------------------------------------------------------
// out_a[j] += sum_t a[t,j] * w(t,j), out_b[j] += sum_t a[t,j], with w = xhat of a LayerNorm input
// (MODE 1: plain rows x; MODE 2: embedding rows) or out_b only (MODE 0: bias gradient).
// Block: 128 columns x rpb rows (rpb = gridDim.y's share of the rows, a multiple of 4); lanes own column pairs; waves
// stride rows, eight loads in flight each; LDS combine; one fp32 atomic per column per block.
constexpr int COLSUM_ROWS = 128;
// rows per block: COLSUM_ROWS, fewer where that would leave most of the chip without a block
inline int colsum_rows_per_block(long long rows, int n) {
  int rpb = COLSUM_ROWS;
  while (rpb > 16 && ((rows + rpb - 1) / rpb) * ((n + 127) / 128) < 1024) rpb /= 2;
  return rpb;
}
template <typename T, int MODE>
__global__ __launch_bounds__(256) void colsum_kernel(const T* a, long long lda, const T* x, const float* mean,
                                                     const float* rstd, const int32_t* tokens, const T* E, const T* pos,
                                                     int S, float* out_a, float* out_b, int rows, int n,
                                                     const int* rows_dev, int V, int rpb) {
  __shared__ float red[4][2][128];
  if (rows_dev) rows = min(rows, *rows_dev);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int j = blockIdx.x * 128 + lane * 2;
  const int r0 = blockIdx.y * rpb;
  if (r0 >= rows) return;
  const int r1 = min(rows, r0 + rpb);
  float sa0 = 0.f, sa1 = 0.f, sb0 = 0.f, sb1 = 0.f;
  if (j < n) {
#pragma unroll 8
    for (int r = r0 + w; r < r1; r += 4) {
      const float d0 = to_f32(a[(long long)r * lda + j]), d1 = to_f32(a[(long long)r * lda + j + 1]);
      sb0 += d0;
      sb1 += d1;
      if (MODE != 0) {
        float x0, x1;
        if (MODE == 1) {
          x0 = to_f32(x[(long long)r * n + j]);
          x1 = to_f32(x[(long long)r * n + j + 1]);
        } else {
          const long long tok = min(max(tokens[r], 0), V - 1);
          const int s = r % S;
          x0 = to_f32(E[tok * n + j]) + to_f32(pos[(long long)s * n + j]);
          x1 = to_f32(E[tok * n + j + 1]) + to_f32(pos[(long long)s * n + j + 1]);
        }
        const float mu = mean[r], rs = rstd[r];
        sa0 += d0 * ((x0 - mu) * rs);
        sa1 += d1 * ((x1 - mu) * rs);
      }
    }
  }
  red[w][0][lane * 2] = sa0; red[w][0][lane * 2 + 1] = sa1;
  red[w][1][lane * 2] = sb0; red[w][1][lane * 2 + 1] = sb1;
  __syncthreads();
  const int t = threadIdx.x;  // 256 threads: 2 outputs x 128 columns
  const int which = t >> 7, c = t & 127;
  const int col = blockIdx.x * 128 + c;
  if (col < n && (MODE != 0 || which == 1)) {
    const float s = red[0][which][c] + red[1][which][c] + red[2][which][c] + red[3][which][c];
    atomicAdd((which == 0 ? out_a : out_b) + col, s);
  }
}

// ---- softmax ---------------------------------------------------------------------------------------
// In place: p[r,:] = softmax(p[r,:]) for rows of length n.
template <typename T>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(T* p, long long rows, int n) {
  const int lane = threadIdx.x & 63;
  const long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  T* row = p + r * n;
  float mx = -INFINITY;
  for (int j = lane; j < n; j += WAVE) mx = fmaxf(mx, to_f32(row[j]));
  mx = wave_max(mx);
  float s = 0.f;
  for (int j = lane; j < n; j += WAVE) s += __expf(to_f32(row[j]) - mx);
  s = 1.0f / wave_sum(s);
  for (int j = lane; j < n; j += WAVE) row[j] = from_f32<T>(__expf(to_f32(row[j]) - mx) * s);
}

// In place on dp: ds = p * (dp - sum_j dp*p).
template <typename T>
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const T* p, T* dp, long long rows, int n) {
  const int lane = threadIdx.x & 63;
  const long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const T* pr = p + r * n;
  T* dr = dp + r * n;
  float s = 0.f;
  for (int j = lane; j < n; j += WAVE) s += to_f32(pr[j]) * to_f32(dr[j]);
  s = wave_sum(s);
  for (int j = lane; j < n; j += WAVE) dr[j] = from_f32<T>(to_f32(pr[j]) * (to_f32(dr[j]) - s));
}

// ---- head: label compaction, row gather / scatter, cross-entropy -----------------------------------
// One block per micro-batch: idx[u*T + i] = position of the i-th labelled token (ascending),
// cnt[u] = how many; total[0] += cnt[u].
__global__ __launch_bounds__(256) void label_compact_kernel(const int32_t* labels, int T, int32_t* idx, int32_t* cnt,
                                                            int32_t* total) {
  __shared__ int part[256];
  const int u = blockIdx.x, t = threadIdx.x;
  const int32_t* lab = labels + (long long)u * T;
  const int per = (T + 255) / 256;
  const int b = t * per, e = min(T, b + per);
  int c = 0;
  for (int i = b; i < e; ++i) c += lab[i] >= 0;
  part[t] = c;
  __syncthreads();
  if (t == 0) {
    int run = 0;
    for (int i = 0; i < 256; ++i) { const int v = part[i]; part[i] = run; run += v; }
    cnt[u] = run;
    atomicAdd(total, run);
  }
  __syncthreads();
  int o = part[t];
  for (int i = b; i < e; ++i)
    if (lab[i] >= 0) idx[(long long)u * T + o++] = i;
}

// Joins the per-micro-batch lists into one list over the whole mini-batch: gidx[prefix(u) + i] =
// u * T + idx[u * T + i], and chunk_cnt[c] = how many entries of that list fall into rows
// [c * chunk, (c + 1) * chunk).  One block per micro-batch.
__global__ __launch_bounds__(256) void label_merge_kernel(const int32_t* idx, const int32_t* cnt, int T, int32_t* gidx,
                                                          int32_t* chunk_cnt, int chunk, int nchunks) {
  const int u = blockIdx.x, t = threadIdx.x;
  int before = 0, total = 0;
  for (int v = 0; v < (int)gridDim.x; ++v) {
    const int n = cnt[v];
    if (v < u) before += n;
    total += n;
  }
  const int mine = cnt[u];
  for (int i = t; i < mine; i += 256) gidx[before + i] = u * T + idx[(long long)u * T + i];
  if (u == 0)
    for (int c = t; c < nchunks; c += 256) chunk_cnt[c] = max(0, min(chunk, total - c * chunk));
}

// dst[i,:] = src[idx[i],:] (gather) or dst[idx[i],:] = src[i,:] (SCATTER) for i < *cnt; wave per row.
template <typename T, bool SCATTER>
__global__ __launch_bounds__(256) void rows_by_index_kernel(const T* src, T* dst, const int32_t* idx, const int32_t* cnt,
                                                            int n) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= *cnt) return;
  const long long a = SCATTER ? i : idx[i], b = SCATTER ? idx[i] : i;
  for (int j = lane * 8; j < n; j += WAVE * 8) {
    float v[8];
    load8(src + a * n + j, v);
    store8(dst + b * n + j, v);
  }
}

// Cross-entropy over one row of logits z[Vp] (first V valid): adds (lse - z[label]) / N to *loss and
// writes dz = scale * (softmax(z) - onehot) / N in T (scale: the loss scale of fp16 training, 1 otherwise),
// zero in the padding columns.  One block per row.
template <typename T>
__global__ __launch_bounds__(256) void ce_kernel(const float* z, long long ldz, const int32_t* labels,
                                                 const int32_t* idx, const int32_t* cnt, const int32_t* total, T* dz,
                                                 float* loss, int V, int Vp, float scale, int32_t* bad_ids) {
  __shared__ float red[4];
  const int i = blockIdx.x;
  if (i >= *cnt) return;
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const float* row = z + (long long)i * ldz;
  float mx = -INFINITY;
  for (int j = t; j < V; j += 256) mx = fmaxf(mx, row[j]);
  mx = wave_max(mx);
  if (lane == 0) red[w] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float s = 0.f;
  for (int j = t; j < V; j += 256) s += __expf(row[j] - mx);
  s = wave_sum(s);
  if (lane == 0) red[w] = s;
  __syncthreads();
  s = red[0] + red[1] + red[2] + red[3];
  const float inv_n = 1.0f / (float)(*total);
  int label = labels[idx[i]];    // >= 0: the row is in the list of labelled rows
  if (label >= V) {
    if (t == 0) atomicOr(bad_ids, 1);
    label = V - 1;
  }
  const float lse = mx + __logf(s);
  if (t == 0) atomicAdd(loss, (lse - row[label]) * inv_n);
  T* d = dz + (long long)i * Vp;
  const float inv_s = 1.0f / s;
  for (int j = t; j < Vp; j += 256) {
    float v = 0.f;
    if (j < V) v = (__expf(row[j] - mx) * inv_s - (j == label ? 1.0f : 0.0f)) * (inv_n * scale);
    d[j] = from_f32<T>(v);
  }
}

// ---- sequence-classification head --------------------------------------------------------------------
// dst[q,:] = src[q * S,:] (first token of sequence q) or, SCATTER, dst[q * S,:] = src[q,:]; wave per sequence.
template <typename T, bool SCATTER>
__global__ __launch_bounds__(256) void first_token_rows_kernel(const T* src, T* dst, int nseq, int S, int n) {
  const int lane = threadIdx.x & 63;
  const int q = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (q >= nseq) return;
  const long long a = SCATTER ? q : (long long)q * S, b = SCATTER ? (long long)q * S : q;
  for (int j = lane * 8; j < n; j += WAVE * 8) {
    float v[8];
    load8(src + a * n + j, v);
    store8(dst + b * n + j, v);
  }
}

// y = tanh(x), or BWD: y = x * (1 - t^2) with t the forward result; n elements, a multiple of 8.
template <typename T, bool BWD>
__global__ __launch_bounds__(256) void tanh_kernel(const T* x, const T* t, T* y, long long n) {
  const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= n) return;
  float v[8], w[8];
  load8(x + i, v);
  if (BWD) {
    load8(t + i, w);
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] *= 1.0f - w[k] * w[k];
  } else {
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = tanhf(v[k]);
  }
  store8(y + i, v);
}

// Cross-entropy over the C class logits of each sequence (z: [nseq, ldz] fp32), one block for the whole
// mini-batch: N = number of sequences with label >= 0; *loss = (1/N) sum (lse - z[label]);
// dz = scale * (softmax(z) - onehot) / N in T, zero for unlabelled sequences and in the padding columns.
template <typename T>
__global__ __launch_bounds__(256) void cls_ce_kernel(const float* z, int ldz, const int32_t* labels, T* dz, float* loss,
                                                     int nseq, int C, float scale, int32_t* bad_ids) {
  __shared__ int cnt[4];
  __shared__ float part[4];
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  int mine = 0;
  for (int q = t; q < nseq; q += 256) mine += labels[q] >= 0;
  mine = (int)wave_sum((float)mine);
  if (lane == 0) cnt[w] = mine;
  __syncthreads();
  const int N = cnt[0] + cnt[1] + cnt[2] + cnt[3];
  const float inv_n = N > 0 ? 1.0f / (float)N : 0.f;
  float l = 0.f;
  for (int q = t; q < nseq; q += 256) {
    const float* row = z + (long long)q * ldz;
    T* d = dz + (long long)q * ldz;
    int label = labels[q];
    if (label >= C) {   // reported and clamped, never followed past the row
      atomicOr(bad_ids, 1);
      label = C - 1;
    }
    if (label < 0) {
      for (int j = 0; j < ldz; ++j) d[j] = from_f32<T>(0.f);
      continue;
    }
    float mx = -INFINITY;
    for (int j = 0; j < C; ++j) mx = fmaxf(mx, row[j]);
    float s = 0.f;
    for (int j = 0; j < C; ++j) s += __expf(row[j] - mx);
    l += (mx + __logf(s) - row[label]) * inv_n;
    const float inv_s = 1.0f / s;
    for (int j = 0; j < ldz; ++j) {
      float v = 0.f;
      if (j < C) v = (__expf(row[j] - mx) * inv_s - (j == label ? 1.0f : 0.0f)) * (inv_n * scale);
      d[j] = from_f32<T>(v);
    }
  }
  l = wave_sum(l);
  if (lane == 0) part[w] = l;
  __syncthreads();
  if (t == 0) *loss = part[0] + part[1] + part[2] + part[3];
}

// out[c, r] = in[r, c] for a bf16 matrix [R, C] (both multiples of 8): 128 x 128 tiles through LDS, so that
// both the reads and the writes are 256-byte row segments moved with 16-byte accesses.  The LDS tile is
// kept as dwords holding (row 2i, row 2i+1) pairs of one column: a 16-byte output chunk (8 consecutive
// rows of one column) is then four dword reads, and the pair packing is done with byte permutes on the way in.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16* in, bf16* out, int R, int C) {
  __shared__ uint32_t tile[64][128 + 1];   // [row pair][column]
  const int r0 = blockIdx.y * 128, c0 = blockIdx.x * 128, t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int u = t + i * 256;            // 64 row pairs x 16 column chunks
    const int rp = u >> 4, cc = (u & 15) * 8;
    u32x4 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
    if (c0 + cc < C) {
      if (r0 + 2 * rp < R) lo = *(const u32x4*)(in + (long long)(r0 + 2 * rp) * C + c0 + cc);
      if (r0 + 2 * rp + 1 < R) hi = *(const u32x4*)(in + (long long)(r0 + 2 * rp + 1) * C + c0 + cc);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      tile[rp][cc + 2 * j] = __builtin_amdgcn_perm(hi[j], lo[j], 0x05040100u);
      tile[rp][cc + 2 * j + 1] = __builtin_amdgcn_perm(hi[j], lo[j], 0x07060302u);
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int u = t + i * 256;            // 128 output rows (columns of in) x 16 chunks of 8 input rows
    const int col = u >> 4, rq = u & 15;
    if (c0 + col < C && r0 + rq * 8 < R) {
      u32x4 v;
      v.x = tile[rq * 4 + 0][col];
      v.y = tile[rq * 4 + 1][col];
      v.z = tile[rq * 4 + 2][col];
      v.w = tile[rq * 4 + 3][col];
      *(u32x4*)(out + (long long)(c0 + col) * R + r0 + rq * 8) = v;
    }
  }
}

// out[i] = in[i] rounded to the 16-bit format E, i < n (in: 16-byte aligned, out: 8-byte aligned)
template <typename E>
__global__ __launch_bounds__(256) void narrow_kernel(const float* in, E* out, long long n) {
  const long long n4 = n / 4, stride = (long long)gridDim.x * 256;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    const f32x4 v = *(const f32x4*)(in + 4 * i);
    typedef __attribute__((ext_vector_type(4))) E e4;
    const e4 o = {from_f32<E>(v.x), from_f32<E>(v.y), from_f32<E>(v.z), from_f32<E>(v.w)};
    *(u32x2*)(out + 4 * i) = __builtin_bit_cast(u32x2, o);
  }
  for (long long i = n4 * 4 + (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) out[i] = from_f32<E>(in[i]);
}

// Sum of the K-split partial results of a GEMM: out[m, n] += sum_s part[s][m, n] (part: `splits` dense [rows, n]
// fp32 matrices, n a multiple of 4; out: row stride ldo, 16-byte aligned rows).
__global__ __launch_bounds__(256) void split_sum_kernel(const float* part, int splits, long long rows, int n, float* out,
                                                        long long ldo) {
  const long long total4 = rows * n / 4, slice = rows * n;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total4; i += (long long)gridDim.x * 256) {
    const long long e = i * 4, r = e / n;
    const int col = (int)(e - r * n);
    f32x4 s = *(const f32x4*)(part + e);
    for (int k = 1; k < splits; ++k) s += *(const f32x4*)(part + k * slice + e);
    f32x4* o = (f32x4*)(out + r * ldo + col);
    *o = *o + s;
  }
}

// p[i] = v for i < n (a kernel rather than a memset so that callers can capture it in a graph).
// 16-byte stores over the aligned body, dwords for the tail.
__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t* p, uint32_t v, long long n) {
  const long long n4 = n / 4;
  const long long stride = (long long)gridDim.x * 256;
  u32x4* p4 = (u32x4*)p;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) p4[i] = u32x4{v, v, v, v};
  for (long long i = n4 * 4 + (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) p[i] = v;
}
