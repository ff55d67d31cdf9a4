// C ABI of the L2L relay-execution library (see include/l2l.h): context, param stage / grad drain
// pipeline, and the per-layer forward / backward schedules over all U micro-batches (Algorithm 2).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <type_traits>
#include <utility>
#include <vector>

#include "../../include/l2l.h"
#include "gemm.h"
#include "gemm_variants.h"
#include "attention.h"
#include "rowwise.h"

// ================================================================================================
// packed layouts (host only)
// ================================================================================================
namespace {

constexpr long long ALIGN = 128;  // elements
inline long long up(long long x, long long a) { return (x + a - 1) / a * a; }

enum { T_WQKV, T_BQKV, T_WO, T_BO, T_G1, T_BE1, T_W1, T_B1, T_W2, T_B2, T_G2, T_BE2, N_LAYER_T };
enum { E_E, E_P, E_GE, E_BE, E_BV, N_EMBED_T };
const char* kLayerNames[N_LAYER_T] = {"Wqkv", "bqkv", "Wo", "bo", "g1", "be1", "W1", "b1", "W2", "b2", "g2", "be2"};
const char* kEmbedNames[N_EMBED_T] = {"E", "P", "ge", "be", "bv"};

struct Layout {
  long long size[N_LAYER_T], off[N_LAYER_T], total;
  long long esize[N_EMBED_T], eoff[N_EMBED_T], etotal;
};

bool config_ok(const l2l_config* c) {
  if (!c) return false;
  if (c->hidden <= 0 || c->heads <= 0 || c->ffn <= 0 || c->seq <= 0 || c->ubatch <= 0 || c->num_ubatches <= 0) return false;
  if (c->hidden % 8 || c->ffn % 8 || c->seq % 8) return false;
  if (c->hidden % c->heads || (c->hidden / c->heads) % 8) return false;
  if (c->dtype != L2L_F32 && c->dtype != L2L_BF16 && c->dtype != L2L_FP16) return false;
  if (c->vocab < 0 || c->vocab % 2) return false;
  if (c->ubatch_group < 0 || c->ubatch_group > c->num_ubatches) return false;
  if (!(c->ln_eps >= 0.f)) return false;
  if ((long long)c->ubatch * c->seq * c->num_ubatches > (1LL << 30)) return false;
  return true;
}

Layout make_layout(const l2l_config* c) {
  Layout L;
  const long long H = c->hidden, F = c->ffn, V = c->vocab, S = c->seq;
  const long long s[N_LAYER_T] = {H * 3 * H, 3 * H, H * H, H, H, H, H * F, F, F * H, H, H, H};
  long long o = 0;
  for (int i = 0; i < N_LAYER_T; ++i) { L.size[i] = s[i]; L.off[i] = o; o = up(o + s[i], ALIGN); }
  L.total = o;
  const long long es[N_EMBED_T] = {V * H, S * H, H, H, V};
  o = 0;
  for (int i = 0; i < N_EMBED_T; ++i) { L.esize[i] = es[i]; L.eoff[i] = o; o = up(o + es[i], ALIGN); }
  L.etotal = o;
  return L;
}

inline size_t esize(int dtype) { return dtype == L2L_F32 ? 4 : 2; }
inline bool is16(int dtype) { return dtype == L2L_BF16 || dtype == L2L_FP16; }

// packed block of the sequence-classification head: Wp[H,H] | bp[H] | Wc[H,C] | bc[C]
enum { C_WP, C_BP, C_WC, C_BC, N_CLS_T };
const char* kClsNames[N_CLS_T] = {"Wp", "bp", "Wc", "bc"};
struct ClsLayout { long long off[N_CLS_T], size[N_CLS_T], total; };
ClsLayout make_cls_layout(const l2l_config* c, int classes) {
  ClsLayout L;
  const long long H = c->hidden, C = classes;
  const long long s[N_CLS_T] = {H * H, H, H * C, C};
  long long o = 0;
  for (int i = 0; i < N_CLS_T; ++i) { L.size[i] = s[i]; L.off[i] = o; o = up(o + s[i], ALIGN); }
  L.total = o;
  return L;
}

}  // namespace

extern "C" {
int l2l_layer_tensor_count(void) { return N_LAYER_T; }
int l2l_embed_tensor_count(void) { return N_EMBED_T; }
long long l2l_layer_tensor_offset(const l2l_config* c, int i) {
  return (!config_ok(c) || i < 0 || i >= N_LAYER_T) ? -1 : make_layout(c).off[i];
}
long long l2l_layer_tensor_size(const l2l_config* c, int i) {
  return (!config_ok(c) || i < 0 || i >= N_LAYER_T) ? -1 : make_layout(c).size[i];
}
const char* l2l_layer_tensor_name(int i) { return (i < 0 || i >= N_LAYER_T) ? nullptr : kLayerNames[i]; }
long long l2l_embed_tensor_offset(const l2l_config* c, int i) {
  return (!config_ok(c) || i < 0 || i >= N_EMBED_T) ? -1 : make_layout(c).eoff[i];
}
long long l2l_embed_tensor_size(const l2l_config* c, int i) {
  return (!config_ok(c) || i < 0 || i >= N_EMBED_T) ? -1 : make_layout(c).esize[i];
}
const char* l2l_embed_tensor_name(int i) { return (i < 0 || i >= N_EMBED_T) ? nullptr : kEmbedNames[i]; }
size_t l2l_layer_param_count(const l2l_config* c) {
  if (!config_ok(c)) return 0;
  const size_t H = c->hidden, F = c->ffn;
  return 4 * H * H + 2 * H * F + 9 * H + F;
}
size_t l2l_layer_packed_elems(const l2l_config* c) { return config_ok(c) ? (size_t)make_layout(c).total : 0; }
size_t l2l_layer_param_bytes(const l2l_config* c) { return config_ok(c) ? (size_t)make_layout(c).total * esize(c->dtype) : 0; }
size_t l2l_layer_grad_bytes(const l2l_config* c) { return config_ok(c) ? (size_t)make_layout(c).total * 4 : 0; }
size_t l2l_embed_packed_elems(const l2l_config* c) { return config_ok(c) ? (size_t)make_layout(c).etotal : 0; }
int l2l_cls_tensor_count(void) { return N_CLS_T; }
const char* l2l_cls_tensor_name(int i) { return (i < 0 || i >= N_CLS_T) ? nullptr : kClsNames[i]; }
long long l2l_cls_tensor_offset(const l2l_config* c, int classes, int i) {
  return (!config_ok(c) || classes < 2 || i < 0 || i >= N_CLS_T) ? -1 : make_cls_layout(c, classes).off[i];
}
long long l2l_cls_tensor_size(const l2l_config* c, int classes, int i) {
  return (!config_ok(c) || classes < 2 || i < 0 || i >= N_CLS_T) ? -1 : make_cls_layout(c, classes).size[i];
}
size_t l2l_cls_packed_elems(const l2l_config* c, int classes) {
  return (config_ok(c) && classes >= 2) ? (size_t)make_cls_layout(c, classes).total : 0;
}
size_t l2l_embed_param_bytes(const l2l_config* c) { return config_ok(c) ? (size_t)make_layout(c).etotal * esize(c->dtype) : 0; }
size_t l2l_embed_grad_bytes(const l2l_config* c) { return config_ok(c) ? (size_t)make_layout(c).etotal * 4 : 0; }
int l2l_config_check(const l2l_config* c) { return config_ok(c) ? L2L_OK : L2L_E_ARG; }
}

// ================================================================================================
// context
// ================================================================================================
struct ProfRec {
  hipEvent_t a, b;
  int cls;
  double flops, bytes;
  int shape = -1;   // GEMM class: index into l2l_ctx::prof_shapes
};

// per distinct GEMM launch shape, for the table of l2l_profile_gemm_table
struct ProfShape {
  int M, N, K, a_kc, b_kc, epi, out_f32;
  int pass;   // 0 forward pass, 1 recompute, 2 backward, 3 elsewhere
  long long launches = 0;
  double ms = 0.0;
};

struct l2l_ctx {
  l2l_config cfg;
  Layout lay;
  hipStream_t cs = nullptr, xs = nullptr;  // compute, copy
  int group = 1;                            // micro-batches per launch
  // tuning and test switches, read from the environment once, by l2l_create (see include/l2l.h)
  int no_fused_attention = 0;               // L2L_NO_FUSED_ATTENTION=1: use the batched-GEMM attention path
  int force_splits = 0;                     // L2L_FORCE_SPLITS=n: split factor of the accumulating fp32 GEMMs
  int split_atomics = 0;                    // L2L_SPLIT_ATOMICS=1: K splits add with atomics, not through the workspace
  int copy_rows = 1;                        // drains issued as rows (DMA engine); L2L_COPY_ROWS=0: as plain copies (the runtime's copy kernel)
  int no_weight_transpose = 0;              // L2L_NO_WEIGHT_TRANSPOSE=1: forward GEMMs read W as stored ([in, out], K-strided B operand)
  int resident_cus = 0;                     // workgroups of a resident GEMM launch (CUs of the device; L2L_GEMM_RESIDENT=0: none)
  int32_t* bad_ids = nullptr;               // device flag: a token id or label outside the vocabulary was seen
  long long T = 0, Mg = 0;                  // tokens per micro-batch, rows per launch group
  size_t dev_bytes = 0;
  std::vector<void*> allocs;

  // parameter slots
  void* slot[2] = {nullptr, nullptr};
  int slot_layer[2] = {-1, -1};
  hipEvent_t slot_staged[2] = {}, slot_released[2] = {};
  // gradient accumulators
  float* gacc[2] = {nullptr, nullptr};
  int gacc_layer[2] = {-1, -1};
  int gacc_state[2] = {0, 0};  // 0 free, 1 holds un-drained grads, 2 drain enqueued
  hipEvent_t gacc_ready[2] = {}, gacc_landed[2] = {}, gacc_drained[2] = {};  // bwd done / D2H landed / cleared again
  int gacc_next = 0;

  // workspace (group-sized)
  void *qkv, *p, *c, *r1, *y1, *u1, *ga, *r2, *dr2, *du1, *dy1, *dr1, *dc, *dp, *dqkv, *ytmp;
  float *mean1, *rstd1, *mean2, *rstd2;
  float *lse = nullptr, *dsum = nullptr;   // chunked attention: row statistics between its kernels
  void* wt[2] = {nullptr, nullptr};  // bf16 mode: per slot, [out, in] copies of the four weight matrices (packed offsets)

  // embedding / head
  void* emb = nullptr;
  float* egacc = nullptr;
  int drain_dtype = L2L_F32;    // format of the drained gradients on the host (l2l_set_drain_dtype)
  void* drain_stage = nullptr;  // 16-bit drains: the rounded copy a drain sends (one suffices: the copy stream runs in order)
  size_t drain_stage_elems = 0;
  float* split_ws = nullptr;    // partial results of K-split GEMMs (fp32, `splits` dense [M, N] matrices)
  size_t split_ws_elems = 0;
  float* colsum_ws = nullptr;   // [rows / 64][max(F, 3H)] fp32: partial column sums written by a GEMM epilogue
  size_t colsum_ws_elems = 0;
  int emb_staged = 0, egacc_state = 0;
  long long egacc_part_next = 0;   // l2l_embed_grad_drain_part: first element of the next piece
  hipEvent_t emb_staged_ev = nullptr, emb_released_ev = nullptr, egacc_ready = nullptr, egacc_landed = nullptr, egacc_drained = nullptr;
  float *emean = nullptr, *erstd = nullptr;
  int32_t *lab_idx = nullptr, *lab_cnt = nullptr, *lab_total = nullptr, *lab_gidx = nullptr, *chunk_cnt = nullptr;
  // sequence-classification head (allocated at the first l2l_cls_stage)
  int cls_classes = 0, cls_staged = 0, cls_state = 0;       // state: 0 clean, 1 gradients ready, 2 drain in flight
  long long cls_off[4] = {}, cls_size[4] = {}, cls_total = 0, cls_cp = 0;
  void *cls_w = nullptr, *cls_x = nullptr, *cls_u = nullptr, *cls_p = nullptr, *cls_dz = nullptr, *cls_dp = nullptr, *cls_du = nullptr,
       *cls_dx = nullptr;
  float *cls_g = nullptr, *cls_z = nullptr;
  hipEvent_t cls_staged_ev = nullptr, cls_released_ev = nullptr, cls_ready = nullptr, cls_landed = nullptr, cls_drained = nullptr;
  long long head_rows = 0;   // labelled rows per pass of the head
  float loss_scale = 1.0f;   // factor on the loss gradient (fp16 training)
  void *xl = nullptr, *dz = nullptr, *dxl = nullptr;
  float* dxl32 = nullptr;   // 16-bit modes: the head's dX in fp32, the target of a K-split GEMM
  float* logits = nullptr;
  long long Vp = 0;

  // profiling
  int prof_on = 0;
  std::vector<ProfRec> prof;
  std::vector<ProfShape> prof_shapes;
  int prof_pass = 3;   // which pass of the relay the launches being recorded belong to
  std::vector<hipEvent_t> ev_pool;
  hipEvent_t prof_base = nullptr;                          // recorded when profiling is switched on
  std::vector<std::pair<float, float>> iv_compute, iv_copy;  // resolved intervals, ms after prof_base
  long long prof_n[L2L_PROF_CLASSES] = {};
  double prof_ms[L2L_PROF_CLASSES] = {}, prof_fl[L2L_PROF_CLASSES] = {}, prof_by[L2L_PROF_CLASSES] = {};

  char err[512] = {0};
};

namespace {

int fail(l2l_ctx* c, int code, const char* fmt, ...) {
  if (c) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(c->err, sizeof(c->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

#define HIP_TRY(ctx, call)                                                                       \
  do {                                                                                           \
    hipError_t e_ = (call);                                                                      \
    if (e_ != hipSuccess) return fail(ctx, L2L_E_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

#define L2L_TRY(call)        \
  do {                       \
    int r_ = (call);         \
    if (r_ != L2L_OK) return r_; \
  } while (0)

int dev_alloc(l2l_ctx* c, void** p, size_t bytes) {
  bytes = (bytes + 255) / 256 * 256;
  if (bytes == 0) bytes = 256;
  hipError_t e = hipMalloc(p, bytes);
  if (e != hipSuccess) return fail(c, L2L_E_NOMEM, "hipMalloc(%zu): %s", bytes, hipGetErrorString(e));
  c->allocs.push_back(*p);
  c->dev_bytes += bytes;
  return L2L_OK;
}

hipEvent_t take_event(l2l_ctx* c) {
  if (!c->ev_pool.empty()) {
    hipEvent_t e = c->ev_pool.back();
    c->ev_pool.pop_back();
    return e;
  }
  hipEvent_t e;
  (void)hipEventCreate(&e);
  return e;
}

// brackets work on the copy stream (profile mode 1 only); call begin after the stream's waits are queued
struct CopyMark { hipEvent_t a = nullptr; };
CopyMark copy_begin(l2l_ctx* c) {
  CopyMark m;
  if (c->prof_on == 1) {
    m.a = take_event(c);
    (void)hipEventRecord(m.a, c->xs);
  }
  return m;
}
void copy_end(l2l_ctx* c, const CopyMark& m, double bytes) {
  if (!m.a) return;
  hipEvent_t b = take_event(c);
  (void)hipEventRecord(b, c->xs);
  c->prof.push_back({m.a, b, L2L_PROF_COPY, 0.0, bytes});
}

template <typename F>
int timed(l2l_ctx* c, int cls, double flops, double bytes, F&& f, int shape = -1) {
  if (!c->prof_on || (c->prof_on == 2 && cls != L2L_PROF_GEMM)) {
    f();
  } else {
    hipEvent_t a = take_event(c), b = take_event(c);
    (void)hipEventRecord(a, c->cs);
    f();
    (void)hipEventRecord(b, c->cs);
    c->prof.push_back({a, b, cls, flops, bytes, shape});
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(c, L2L_E_HIP, "kernel launch: %s", hipGetErrorString(e));
  return L2L_OK;
}

// ------------------------------------------------------------------------------------------------
// GEMM dispatch
// ------------------------------------------------------------------------------------------------
GemmArgs gemm_args(int M, int N, int K, const void* A, long long lda, int a_kc, const void* B, long long ldb, int b_kc,
                   void* C, long long ldc) {
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.A = A; g.B = B; g.C = C;
  g.M = M; g.N = N; g.K = K;
  g.a_kc = a_kc; g.b_kc = b_kc;
  g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.nbatch = 1; g.zdiv = 1;
  g.alpha = 1.0f;
  return g;
}

bool mfma_ok(const GemmArgs& g) {
  auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  if (!al16(g.A) || !al16(g.B)) return false;
  if (g.lda % 8 || g.ldb % 8) return false;
  if (g.a_zo % 8 || g.a_zi % 8 || g.b_zo % 8 || g.b_zi % 8) return false;
  // a chunk is loaded when its first element is in range: pitches must cover the rounded-up extent
  const long long m8 = up(g.M, 8), n8 = up(g.N, 8), k8 = up(g.K, 8);
  if (g.a_kc ? g.lda < k8 : g.lda < m8) return false;
  if (g.b_kc ? g.ldb < k8 : g.ldb < n8) return false;
  if (g.a_kc && g.b_kc && g.K % 8) return false;  // nobody guarantees zero padding in both
  // The kernels address an operand panel through a 32-bit buffer descriptor, with 0x80000000 as the offset that is
  // out of range for sure: every panel (one batch entry's operand, seen from its first element) must end below
  // 2 GiB, and the offsets of the K-strided loads that run up to three k-tiles past the end must not wrap.
  const long long lim = (1LL << 31) - 1;
  const long long ea = g.a_kc ? (long long)(g.M - 1) * g.lda + k8 : (long long)(g.K + 192) * g.lda + m8;
  const long long eb = g.b_kc ? (long long)(g.N - 1) * g.ldb + k8 : (long long)(g.K + 192) * g.ldb + n8;
  if (ea * 2 > lim || eb * 2 > lim) return false;
  return true;
}

// tile variants of the MFMA kernel live in their own translation units (gemm_variant.hip)
struct TileCfg { int bm, bn, bk, wm, wn, direct; };
#define L2L_ROW(i, bm, bn, bk, wm, wn, d) {bm, bn, bk, wm, wn, d},
constexpr TileCfg kTiles[] = {L2L_GEMM_VARIANTS(L2L_ROW)};
#undef L2L_ROW
constexpr int kNumTiles = kNumGemmVariants;

void launch_mfma_variant(int v, const GemmArgs& g, hipStream_t s, int splits, bool out_f32, bool fp16_in) {
  switch (v) {
#define L2L_CASE(i, bm, bn, bk, wm, wn, d) \
  case i: fp16_in ? l2l_launch_mfma_h##i(g, s, splits, out_f32) : l2l_launch_mfma_v##i(g, s, splits, out_f32); break;
    L2L_GEMM_VARIANTS(L2L_CASE)
#undef L2L_CASE
    default: break;
  }
}

template <typename T, typename TC>
void launch_plain(const GemmArgs& g, hipStream_t s) {
  dim3 grid((g.N + 63) / 64, (g.M + 63) / 64, g.nbatch);
  hipLaunchKernelGGL((gemm_plain_kernel<T, TC>), grid, dim3(256), 0, s, g);
}

// tile variant and split-K factor for one launch
void pick_tile(const GemmArgs& g, bool out_f32, int* variant, int* splits) {
  int v = 0;
  *splits = 1;
  const long long small = std::min(g.M, g.N);
  const bool kc = g.a_kc || !g.b_kc;   // the direct-to-LDS kernel covers every layout pair but (A K-strided, B K-contiguous)
  if (small >= 256 && g.K >= 256) v = kc ? 6 : 3;
  else if (g.M >= 256 && g.N >= 128) v = kc ? 8 : 2;
  else if (g.N <= 64) v = 1;
  else v = kc ? 7 : 0;
  const TileCfg t = kTiles[v];
  // split K when an accumulating fp32 GEMM has too few tiles to fill 256 CUs
  if (out_f32 && (g.epi == EPI_ACCUM) && !g.k_dev) {
    const long long tiles = (long long)((g.M + t.bm - 1) / t.bm) * ((g.N + t.bn - 1) / t.bn) * g.nbatch;
    const int nk = (g.K + t.bk - 1) / t.bk;
    // one resident workgroup per CU: tiles x splits as close to the 256 CUs as it gets without exceeding
    // them (measured best for the dW shapes, partial results through the workspace: 64 x 4, 48 x 5, 16 x 16)
    long long want = tiles < 256 ? 256 / tiles : 1;
    want = std::min<long long>(want, std::max(1, nk / 8));
    *splits = (int)std::max<long long>(1, std::min<long long>(want, 64));
  }
  *variant = v;
}

// whether gemm() will run this launch on the direct-to-LDS kernel, the one that honours EPI_COLSUM; otherwise the
// caller runs the column-sum kernel itself
// *rows: rows of the partial-sum matrix the kernel will fill (one per wave-tile row of C)
bool colsum_in_gemm_ok(int dtype, bool out_f32, const GemmArgs& g, int* rows = nullptr) {
  if (!is16(dtype) || out_f32 || !mfma_ok(g) || g.nbatch != 1 || g.m_dev || g.k_dev) return false;
  int v, splits;
  pick_tile(g, out_f32, &v, &splits);
  if (!(kTiles[v].direct && (g.a_kc || !g.b_kc) && splits == 1)) return false;
  if (rows) *rows = (g.M + kTiles[v].wm - 1) / kTiles[v].wm;
  return gemm_vec_ok(g, g.epi | EPI_COLSUM, g.C);
}

// An accumulating fp32 GEMM split over K whose splits store their partial tiles in `ws` (fp32, room for ws_elems
// elements; `splits` dense [M, N] slices, every element of every slice written) and are then added into C by one
// kernel.  Returns false, with nothing launched, where the shape, the tile variant or the room do not allow it.
enum { SPLIT_NOT_APPLICABLE = 0, SPLIT_LAUNCHED = 1, SPLIT_NO_ROOM = 2 };
int launch_split_through_workspace(int v, const GemmArgs& g, hipStream_t s, int splits, bool out_f32, bool fp16_in, float* ws,
                                   size_t ws_elems) {
  const long long slice = (long long)g.M * g.N;
  if (!(splits > 1 && out_f32 && g.epi == EPI_ACCUM && kTiles[v].direct && g.nbatch == 1 && g.N % 8 == 0 && g.ldc % 4 == 0 &&
        ((uintptr_t)g.C & 15) == 0 && ws && !g.m_dev && !g.k_dev))
    return SPLIT_NOT_APPLICABLE;
  const int nk = (g.K + kTiles[v].bk - 1) / kTiles[v].bk, per = (nk + splits - 1) / splits;
  splits = (nk + per - 1) / per;   // no empty split: every slice of the workspace gets written
  if (splits <= 1) return SPLIT_NOT_APPLICABLE;
  if ((size_t)splits * slice > ws_elems) return SPLIT_NO_ROOM;
  GemmArgs p = g;
  p.C = ws; p.ldc = g.N; p.split_stride = slice; p.epi = 0;
  const unsigned blocks = (unsigned)std::min<long long>((slice / 4 + 255) / 256, 4096);
  launch_mfma_variant(v, p, s, splits, out_f32, fp16_in);
  hipLaunchKernelGGL(split_sum_kernel, dim3(blocks), dim3(256), 0, s, ws, splits, (long long)g.M, g.N, (float*)g.C, g.ldc);
  return SPLIT_LAUNCHED;
}

// impl: 0 auto, 1 plain, 2 mfma (auto tile), 100 + v: mfma tile variant v (tuning)
int gemm(l2l_ctx* c, int dtype, bool out_f32, const GemmArgs& g, int impl = 0, int cls = L2L_PROF_GEMM) {
  if (g.M <= 0 || g.N <= 0 || g.nbatch <= 0) return L2L_OK;
  if (g.nbatch > 65535 || (g.M + 63) / 64 > 65535) return fail(c, L2L_E_ARG, "gemm: grid too large");
  const bool can_mfma = is16(dtype) && mfma_ok(g);
  if (impl >= 2 && !can_mfma) return fail(c, L2L_E_ARG, "gemm: shape/alignment not supported by the MFMA kernel");
  if (impl >= 100 + kNumTiles) return fail(c, L2L_E_ARG, "gemm: no such tile variant");
  if ((g.epi & EPI_COLSUM) && (impl != 0 || !g.colsum || !colsum_in_gemm_ok(dtype, out_f32, g)))
    return fail(c, L2L_E_ARG, "gemm: column sums are not available on this path");
  const bool use_mfma = impl >= 2 || (impl == 0 && can_mfma);
  const double flops = 2.0 * g.M * g.N * (double)g.K * g.nbatch;
  const double es = esize(dtype);
  const double bytes = ((double)g.M * g.K + (double)g.K * g.N) * es * g.nbatch + (double)g.M * g.N * (out_f32 ? 4 : es) * g.nbatch;
  int shape = -1;
  if (c->prof_on && cls == L2L_PROF_GEMM) {   // the launch's row in the per-shape table
    for (size_t i = 0; i < c->prof_shapes.size() && shape < 0; ++i) {
      const ProfShape& p = c->prof_shapes[i];
      if (p.M == g.M && p.N == g.N && p.K == g.K && p.a_kc == g.a_kc && p.b_kc == g.b_kc && p.epi == g.epi && p.out_f32 == (int)out_f32 && p.pass == c->prof_pass) shape = (int)i;
    }
    if (shape < 0) {
      ProfShape p;
      p.M = g.M; p.N = g.N; p.K = g.K; p.a_kc = g.a_kc; p.b_kc = g.b_kc; p.epi = g.epi; p.out_f32 = out_f32; p.pass = c->prof_pass;
      c->prof_shapes.push_back(p);
      shape = (int)c->prof_shapes.size() - 1;
    }
  }
  return timed(c, cls, flops, bytes, [&] {
    if (use_mfma) {
      int v, splits;
      pick_tile(g, out_f32, &v, &splits);
      if (impl >= 100) v = impl - 100;
      if (kTiles[v].direct && !g.a_kc && g.b_kc) v = 3;   // no direct-to-LDS kernel for A K-strided with B K-contiguous
      if (c->force_splits > 0 && out_f32 && g.epi == EPI_ACCUM) splits = c->force_splits;
      GemmArgs gr = g;
      gr.resident = c->resident_cus;
      // K split over grid.y: with a workspace the splits store their partial tiles (16-byte stores) and one kernel
      // adds them into C; without, they add into C with fp32 atomics, which run at the L2's atomic rate (65536 per
      // workgroup: 40 % of the time of a 1024 x 1024 x 32768 GEMM) and in no fixed order
      if (c->split_ws && !c->split_atomics &&
          launch_split_through_workspace(v, gr, c->cs, splits, out_f32, dtype == L2L_FP16, c->split_ws, c->split_ws_elems) ==
              SPLIT_LAUNCHED)
        return;
      launch_mfma_variant(v, gr, c->cs, splits, out_f32, dtype == L2L_FP16);
    } else if (dtype == L2L_BF16) {
      if (out_f32) launch_plain<bf16, float>(g, c->cs);
      else launch_plain<bf16, bf16>(g, c->cs);
    } else if (dtype == L2L_FP16) {
      if (out_f32) launch_plain<fp16, float>(g, c->cs);
      else launch_plain<fp16, fp16>(g, c->cs);
    } else {
      launch_plain<float, float>(g, c->cs);
    }
  }, shape);
}

// ------------------------------------------------------------------------------------------------
// typed launch helpers for the row-wise kernels
// ------------------------------------------------------------------------------------------------
template <typename T>
int ln_fwd(l2l_ctx* c, const void* x, const void* gamma, const void* beta, void* y, float* mean, float* rstd, long long rows,
           int n, float eps) {
  if (rows <= 0) return L2L_OK;
  return timed(c, L2L_PROF_ROWWISE, 0, 2.0 * rows * n * sizeof(T), [&] {
    hipLaunchKernelGGL(ln_fwd_kernel<T>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, c->cs, (const T*)x, (const T*)gamma,
                       (const T*)beta, (T*)y, mean, rstd, (int)rows, n, eps);
  });
}

template <typename T>
int bias_grad(l2l_ctx* c, const void* a, long long lda, float* out, long long rows, int n, const int* rows_dev = nullptr);

// whether the one-pass kernel may take its rows through the LDS ring: every column group in use (the kernel counts
// one store per group and row), and the ring's slots fit the buffer the column sums are combined in
constexpr int LNF_RING = 3;   // slots per wave: two rows on their way while one is worked on (five slots measured the same)
bool ln_bwd_ring_ok(int n, int nch) { return (n + 511) / 512 == nch && 4 * LNF_RING * 2 * nch * 1024 <= 80 * 1024; }   // (two blocks per CU)
// dynamic LDS of the one-pass kernel: the buffer the four waves' column sums meet in, or the ring's slots if those take more
size_t ln_bwd_lds_bytes(int n, int nch, bool is16) {
  const size_t red = (size_t)4 * 3 * nch * 512 * sizeof(float);
  const size_t ring = is16 && ln_bwd_ring_ok(n, nch) ? (size_t)4 * LNF_RING * 2 * nch * 1024 : 0;
  return std::max(red, ring);
}

// whether LayerNorm backward runs as the one-pass kernel, which can also compute the row statistics itself
bool ln_bwd_one_pass(int n) { return n % 8 == 0 && n <= 2048; }

// LayerNorm backward: dx, dgamma, dbeta, and dbias = colsum(dx) (the bias in front of the LayerNorm).
// mean == rstd == nullptr (one-pass kernel only): the statistics are recomputed from x with `eps`.
template <typename T>
int ln_bwd(l2l_ctx* c, const void* dy, const void* x, const float* mean, const float* rstd, const void* gamma, void* dx,
           float* dgamma, float* dbeta, float* dbias, long long rows, int n, float eps) {
  if (rows <= 0) return L2L_OK;
  if (!mean && !ln_bwd_one_pass(n)) return fail(c, L2L_E_STATE, "ln_bwd: statistics missing");
  if (ln_bwd_one_pass(n)) {   // one pass, column sums included
    const int nch = n <= 512 ? 1 : n <= 1024 ? 2 : 4;
    const size_t lds = ln_bwd_lds_bytes(n, nch, sizeof(T) == 2);
    return timed(c, L2L_PROF_ROWWISE, 0, 3.0 * rows * n * sizeof(T), [&] {
      const dim3 grid((unsigned)((rows + LNF_ROWS - 1) / LNF_ROWS));
      auto go = [&](auto kern) {
        static_cast<void>(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, c->cs, (const T*)dy, (const T*)x, mean, rstd, (const T*)gamma, (T*)dx,
                           dgamma, dbeta, dbias, (int)rows, n, eps, (const T*)nullptr);
      };
      if constexpr (sizeof(T) == 2) {
        if (ln_bwd_ring_ok(n, nch)) {   // rows through LDS (same LDS size: the ring's slots are the reduction's buffer)
          if (nch == 1) go(ln_bwd_fused_kernel<T, 1, false, LNF_RING>);
          else if (nch == 2) go(ln_bwd_fused_kernel<T, 2, false, LNF_RING>);
          else go(ln_bwd_fused_kernel<T, 4, false, LNF_RING>);
          return;
        }
      }
      if (nch == 1) go(ln_bwd_fused_kernel<T, 1>);
      else if (nch == 2) go(ln_bwd_fused_kernel<T, 2>);
      else go(ln_bwd_fused_kernel<T, 4>);
    });
  }
  L2L_TRY(timed(c, L2L_PROF_ROWWISE, 0, 3.0 * rows * n * sizeof(T), [&] {
    hipLaunchKernelGGL(ln_bwd_dx_kernel<T>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, c->cs, (const T*)dy, (const T*)x,
                       mean, rstd, (const T*)gamma, (T*)dx, (int)rows, n);
  }));
  L2L_TRY(timed(c, L2L_PROF_COLSUM, 0, 2.0 * rows * n * sizeof(T), [&] {
    const int rpb = colsum_rows_per_block(rows, n);
    dim3 grid((n + 127) / 128, (unsigned)((rows + rpb - 1) / rpb));
    hipLaunchKernelGGL((colsum_kernel<T, 1>), grid, dim3(256), 0, c->cs, (const T*)dy, (long long)n, (const T*)x, mean, rstd,
                       (const int32_t*)nullptr, (const T*)nullptr, (const T*)nullptr, 0, dgamma, dbeta, (int)rows, n,
                       (const int*)nullptr, 0, rpb);
  }));
  return bias_grad<T>(c, dx, n, dbias, rows, n);
}

// LayerNorm backward from the OUTPUT y of the LayerNorm and the 1/sigma kept by the forward pass (one-pass kernel only)
template <typename T>
int ln_bwd_from_y(l2l_ctx* c, const void* dy, const void* y, const float* rstd, const void* gamma, const void* beta, void* dx,
                  float* dgamma, float* dbeta, float* dbias, long long rows, int n) {
  if (rows <= 0) return L2L_OK;
  if (!ln_bwd_one_pass(n) || !rstd) return fail(c, L2L_E_STATE, "ln_bwd_from_y: needs the one-pass kernel and the kept statistics");
  const int nch = n <= 512 ? 1 : n <= 1024 ? 2 : 4;
  const size_t lds = ln_bwd_lds_bytes(n, nch, sizeof(T) == 2);
  return timed(c, L2L_PROF_ROWWISE, 0, 3.0 * rows * n * sizeof(T), [&] {
    const dim3 grid((unsigned)((rows + LNF_ROWS - 1) / LNF_ROWS));
    auto go = [&](auto kern) {
      static_cast<void>(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
      hipLaunchKernelGGL(kern, grid, dim3(256), lds, c->cs, (const T*)dy, (const T*)y, (const float*)nullptr, rstd, (const T*)gamma, (T*)dx,
                         dgamma, dbeta, dbias, (int)rows, n, 0.f, (const T*)beta);
    };
    if constexpr (sizeof(T) == 2) {
      if (ln_bwd_ring_ok(n, nch)) {
        if (nch == 1) go(ln_bwd_fused_kernel<T, 1, true, LNF_RING>);
        else if (nch == 2) go(ln_bwd_fused_kernel<T, 2, true, LNF_RING>);
        else go(ln_bwd_fused_kernel<T, 4, true, LNF_RING>);
        return;
      }
    }
    if (nch == 1) go(ln_bwd_fused_kernel<T, 1, true>);
    else if (nch == 2) go(ln_bwd_fused_kernel<T, 2, true>);
    else go(ln_bwd_fused_kernel<T, 4, true>);
  });
}

template <typename T>
int bias_grad(l2l_ctx* c, const void* a, long long lda, float* out, long long rows, int n, const int* rows_dev) {
  if (rows <= 0) return L2L_OK;
  return timed(c, L2L_PROF_COLSUM, 0, 1.0 * rows * n * sizeof(T), [&] {
    const int rpb = colsum_rows_per_block(rows, n);
    dim3 grid((n + 127) / 128, (unsigned)((rows + rpb - 1) / rpb));
    hipLaunchKernelGGL((colsum_kernel<T, 0>), grid, dim3(256), 0, c->cs, (const T*)a, lda, (const T*)nullptr,
                       (const float*)nullptr, (const float*)nullptr, (const int32_t*)nullptr, (const T*)nullptr,
                       (const T*)nullptr, 0, (float*)nullptr, out, (int)rows, n, rows_dev, 0, rpb);
  });
}

// zero on the copy stream: keeps the clearing of a drained accumulator off the compute stream
int fill_zero_copy_stream(l2l_ctx* c, void* p, size_t bytes) {
  const long long n = (long long)(bytes / 4);
  if (n <= 0) return L2L_OK;
  const unsigned blocks = (unsigned)std::min<long long>((n / 4 + 255) / 256 + 1, 2048);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks), dim3(256), 0, c->xs, (uint32_t*)p, 0u, n);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(c, L2L_E_HIP, "fill launch: %s", hipGetErrorString(e));
  return L2L_OK;
}

// the fused attention kernels take the 16-bit formats, head width 64 and sequences of 32, 64, 96 or 128 tokens ...
template <typename T>
using attn_elem = typename std::conditional<std::is_same<T, fp16>::value, fp16, bf16>::type;   // (fp32 never gets there)
bool fused_attention_ok(const l2l_ctx* c) {
  const l2l_config& f = c->cfg;
  return is16(f.dtype) && f.hidden / f.heads == 64 && f.seq % 32 == 0 && f.seq <= attn::SMAX && !c->no_fused_attention;
}
// ... and the chunked ones longer sequences
bool fused_attention_long_ok(const l2l_ctx* c) {
  const l2l_config& f = c->cfg;
  return is16(f.dtype) && f.hidden / f.heads == 64 && f.seq % 32 == 0 && f.seq > attn::SMAX && !c->no_fused_attention;
}

int fill_zero(l2l_ctx* c, void* p, size_t bytes) {
  const long long n = (long long)(bytes / 4);
  if (n <= 0) return L2L_OK;
  const unsigned blocks = (unsigned)std::min<long long>((n / 4 + 255) / 256 + 1, 2048);
  return timed(c, L2L_PROF_OTHER, 0, (double)bytes, [&] {
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks), dim3(256), 0, c->cs, (uint32_t*)p, 0u, n);
  });
}

// bf16 mode: the forward GEMMs X W want W with its input index contiguous, like every other operand
// of the MFMA kernel's fastest path; the four matrices of a staged layer (25 MB at BERT-Large) are
// transposed once, on the copy stream right behind the stage's DMA, so that the work overlaps the
// previous layer's compute and all micro-batches share the result.
int transpose_weights(l2l_ctx* c, int slot) {
  if (!is16(c->cfg.dtype) || c->no_weight_transpose) return L2L_OK;   // the transpose moves 16-bit elements whatever their format
  const int H = c->cfg.hidden, F = c->cfg.ffn;
  const long long* off = c->lay.off;
  const struct { int t, rows, cols; } m[4] = {{T_WQKV, H, 3 * H}, {T_WO, H, H}, {T_W1, H, F}, {T_W2, F, H}};
  for (const auto& w : m) {
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((w.cols + 127) / 128, (w.rows + 127) / 128), dim3(256), 0, c->xs,
                       (const bf16*)c->slot[slot] + off[w.t], (bf16*)c->wt[slot] + off[w.t], w.rows, w.cols);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(c, L2L_E_HIP, "transpose launch: %s", hipGetErrorString(e));
  return L2L_OK;
}

// ------------------------------------------------------------------------------------------------
// one encoder layer, forward, on `ng` micro-batches starting at row block x (rows = ng * T)
// keep: also keep the GELU pre-activation and both LayerNorm statistics (backward recompute)
// ------------------------------------------------------------------------------------------------
// rstd2_out (forward pass only): where to keep LayerNorm 2's 1/sigma per row, or null.
// skip_ffn2 (recompute pass only): the backward pass takes LayerNorm 2's xhat from the stashed layer output and its
// kept 1/sigma, so the FFN2 product, whose only use in the backward pass is that LayerNorm's input, is not recomputed.
template <typename T>
int layer_forward_group(l2l_ctx* c, int slot, const void* x, void* y, int ng, bool keep, float* rstd2_out = nullptr,
                        bool skip_ffn2 = false) {
  const void* params = c->slot[slot];
  const l2l_config& f = c->cfg;
  const int H = f.hidden, A = f.heads, F = f.ffn, S = f.seq, d = H / A;
  const long long M = (long long)ng * c->T;
  const int nseq = ng * f.ubatch;
  const int dt = f.dtype;
  const T* P = (const T*)params;
  const long long* off = c->lay.off;
  T* qkv = (T*)c->qkv;
  c->prof_pass = keep ? 1 : 0;
  // weight operand of a forward GEMM: [out, in] copy (bf16) or the packed [in, out] matrix (fp32)
  const bool tw = is16(dt) && !c->no_weight_transpose;
  const T* W = tw ? (const T*)c->wt[slot] : P;
  auto wld = [&](int in, int out) { return (long long)(tw ? in : out); };

  // QKV projection with bias
  {
    GemmArgs g = gemm_args((int)M, 3 * H, H, x, H, 1, W + off[T_WQKV], wld(H, 3 * H), tw, qkv, 3 * H);
    g.epi = EPI_BIAS; g.bias = P + off[T_BQKV];
    L2L_TRY(gemm(c, dt, false, g));
  }
  // scores = Q K^T / sqrt(d) per (sequence, head), softmax over keys, context = P V
  if (fused_attention_ok(c)) {
    const double fl = 4.0 * S * S * d * nseq * A;
    L2L_TRY(timed(c, L2L_PROF_ATTN, fl, (3.0 + 1.0) * M * H * sizeof(T), [&] {
      using E = attn_elem<T>;
      hipLaunchKernelGGL(attn::attn_fwd_kernel<E>, dim3(nseq * A), dim3(256), 0, c->cs, (const E*)qkv, (E*)c->c, S, H, A,
                         1.0f / sqrtf((float)d));
    }));
  } else if (fused_attention_long_ok(c)) {
    const double fl = 4.0 * S * S * d * nseq * A;
    L2L_TRY(timed(c, L2L_PROF_ATTN, fl, (3.0 + 1.0) * M * H * sizeof(T), [&] {
      using E = attn_elem<T>;
      // (the row statistics are for the backward kernels: only the recompute pass keeps them)
      auto go = [&](auto kern) {
        hipLaunchKernelGGL(kern, dim3(nseq * A * ((S + attn::CH - 1) / attn::CH)), dim3(256), 0, c->cs, (const E*)qkv, (E*)c->c,
                           keep ? c->lse : nullptr, S, H, A, 1.0f / sqrtf((float)d));
      };
      if (S % attn::CH) go(attn::attn_fwd_long_kernel<E, true>); else go(attn::attn_fwd_long_kernel<E, false>);
    }));
  } else
  {
    GemmArgs g = gemm_args(S, S, d, qkv, 3 * H, 1, qkv + H, 3 * H, 1, c->p, S);
    g.nbatch = nseq * A; g.zdiv = A;
    g.a_zo = (long long)S * 3 * H; g.a_zi = d; g.b_zo = g.a_zo; g.b_zi = d;
    g.c_zo = (long long)A * S * S; g.c_zi = (long long)S * S;
    g.alpha = 1.0f / sqrtf((float)d);
    L2L_TRY(gemm(c, dt, false, g, 0, L2L_PROF_ATTN));
    const long long rows = (long long)nseq * A * S;
    L2L_TRY(timed(c, L2L_PROF_ATTN, 0, 2.0 * rows * S * sizeof(T), [&] {
      hipLaunchKernelGGL(softmax_fwd_kernel<T>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, c->cs, (T*)c->p, rows, S);
    }));
    GemmArgs h = gemm_args(S, d, S, c->p, S, 1, qkv + 2 * H, 3 * H, 0, c->c, H);
    h.nbatch = nseq * A; h.zdiv = A;
    h.a_zo = (long long)A * S * S; h.a_zi = (long long)S * S;
    h.b_zo = (long long)S * 3 * H; h.b_zi = d;
    h.c_zo = (long long)S * H; h.c_zi = d;
    L2L_TRY(gemm(c, dt, false, h, 0, L2L_PROF_ATTN));
  }
  // output projection + bias + residual, LayerNorm 1
  {
    GemmArgs g = gemm_args((int)M, H, H, c->c, H, 1, W + off[T_WO], wld(H, H), tw, c->r1, H);
    g.epi = EPI_BIAS | EPI_RESID; g.bias = P + off[T_BO]; g.resid = x; g.ldr = H;
    L2L_TRY(gemm(c, dt, false, g));
    L2L_TRY(ln_fwd<T>(c, c->r1, P + off[T_G1], P + off[T_BE1], c->y1, keep ? c->mean1 : nullptr, keep ? c->rstd1 : nullptr, M, H,
                      f.ln_eps));
  }
  // FFN1 + bias + GELU, FFN2 + bias + residual, LayerNorm 2
  {
    GemmArgs g = gemm_args((int)M, F, H, c->y1, H, 1, W + off[T_W1], wld(H, F), tw, c->ga, F);
    // (the recompute pass leaves gelu'(U1) behind instead of U1: the backward pass needs U1 for nothing else, and
    // here it costs one exponential next to the Phi(U1) that GELU needs anyway)
    g.epi = EPI_BIAS | EPI_GELU | (keep ? EPI_KEEPGRAD : 0); g.bias = P + off[T_B1]; g.aux_out = keep ? c->u1 : nullptr; g.ldaux = F;
    L2L_TRY(gemm(c, dt, false, g));
    if (keep && skip_ffn2) return L2L_OK;
    GemmArgs h = gemm_args((int)M, H, F, c->ga, F, 1, W + off[T_W2], wld(F, H), tw, c->r2, H);
    h.epi = EPI_BIAS | EPI_RESID; h.bias = P + off[T_B2]; h.resid = c->y1; h.ldr = H;
    L2L_TRY(gemm(c, dt, false, h));
    if (keep) {
      // backward needs only the statistics of LN2 (y itself was stashed by the forward pass), and the one-pass
      // backward kernel computes them itself
      if (!ln_bwd_one_pass(H))
        L2L_TRY(ln_fwd<T>(c, c->r2, P + off[T_G2], P + off[T_BE2], c->ytmp, c->mean2, c->rstd2, M, H, f.ln_eps));
    } else {
      L2L_TRY(ln_fwd<T>(c, c->r2, P + off[T_G2], P + off[T_BE2], y, rstd2_out ? c->mean2 : nullptr, rstd2_out, M, H, f.ln_eps));
    }
  }
  return L2L_OK;
}

// LayerNorm 2's backward from the stashed output, on its own: it needs nothing of the recompute pass, so it can run in
// front of it (see layer_bwd_impl) and leave dR2 in the workspace
template <typename T>
int layer_ln2_backward_from_y(l2l_ctx* c, const void* params, const void* dydx, float* G, int ng, const void* y, const float* rstd2) {
  const int H = c->cfg.hidden;
  const long long M = (long long)ng * c->T;
  const T* P = (const T*)params;
  const long long* off = c->lay.off;
  c->prof_pass = 2;
  return ln_bwd_from_y<T>(c, dydx, y, rstd2, P + off[T_G2], P + off[T_BE2], c->dr2, G + off[T_G2], G + off[T_BE2], G + off[T_B2], M, H);
}

// backward of the group whose forward intermediates are in the workspace; dy -> dx in place
// y, rstd2: the layer's stashed output and LayerNorm 2's kept 1/sigma for these rows (then the workspace holds no R2:
// the recompute pass skipped FFN2), or null
template <typename T>
int layer_backward_group(l2l_ctx* c, const void* params, const void* x, void* dydx, float* G, int ng, const void* y = nullptr,
                         const float* rstd2 = nullptr, bool ln2_done = false) {
  const l2l_config& f = c->cfg;
  const int H = f.hidden, A = f.heads, F = f.ffn, S = f.seq, d = H / A;
  const long long M = (long long)ng * c->T;
  const int nseq = ng * f.ubatch;
  const int dt = f.dtype;
  const T* P = (const T*)params;
  const long long* off = c->lay.off;
  T* qkv = (T*)c->qkv;
  T* dqkv = (T*)c->dqkv;
  const float alpha = 1.0f / sqrtf((float)d);
  c->prof_pass = 2;

  // LN2 backward
  bool db1_in_gemm = false;
  const bool own_stats = ln_bwd_one_pass(H);   // then the recompute pass did not run LN2
  if (ln2_done) {
    // layer_ln2_backward_from_y ran ahead of the recompute pass: dR2 is in the workspace
  } else if (y)
    L2L_TRY(ln_bwd_from_y<T>(c, dydx, y, rstd2, P + off[T_G2], P + off[T_BE2], c->dr2, G + off[T_G2], G + off[T_BE2], G + off[T_B2], M, H));
  else
    L2L_TRY(ln_bwd<T>(c, dydx, c->r2, own_stats ? nullptr : c->mean2, own_stats ? nullptr : c->rstd2, P + off[T_G2], c->dr2,
                      G + off[T_G2], G + off[T_BE2], G + off[T_B2], M, H, f.ln_eps));
  // FFN2 backward: dU1 = (dR2 W2^T) * gelu'(U1); dW2 += G^T dR2 (db2 came with LN2's backward)
  {
    GemmArgs g = gemm_args((int)M, F, H, c->dr2, H, 1, P + off[T_W2], H, 1, c->du1, F);
    g.epi = EPI_MULAUX; g.aux = c->u1; g.ldaux = F;   // u1 holds gelu'(U1), kept by the recompute pass
    // db1 = colsum(dU1) comes out of this GEMM's epilogue where it can: one row of partial sums per 128 rows of dU1,
    // added up by the column-sum kernel (256 x F floats instead of M x F elements)
    int ws_rows = 0;
    g.colsum = c->colsum_ws;
    db1_in_gemm = c->colsum_ws && colsum_in_gemm_ok(dt, false, g, &ws_rows) && (size_t)ws_rows * F <= c->colsum_ws_elems;
    if (db1_in_gemm) g.epi |= EPI_COLSUM; else g.colsum = nullptr;
    L2L_TRY(gemm(c, dt, false, g));
    if (db1_in_gemm) L2L_TRY(bias_grad<float>(c, c->colsum_ws, F, G + off[T_B1], ws_rows, F));
    GemmArgs w = gemm_args(F, H, (int)M, c->ga, F, 0, c->dr2, H, 0, G + off[T_W2], H);
    w.epi = EPI_ACCUM;
    L2L_TRY(gemm(c, dt, true, w));
  }
  // FFN1 backward: dY1 = dR2 + dU1 W1^T; dW1 += Y1^T dU1; db1 += colsum(dU1)
  {
    GemmArgs g = gemm_args((int)M, H, F, c->du1, F, 1, P + off[T_W1], F, 1, c->dy1, H);
    g.epi = EPI_RESID; g.resid = c->dr2; g.ldr = H;
    L2L_TRY(gemm(c, dt, false, g));
    GemmArgs w = gemm_args(H, F, (int)M, c->y1, H, 0, c->du1, F, 0, G + off[T_W1], F);
    w.epi = EPI_ACCUM;
    L2L_TRY(gemm(c, dt, true, w));
    if (!db1_in_gemm) L2L_TRY(bias_grad<T>(c, c->du1, F, G + off[T_B1], M, F));
  }
  // LN1 backward
  L2L_TRY(ln_bwd<T>(c, c->dy1, c->r1, c->mean1, c->rstd1, P + off[T_G1], c->dr1, G + off[T_G1], G + off[T_BE1], G + off[T_BO], M, H, f.ln_eps));
  // output projection backward
  {
    GemmArgs g = gemm_args((int)M, H, H, c->dr1, H, 1, P + off[T_WO], H, 1, c->dc, H);
    L2L_TRY(gemm(c, dt, false, g));
    GemmArgs w = gemm_args(H, H, (int)M, c->c, H, 0, c->dr1, H, 0, G + off[T_WO], H);
    w.epi = EPI_ACCUM;
    L2L_TRY(gemm(c, dt, true, w));
  }
  // attention backward per (sequence, head)
  // The bias gradient of the QKV projection is colsum(dQKV).  With the fused kernel it does not take a pass over dQKV:
  // the Q part comes out of the kernel (one row of partial sums per 32 queries), the V part equals colsum(dC) because
  // every row of P sums to one, and the K part is zero because every row of dS sums to zero (a bias on the keys
  // shifts all scores of a query alike, which the softmax does not see).
  bool dbqkv_done = false;
  if (fused_attention_ok(c)) {
    const long long part_rows = (long long)nseq * (S / 32);
    float* dq_part = c->colsum_ws && (size_t)part_rows * H <= c->colsum_ws_elems ? c->colsum_ws : nullptr;
    const double fl = 10.0 * S * S * d * nseq * A;
    L2L_TRY(timed(c, L2L_PROF_ATTN, fl, (3.0 + 1.0 + 3.0) * M * H * sizeof(T), [&] {
      using E = attn_elem<T>;
      hipLaunchKernelGGL(attn::attn_bwd_kernel<E>, dim3(nseq * A), dim3(256), attn::BWD_LDS, c->cs, (const E*)qkv,
                         (const E*)c->dc, (E*)dqkv, dq_part, S, H, A, alpha);
    }));
    if (dq_part) {
      L2L_TRY(bias_grad<float>(c, dq_part, H, G + off[T_BQKV], part_rows, H));
      L2L_TRY(bias_grad<T>(c, c->dc, H, G + off[T_BQKV] + 2 * H, M, H));
      dbqkv_done = true;
    }
  } else if (fused_attention_long_ok(c)) {
    using E = attn_elem<T>;
    const dim3 grid(nseq * A * ((S + attn::CH - 1) / attn::CH));
    L2L_TRY(timed(c, L2L_PROF_ATTN, 4.0 * S * S * d * nseq * A, (3.0 + 1.0 + 1.0 + 1.0) * M * H * sizeof(T), [&] {
      auto go = [&](auto kern) {
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, c->cs, (const E*)qkv, (const E*)c->dc, (const E*)c->c, c->lse, c->dsum,
                           (E*)dqkv, S, H, A, alpha);
      };
      if (S % attn::CH) go(attn::attn_bwd_dq_long_kernel<E, true>); else go(attn::attn_bwd_dq_long_kernel<E, false>);
    }));
    L2L_TRY(timed(c, L2L_PROF_ATTN, 6.0 * S * S * d * nseq * A, (3.0 + 1.0 + 2.0) * M * H * sizeof(T), [&] {
      auto go = [&](auto kern) {
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, c->cs, (const E*)qkv, (const E*)c->dc, c->lse, c->dsum, (E*)dqkv, S, H, A,
                           alpha);
      };
      if (S % attn::CH) go(attn::attn_bwd_dkv_long_kernel<E, true>); else go(attn::attn_bwd_dkv_long_kernel<E, false>);
    }));
  } else
  {
    const long long zq = (long long)S * 3 * H, zp = (long long)A * S * S, zc = (long long)S * H;
    auto batch = [&](GemmArgs& g, long long azo, long long azi, long long bzo, long long bzi, long long czo, long long czi) {
      g.nbatch = nseq * A; g.zdiv = A;
      g.a_zo = azo; g.a_zi = azi; g.b_zo = bzo; g.b_zi = bzi; g.c_zo = czo; g.c_zi = czi;
    };
    // dV = P^T dC
    GemmArgs g1 = gemm_args(S, d, S, c->p, S, 0, c->dc, H, 0, dqkv + 2 * H, 3 * H);
    batch(g1, zp, (long long)S * S, zc, d, zq, d);
    L2L_TRY(gemm(c, dt, false, g1, 0, L2L_PROF_ATTN));
    // dP = dC V^T
    GemmArgs g2 = gemm_args(S, S, d, c->dc, H, 1, qkv + 2 * H, 3 * H, 1, c->dp, S);
    batch(g2, zc, d, zq, d, zp, (long long)S * S);
    L2L_TRY(gemm(c, dt, false, g2, 0, L2L_PROF_ATTN));
    // dS = P * (dP - rowsum(dP * P)), in place
    const long long rows = (long long)nseq * A * S;
    L2L_TRY(timed(c, L2L_PROF_ATTN, 0, 3.0 * rows * S * sizeof(T), [&] {
      hipLaunchKernelGGL(softmax_bwd_kernel<T>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, c->cs, (const T*)c->p, (T*)c->dp,
                         rows, S);
    }));
    // dQ = dS K / sqrt(d)
    GemmArgs g3 = gemm_args(S, d, S, c->dp, S, 1, qkv + H, 3 * H, 0, dqkv, 3 * H);
    batch(g3, zp, (long long)S * S, zq, d, zq, d);
    g3.alpha = alpha;
    L2L_TRY(gemm(c, dt, false, g3, 0, L2L_PROF_ATTN));
    // dK = dS^T Q / sqrt(d)
    GemmArgs g4 = gemm_args(S, d, S, c->dp, S, 0, qkv, 3 * H, 0, dqkv + H, 3 * H);
    batch(g4, zp, (long long)S * S, zq, d, zq, d);
    g4.alpha = alpha;
    L2L_TRY(gemm(c, dt, false, g4, 0, L2L_PROF_ATTN));
  }
  // QKV projection backward: dX = dR1 + dQKV Wqkv^T (over dY in place); dWqkv += X^T dQKV
  {
    GemmArgs g = gemm_args((int)M, H, 3 * H, dqkv, 3 * H, 1, P + off[T_WQKV], 3 * H, 1, dydx, H);
    g.epi = EPI_RESID; g.resid = c->dr1; g.ldr = H;
    L2L_TRY(gemm(c, dt, false, g));
    GemmArgs w = gemm_args(H, 3 * H, (int)M, x, H, 0, dqkv, 3 * H, 0, G + off[T_WQKV], 3 * H);
    w.epi = EPI_ACCUM;
    L2L_TRY(gemm(c, dt, true, w));
    if (!dbqkv_done) L2L_TRY(bias_grad<T>(c, dqkv, 3 * H, G + off[T_BQKV], M, 3 * H));
  }
  return L2L_OK;
}

template <typename T>
int embed_fwd_t(l2l_ctx* c, const int32_t* tokens, void* x_out) {
  const long long rows = c->T * c->cfg.num_ubatches;
  const T* E = (const T*)c->emb;
  const long long* eo = c->lay.eoff;
  const int H = c->cfg.hidden;
  return timed(c, L2L_PROF_ROWWISE, 0, 2.0 * rows * H * sizeof(T), [&] {
    hipLaunchKernelGGL(embed_fwd_kernel<T>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, c->cs, tokens, E + eo[E_E],
                       E + eo[E_P], E + eo[E_GE], E + eo[E_BE], (T*)x_out, c->emean, c->erstd, (int)rows, c->cfg.seq, H,
                       c->cfg.ln_eps, c->cfg.vocab, c->bad_ids);
  });
}

template <typename T>
int head_loss_t(l2l_ctx* c, const void* x_last, const int32_t* labels, void* dy_out, float* loss_out) {
  const l2l_config& f = c->cfg;
  const int H = f.hidden, V = f.vocab, U = f.num_ubatches, dt = f.dtype;
  const int Tn = (int)c->T;
  const long long Vp = c->Vp;
  const T* E = (const T*)c->emb;
  const long long* eo = c->lay.eoff;
  const long long UT = (long long)U * Tn, RC = c->head_rows;
  const int nchunks = (int)((UT + RC - 1) / RC);
  L2L_TRY(fill_zero(c, c->lab_cnt, (U + 1) * 4));
  L2L_TRY(fill_zero(c, loss_out, 4));
  L2L_TRY(fill_zero(c, dy_out, (size_t)UT * H * sizeof(T)));
  L2L_TRY(timed(c, L2L_PROF_OTHER, 0, 4.0 * UT, [&] {
    hipLaunchKernelGGL(label_compact_kernel, dim3(U), dim3(256), 0, c->cs, labels, Tn, c->lab_idx, c->lab_cnt, c->lab_total);
  }));
  L2L_TRY(timed(c, L2L_PROF_OTHER, 0, 0, [&] {
    hipLaunchKernelGGL(label_merge_kernel, dim3(U), dim3(256), 0, c->cs, c->lab_idx, c->lab_cnt, Tn, c->lab_gidx, c->chunk_cnt,
                       (int)RC, nchunks);
  }));
  // The labelled rows of the whole mini-batch, RC at a time (one pass at the usual masking rates): the
  // vocabulary GEMMs then have enough rows to fill the chip, and E is read once per pass, not once per
  // micro-batch.  Passes beyond the labelled count find a zero in chunk_cnt and do nothing.
  for (int ch = 0; ch < nchunks; ++ch) {
    const int32_t* idx = c->lab_gidx + (long long)ch * RC;
    const int32_t* cnt = c->chunk_cnt + ch;
    const int rows = (int)std::min<long long>(RC, UT - (long long)ch * RC);
    L2L_TRY(timed(c, L2L_PROF_OTHER, 0, 0, [&] {
      hipLaunchKernelGGL((rows_by_index_kernel<T, false>), dim3((rows + 3) / 4), dim3(256), 0, c->cs, (const T*)x_last, (T*)c->xl,
                         idx, cnt, H);
    }));
    // logits = Xl E^T + bv.  The GEMM runs over the padded vocabulary Vp (a multiple of 64; the logits buffer has that
    // many columns) so that its epilogue takes the 16-byte path, which wants N % 8 == 0: columns V .. Vp - 1 come from
    // the rows that follow E in the embedding block and from the bias tensor's padding, and nobody reads them.
    GemmArgs g = gemm_args(rows, (int)Vp, H, c->xl, H, 1, E + eo[E_E], H, 1, c->logits, Vp);
    g.epi = EPI_BIAS; g.bias = E + eo[E_BV]; g.m_dev = cnt;
    L2L_TRY(gemm(c, dt, true, g, 0, L2L_PROF_OTHER));
    L2L_TRY(timed(c, L2L_PROF_OTHER, 0, 0, [&] {
      hipLaunchKernelGGL(ce_kernel<T>, dim3(rows), dim3(256), 0, c->cs, c->logits, Vp, labels, idx, cnt, c->lab_total, (T*)c->dz,
                         loss_out, V, (int)Vp, c->loss_scale, c->bad_ids);
    }));
    // dXl = dz E
    if constexpr (sizeof(T) == 2) {
      // few tiles (rows x H) and a long contraction (the vocabulary): as an accumulating fp32 GEMM into a cleared
      // buffer it is split over K like the dW GEMMs, and rounded to the 16-bit format afterwards
      L2L_TRY(fill_zero(c, c->dxl32, (size_t)rows * H * 4));
      GemmArgs h = gemm_args(rows, H, V, c->dz, Vp, 1, E + eo[E_E], H, 0, c->dxl32, H);
      h.m_dev = cnt;
      h.epi = EPI_ACCUM;
      L2L_TRY(gemm(c, dt, true, h, 0, L2L_PROF_OTHER));
      const long long n = (long long)rows * H;
      L2L_TRY(timed(c, L2L_PROF_OTHER, 0, 6.0 * n, [&] {
        const unsigned blocks = (unsigned)std::min<long long>((n / 4 + 255) / 256 + 1, 2048);
        hipLaunchKernelGGL(narrow_kernel<T>, dim3(blocks), dim3(256), 0, c->cs, c->dxl32, (T*)c->dxl, n);
      }));
    } else {
      GemmArgs h = gemm_args(rows, H, V, c->dz, Vp, 1, E + eo[E_E], H, 0, c->dxl, H);
      h.m_dev = cnt;
      L2L_TRY(gemm(c, dt, false, h, 0, L2L_PROF_OTHER));
    }
    L2L_TRY(timed(c, L2L_PROF_OTHER, 0, 0, [&] {
      hipLaunchKernelGGL((rows_by_index_kernel<T, true>), dim3((rows + 3) / 4), dim3(256), 0, c->cs, (const T*)c->dxl, (T*)dy_out,
                         idx, cnt, H);
    }));
    // dE += dz^T Xl ; dbv += colsum(dz)
    GemmArgs w = gemm_args(V, H, rows, c->dz, Vp, 0, c->xl, H, 0, c->egacc + eo[E_E], H);
    w.epi = EPI_ACCUM; w.k_dev = cnt;
    L2L_TRY(gemm(c, dt, true, w, 0, L2L_PROF_OTHER));
    L2L_TRY(bias_grad<T>(c, c->dz, Vp, c->egacc + eo[E_BV], rows, V, cnt));
  }
  return L2L_OK;
}

template <typename T>
int embed_bwd_t(l2l_ctx* c, const int32_t* tokens, const void* dy) {
  const long long rows = c->T * c->cfg.num_ubatches;
  const T* E = (const T*)c->emb;
  const long long* eo = c->lay.eoff;
  const int H = c->cfg.hidden, S = c->cfg.seq;
  L2L_TRY(timed(c, L2L_PROF_ROWWISE, 0, 0, [&] {
    const unsigned nseq = (unsigned)(rows / S);
    const bool turned = (size_t)5 * H * sizeof(float) <= (size_t)128 << 10;   // room for a row per wave in LDS
    const size_t lds = (size_t)(turned ? 5 : 1) * H * sizeof(float);
    static_cast<void>(hipFuncSetAttribute((const void*)embed_bwd_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(embed_bwd_kernel<T>, dim3((unsigned)S * ((nseq + EMB_SEQS - 1) / EMB_SEQS)), dim3(256), lds, c->cs, tokens, E + eo[E_E], E + eo[E_P],
                       E + eo[E_GE], (const T*)dy, c->emean, c->erstd, c->egacc + eo[E_E], c->egacc + eo[E_P], (int)rows, S, H, turned, c->cfg.vocab);
  }));
  return timed(c, L2L_PROF_COLSUM, 0, 0, [&] {
    const int rpb = colsum_rows_per_block(rows, H);
    dim3 grid((H + 127) / 128, (unsigned)((rows + rpb - 1) / rpb));
    hipLaunchKernelGGL((colsum_kernel<T, 2>), grid, dim3(256), 0, c->cs, (const T*)dy, (long long)H, (const T*)nullptr, c->emean,
                       c->erstd, tokens, E + eo[E_E], E + eo[E_P], S, c->egacc + eo[E_GE], c->egacc + eo[E_BE], (int)rows, H,
                       (const int*)nullptr, c->cfg.vocab, rpb);
  });
}

// Sequence-classification head, forward and backward over all sequences of the mini-batch: pooled = tanh(x0 Wp + bp),
// z = pooled Wc + bc, cross-entropy over the labelled sequences; gradients of the four tensors into cls_g, dL/dx into
// the first-token rows of dy_out (zero elsewhere).
template <typename T>
int cls_head_t(l2l_ctx* c, const void* x_last, const int32_t* seq_labels, void* dy_out, float* loss_out) {
  const l2l_config& f = c->cfg;
  const int H = f.hidden, S = f.seq, C = c->cls_classes, dt = f.dtype;
  const int nseq = f.ubatch * f.num_ubatches;
  const int Cp = (int)c->cls_cp;
  const T* W = (const T*)c->cls_w;
  const long long* o = c->cls_off;
  float* G = c->cls_g;
  const unsigned rb = (unsigned)((nseq + 3) / 4);
  L2L_TRY(fill_zero(c, dy_out, (size_t)nseq * S * H * sizeof(T)));
  L2L_TRY(timed(c, L2L_PROF_OTHER, 0, 0, [&] {
    hipLaunchKernelGGL((first_token_rows_kernel<T, false>), dim3(rb), dim3(256), 0, c->cs, (const T*)x_last, (T*)c->cls_x, nseq, S, H);
  }));
  GemmArgs g = gemm_args(nseq, H, H, c->cls_x, H, 1, W + o[C_WP], H, 0, c->cls_u, H);
  g.epi = EPI_BIAS; g.bias = W + o[C_BP];
  L2L_TRY(gemm(c, dt, false, g, 0, L2L_PROF_OTHER));
  const long long ne = (long long)nseq * H;
  const unsigned eb = (unsigned)((ne / 8 + 255) / 256);
  L2L_TRY(timed(c, L2L_PROF_OTHER, 0, 0, [&] {
    hipLaunchKernelGGL((tanh_kernel<T, false>), dim3(eb), dim3(256), 0, c->cs, (const T*)c->cls_u, (const T*)nullptr, (T*)c->cls_p, ne);
  }));
  GemmArgs z = gemm_args(nseq, C, H, c->cls_p, H, 1, W + o[C_WC], C, 0, c->cls_z, Cp);
  z.epi = EPI_BIAS; z.bias = W + o[C_BC];
  L2L_TRY(gemm(c, dt, true, z, 0, L2L_PROF_OTHER));
  L2L_TRY(timed(c, L2L_PROF_OTHER, 0, 0, [&] {
    hipLaunchKernelGGL(cls_ce_kernel<T>, dim3(1), dim3(256), 0, c->cs, c->cls_z, Cp, seq_labels, (T*)c->cls_dz, loss_out, nseq, C,
                       c->loss_scale, c->bad_ids);
  }));
  // dWc += pooled^T dz ; dbc += colsum(dz) ; dpooled = dz Wc^T
  GemmArgs wc = gemm_args(H, C, nseq, c->cls_p, H, 0, c->cls_dz, Cp, 0, G + o[C_WC], C);
  wc.epi = EPI_ACCUM;
  L2L_TRY(gemm(c, dt, true, wc, 0, L2L_PROF_OTHER));
  L2L_TRY(bias_grad<T>(c, c->cls_dz, Cp, G + o[C_BC], nseq, C, nullptr));
  GemmArgs dp = gemm_args(nseq, H, C, c->cls_dz, Cp, 1, W + o[C_WC], C, 1, c->cls_dp, H);
  L2L_TRY(gemm(c, dt, false, dp, 0, L2L_PROF_OTHER));
  L2L_TRY(timed(c, L2L_PROF_OTHER, 0, 0, [&] {
    hipLaunchKernelGGL((tanh_kernel<T, true>), dim3(eb), dim3(256), 0, c->cs, (const T*)c->cls_dp, (const T*)c->cls_p, (T*)c->cls_du, ne);
  }));
  // dWp += x0^T du ; dbp += colsum(du) ; dx0 = du Wp^T
  GemmArgs wp = gemm_args(H, H, nseq, c->cls_x, H, 0, c->cls_du, H, 0, G + o[C_WP], H);
  wp.epi = EPI_ACCUM;
  L2L_TRY(gemm(c, dt, true, wp, 0, L2L_PROF_OTHER));
  L2L_TRY(bias_grad<T>(c, c->cls_du, H, G + o[C_BP], nseq, H, nullptr));
  GemmArgs dx = gemm_args(nseq, H, H, c->cls_du, H, 1, W + o[C_WP], H, 1, c->cls_dx, H);
  L2L_TRY(gemm(c, dt, false, dx, 0, L2L_PROF_OTHER));
  return timed(c, L2L_PROF_OTHER, 0, 0, [&] {
    hipLaunchKernelGGL((first_token_rows_kernel<T, true>), dim3(rb), dim3(256), 0, c->cs, (const T*)c->cls_dx, (T*)dy_out, nseq, S, H);
  });
}

int check_slot_call(l2l_ctx* c, int layer, int slot, const void* a, const void* b, const char* who) {
  if (!c) return L2L_E_ARG;
  if (!a || !b) return fail(c, L2L_E_ARG, "%s: null pointer", who);
  if (layer < 0) return fail(c, L2L_E_ARG, "%s: layer %d < 0", who, layer);
  if (slot != 0 && slot != 1) return fail(c, L2L_E_ARG, "%s: slot %d not 0 or 1", who, slot);
  if (c->slot_layer[slot] != layer)
    return fail(c, L2L_E_STATE, "%s: slot %d holds layer %d, not layer %d (stage it first)", who, slot, c->slot_layer[slot], layer);
  return L2L_OK;
}

}  // namespace

// ================================================================================================
// public API
// ================================================================================================
extern "C" {

int l2l_create(const l2l_config* cfg, void* compute_stream, void* copy_stream, l2l_ctx** out) {
  if (!out) return L2L_E_ARG;
  *out = nullptr;
  if (!config_ok(cfg)) return L2L_E_ARG;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
    (void)hipGetLastError();
    return L2L_E_HIP;
  }
  l2l_ctx* c = new l2l_ctx;
  c->cfg = *cfg;
  c->lay = make_layout(cfg);
  c->cs = (hipStream_t)compute_stream;
  c->xs = (hipStream_t)copy_stream;
  c->T = (long long)cfg->ubatch * cfg->seq;
  int g = cfg->ubatch_group;
  if (g == 0) {  // default: as many micro-batches per launch as keep a launch within 32768 rows and its widest
    g = 1;       // activation below the 2 GiB that the MFMA kernels' 32-bit operand addressing covers
    const long long widest = std::max<long long>(cfg->ffn, 3LL * cfg->hidden) * 2;
    for (int k = 1; k <= cfg->num_ubatches; ++k)
      if (cfg->num_ubatches % k == 0 && k * c->T <= 32768 && k * c->T * widest < (1LL << 31)) g = k;
  }
  // attention launches batch (sequence, head) pairs along grid z
  while (g > 1 && (long long)g * cfg->ubatch * cfg->heads > 65535) --g;
  if ((long long)cfg->ubatch * cfg->heads > 65535) {
    delete c;
    return L2L_E_ARG;
  }
  c->group = g;
  c->Mg = g * c->T;
  // the switches of the environment are read here, once, and nowhere else
  if (const char* e = getenv("L2L_NO_FUSED_ATTENTION")) c->no_fused_attention = atoi(e) != 0;
  if (const char* e = getenv("L2L_COPY_ROWS")) c->copy_rows = atoi(e) != 0;
  if (const char* e = getenv("L2L_NO_WEIGHT_TRANSPOSE")) c->no_weight_transpose = atoi(e) != 0;
  if (const char* e = getenv("L2L_FORCE_SPLITS")) c->force_splits = std::max(0, atoi(e));
  if (const char* e = getenv("L2L_SPLIT_ATOMICS")) c->split_atomics = atoi(e) != 0;
  {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 0;
    (void)hipGetLastError();
    c->resident_cus = n;
    if (const char* e = getenv("L2L_GEMM_RESIDENT")) if (atoi(e) == 0) c->resident_cus = 0;
  }
  (void)hipFuncSetAttribute((const void*)attn::attn_bwd_kernel<bf16>, hipFuncAttributeMaxDynamicSharedMemorySize, attn::BWD_LDS);
  (void)hipFuncSetAttribute((const void*)attn::attn_bwd_kernel<fp16>, hipFuncAttributeMaxDynamicSharedMemorySize, attn::BWD_LDS);
  *out = c;  // from here on the caller can read l2l_last_error and must l2l_destroy

  const size_t es = esize(cfg->dtype);
  const long long H = cfg->hidden, F = cfg->ffn, S = cfg->seq, A = cfg->heads, Mg = c->Mg;
  // the attention matrices P and dP exist in memory only on the batched-GEMM path
  const bool fused = fused_attention_ok(c) || fused_attention_long_ok(c);
  const long long pe = fused ? 0 : (long long)g * cfg->ubatch * A * S * S;
  for (int i = 0; i < 2; ++i) {
    L2L_TRY(dev_alloc(c, &c->slot[i], c->lay.total * es));
    L2L_TRY(dev_alloc(c, (void**)&c->gacc[i], c->lay.total * 4));
    HIP_TRY(c, hipMemset(c->gacc[i], 0, c->lay.total * 4));
    HIP_TRY(c, hipEventCreateWithFlags(&c->slot_staged[i], hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->slot_released[i], hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->gacc_ready[i], hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->gacc_drained[i], hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->gacc_landed[i], hipEventDisableTiming));
  }
  struct { void** p; long long n; } bufs[] = {
      {&c->qkv, Mg * 3 * H}, {&c->p, pe}, {&c->c, Mg * H}, {&c->r1, Mg * H}, {&c->y1, Mg * H}, {&c->u1, Mg * F},
      {&c->ga, Mg * F}, {&c->r2, Mg * H}, {&c->dr2, Mg * H}, {&c->du1, Mg * F}, {&c->dy1, Mg * H}, {&c->dr1, Mg * H},
      {&c->dc, Mg * H}, {&c->dp, pe}, {&c->dqkv, Mg * 3 * H}, {&c->ytmp, Mg * H}};
  for (auto& b : bufs) L2L_TRY(dev_alloc(c, b.p, b.n * es));
  if (is16(cfg->dtype) && !c->no_weight_transpose)
    for (int i = 0; i < 2; ++i) L2L_TRY(dev_alloc(c, &c->wt[i], c->lay.total * es));
  if (is16(cfg->dtype)) {   // workspace of the K-split dW GEMMs: the largest of the layer's four, by the split rule in use
    size_t need = 0;
    const int h = cfg->hidden, f = cfg->ffn;
    const int shapes[4][2] = {{h, 3 * h}, {h, h}, {h, f}, {f, h}};
    for (const auto& s : shapes) {
      GemmArgs w = gemm_args(s[0], s[1], (int)Mg, nullptr, s[0], 0, nullptr, s[1], 0, nullptr, s[1]);
      w.epi = EPI_ACCUM;
      int v, splits;
      pick_tile(w, true, &v, &splits);
      if (splits > 1) need = std::max(need, (size_t)splits * s[0] * s[1]);
    }
    if (const char* e = getenv("L2L_SPLIT_WS_MB")) need = (size_t)atoll(e) << 18;   // tuning: room for other split factors
    if (need > 0 && need * 4 <= (size_t)256 << 20) {
      c->split_ws_elems = need;
      L2L_TRY(dev_alloc(c, (void**)&c->split_ws, need * 4));
    }
  }
  if (is16(cfg->dtype)) {   // partial column sums out of a GEMM epilogue: one row per 64 rows of the group at most
    c->colsum_ws_elems = (size_t)((Mg + 63) / 64) * std::max(F, 3 * H);
    L2L_TRY(dev_alloc(c, (void**)&c->colsum_ws, c->colsum_ws_elems * 4));
  }
  L2L_TRY(dev_alloc(c, (void**)&c->bad_ids, 4));
  HIP_TRY(c, hipMemset(c->bad_ids, 0, 4));
  float** stats[] = {&c->mean1, &c->rstd1, &c->mean2, &c->rstd2};
  for (auto s : stats) L2L_TRY(dev_alloc(c, (void**)s, Mg * 4));
  if (fused_attention_long_ok(c)) {   // per (sequence, head, query): log-sum-exp of the scores, rowsum(dO O)
    L2L_TRY(dev_alloc(c, (void**)&c->lse, Mg * A * 4));
    L2L_TRY(dev_alloc(c, (void**)&c->dsum, Mg * A * 4));
  }

  if (cfg->vocab > 0) {
    const long long V = cfg->vocab, UT = c->T * cfg->num_ubatches;
    c->Vp = up(V, 64);
    // (+ 64 rows: the logits GEMM reads the rows of E up to the padded vocabulary size, wherever the block ends)
    L2L_TRY(dev_alloc(c, &c->emb, (c->lay.etotal + 64 * (long long)cfg->hidden) * es));
    HIP_TRY(c, hipMemset(c->emb, 0, (c->lay.etotal + 64 * (long long)cfg->hidden) * es));
    L2L_TRY(dev_alloc(c, (void**)&c->egacc, c->lay.etotal * 4));
    HIP_TRY(c, hipMemset(c->egacc, 0, c->lay.etotal * 4));
    L2L_TRY(dev_alloc(c, (void**)&c->emean, UT * 4));
    L2L_TRY(dev_alloc(c, (void**)&c->erstd, UT * 4));
    L2L_TRY(dev_alloc(c, (void**)&c->lab_idx, UT * 4));
    L2L_TRY(dev_alloc(c, (void**)&c->lab_cnt, (cfg->num_ubatches + 1) * 4));
    c->lab_total = c->lab_cnt + cfg->num_ubatches;
    c->head_rows = std::min<long long>(UT, 8192);
    if (const char* e = getenv("L2L_HEAD_ROWS"))   // smaller passes, for tests of the multi-pass path
      if (atoll(e) > 0) c->head_rows = std::min<long long>(UT, atoll(e));
    L2L_TRY(dev_alloc(c, (void**)&c->lab_gidx, UT * 4));
    L2L_TRY(dev_alloc(c, (void**)&c->chunk_cnt, ((UT + c->head_rows - 1) / c->head_rows) * 4));
    L2L_TRY(dev_alloc(c, &c->xl, c->head_rows * H * es));
    L2L_TRY(dev_alloc(c, &c->dxl, c->head_rows * H * es));
    if (is16(cfg->dtype)) L2L_TRY(dev_alloc(c, (void**)&c->dxl32, c->head_rows * H * 4));
    L2L_TRY(dev_alloc(c, (void**)&c->logits, c->head_rows * c->Vp * 4));
    L2L_TRY(dev_alloc(c, &c->dz, c->head_rows * c->Vp * es));
    HIP_TRY(c, hipEventCreateWithFlags(&c->emb_staged_ev, hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->emb_released_ev, hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->egacc_ready, hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->egacc_drained, hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->egacc_landed, hipEventDisableTiming));
  }
  return L2L_OK;
}

int l2l_destroy(l2l_ctx* c) {
  if (!c) return L2L_E_ARG;
  (void)hipDeviceSynchronize();
  for (void* p : c->allocs) (void)hipFree(p);
  for (auto& r : c->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  for (auto e : c->ev_pool) (void)hipEventDestroy(e);
  hipEvent_t evs[] = {c->slot_staged[0], c->slot_staged[1], c->slot_released[0], c->slot_released[1], c->gacc_ready[0],
                      c->gacc_ready[1], c->gacc_drained[0], c->gacc_drained[1], c->gacc_landed[0], c->gacc_landed[1], c->egacc_landed, c->emb_staged_ev, c->emb_released_ev,
                      c->egacc_ready, c->egacc_drained, c->cls_staged_ev, c->cls_released_ev, c->cls_ready, c->cls_landed, c->cls_drained,
                      c->prof_base};
  for (hipEvent_t e : evs)
    if (e) (void)hipEventDestroy(e);
  delete c;
  return L2L_OK;
}

size_t l2l_device_bytes(const l2l_ctx* c) { return c ? c->dev_bytes : 0; }
const char* l2l_last_error(const l2l_ctx* c) { return c ? c->err : "null context"; }

int l2l_sync(l2l_ctx* c) {
  if (!c) return L2L_E_ARG;
  HIP_TRY(c, hipStreamSynchronize(c->cs));
  HIP_TRY(c, hipStreamSynchronize(c->xs));
  if (c->bad_ids) {   // set by the embedding and loss kernels, which clamp such ids instead of following them
    int32_t bad = 0;
    HIP_TRY(c, hipMemcpy(&bad, c->bad_ids, 4, hipMemcpyDeviceToHost));
    if (bad) {
      HIP_TRY(c, hipMemset(c->bad_ids, 0, 4));
      return fail(c, L2L_E_ARG, "a token id or label outside its range (vocabulary %d, or the head's classes) was passed since the last l2l_sync; such ids are clamped and the results are not meaningful",
                  c->cfg.vocab);
    }
  }
  return L2L_OK;
}

int l2l_param_stage(l2l_ctx* c, int layer, const void* host_params, int slot) {
  if (!c) return L2L_E_ARG;
  if (!host_params) return fail(c, L2L_E_ARG, "l2l_param_stage: null host pointer");
  if (layer < 0) return fail(c, L2L_E_ARG, "l2l_param_stage: layer %d < 0", layer);
  if (slot != 0 && slot != 1) return fail(c, L2L_E_ARG, "l2l_param_stage: slot %d not 0 or 1", slot);
  // the copy may start only when every kernel that reads the slot's previous contents is done
  if (c->slot_layer[slot] >= 0) HIP_TRY(c, hipStreamWaitEvent(c->xs, c->slot_released[slot], 0));
  const CopyMark mark = copy_begin(c);
  HIP_TRY(c, hipMemcpyAsync(c->slot[slot], host_params, c->lay.total * esize(c->cfg.dtype), hipMemcpyHostToDevice, c->xs));
  L2L_TRY(transpose_weights(c, slot));
  copy_end(c, mark, (double)c->lay.total * esize(c->cfg.dtype));
  HIP_TRY(c, hipEventRecord(c->slot_staged[slot], c->xs));
  c->slot_layer[slot] = layer;
  return L2L_OK;
}

static int layer_fwd_impl(l2l_ctx* c, int layer, int slot, const void* x_stash, void* y_out, float* rstd_out) {
  L2L_TRY(check_slot_call(c, layer, slot, x_stash, y_out, "l2l_layer_fwd"));
  HIP_TRY(c, hipStreamWaitEvent(c->cs, c->slot_staged[slot], 0));
  const size_t es = esize(c->cfg.dtype);
  const int U = c->cfg.num_ubatches;
  for (int u0 = 0; u0 < U; u0 += c->group) {
    const int ng = std::min(c->group, U - u0);
    const size_t o = (size_t)u0 * c->T * c->cfg.hidden * es;
    const void* x = (const char*)x_stash + o;
    void* y = (char*)y_out + o;
    float* rs = rstd_out ? rstd_out + (size_t)u0 * c->T : nullptr;
    if (c->cfg.dtype == L2L_BF16) L2L_TRY(layer_forward_group<bf16>(c, slot, x, y, ng, false, rs));
    else if (c->cfg.dtype == L2L_FP16) L2L_TRY(layer_forward_group<fp16>(c, slot, x, y, ng, false, rs));
    else L2L_TRY(layer_forward_group<float>(c, slot, x, y, ng, false, rs));
  }
  HIP_TRY(c, hipEventRecord(c->slot_released[slot], c->cs));
  return L2L_OK;
}

int l2l_layer_fwd(l2l_ctx* c, int layer, int slot, const void* x_stash, void* y_out) {
  return layer_fwd_impl(c, layer, slot, x_stash, y_out, nullptr);
}

int l2l_layer_fwd_stats(l2l_ctx* c, int layer, int slot, const void* x_stash, void* y_out, float* rstd_out) {
  if (c && !rstd_out) return fail(c, L2L_E_ARG, "l2l_layer_fwd_stats: null pointer");
  return layer_fwd_impl(c, layer, slot, x_stash, y_out, rstd_out);
}

static int layer_bwd_impl(l2l_ctx* c, int layer, int slot, const void* x_stash, void* dy_dx, const void* y_stash, const float* rstd) {
  L2L_TRY(check_slot_call(c, layer, slot, x_stash, dy_dx, "l2l_layer_bwd"));
  // the shortcut through the stashed output needs the one-pass LayerNorm backward kernel; wider rows recompute in full
  const bool from_y = y_stash && rstd && ln_bwd_one_pass(c->cfg.hidden);
  const int a = c->gacc_next;
  if (c->gacc_state[a] == 1)
    return fail(c, L2L_E_STATE, "l2l_layer_bwd: gradients of layer %d were never drained", c->gacc_layer[a]);
  HIP_TRY(c, hipStreamWaitEvent(c->cs, c->slot_staged[slot], 0));
  if (c->gacc_state[a] == 2) HIP_TRY(c, hipStreamWaitEvent(c->cs, c->gacc_drained[a], 0));
  float* G = c->gacc[a];   // zero: cleared at creation and again, on the copy stream, after every drain
  const size_t es = esize(c->cfg.dtype);
  const int U = c->cfg.num_ubatches;
  for (int u0 = 0; u0 < U; u0 += c->group) {
    const int ng = std::min(c->group, U - u0);
    const size_t o = (size_t)u0 * c->T * c->cfg.hidden * es;
    const void* x = (const char*)x_stash + o;
    void* dy = (char*)dy_dx + o;
    const void* y = from_y ? (const char*)y_stash + o : nullptr;
    const float* rs = from_y ? rstd + (size_t)u0 * c->T : nullptr;
    // With the stashed output in hand LayerNorm 2's backward goes first: the recompute pass ends with the FFN1 GEMM,
    // whose 2 M F elements of output are still on their way to memory when the next kernel starts; a GEMM after it
    // does not notice, a kernel bound by memory does (measured: LayerNorm 2's backward 70 us behind that GEMM, 45 us
    // in front of the recompute pass).
    if (c->cfg.dtype == L2L_BF16) {
      if (from_y) L2L_TRY(layer_ln2_backward_from_y<bf16>(c, c->slot[slot], dy, G, ng, y, rs));
      L2L_TRY(layer_forward_group<bf16>(c, slot, x, nullptr, ng, true, nullptr, from_y));  // recompute
      L2L_TRY(layer_backward_group<bf16>(c, c->slot[slot], x, dy, G, ng, y, rs, from_y));
    } else if (c->cfg.dtype == L2L_FP16) {
      if (from_y) L2L_TRY(layer_ln2_backward_from_y<fp16>(c, c->slot[slot], dy, G, ng, y, rs));
      L2L_TRY(layer_forward_group<fp16>(c, slot, x, nullptr, ng, true, nullptr, from_y));
      L2L_TRY(layer_backward_group<fp16>(c, c->slot[slot], x, dy, G, ng, y, rs, from_y));
    } else {
      if (from_y) L2L_TRY(layer_ln2_backward_from_y<float>(c, c->slot[slot], dy, G, ng, y, rs));
      L2L_TRY(layer_forward_group<float>(c, slot, x, nullptr, ng, true, nullptr, from_y));
      L2L_TRY(layer_backward_group<float>(c, c->slot[slot], x, dy, G, ng, y, rs, from_y));
    }
  }
  HIP_TRY(c, hipEventRecord(c->slot_released[slot], c->cs));
  HIP_TRY(c, hipEventRecord(c->gacc_ready[a], c->cs));
  c->gacc_layer[a] = layer;
  c->gacc_state[a] = 1;
  c->gacc_next = a ^ 1;
  return L2L_OK;
}

int l2l_layer_bwd(l2l_ctx* c, int layer, int slot, const void* x_stash, void* dy_dx) {
  return layer_bwd_impl(c, layer, slot, x_stash, dy_dx, nullptr, nullptr);
}

int l2l_layer_bwd_stats(l2l_ctx* c, int layer, int slot, const void* x_stash, const void* y_stash, const float* rstd, void* dy_dx) {
  if (c && (!y_stash || !rstd)) return fail(c, L2L_E_ARG, "l2l_layer_bwd_stats: null pointer");
  return layer_bwd_impl(c, layer, slot, x_stash, dy_dx, y_stash, rstd);
}

// A host <-> device copy issued as rows of 64 KiB (hipMemcpy2DAsync) plus a plain copy of the remainder.  This
// runtime carries a plain device-to-host hipMemcpyAsync out with a copy kernel, whose workgroups sit on the compute
// units for the length of the transfer; a resident GEMM workgroup needs a compute unit's whole register file and
// cannot be placed beside them.  Written as rows, the same bytes go through a DMA engine in either direction.
static hipError_t memcpy_rows_async(void* dst, const void* src, size_t bytes, hipMemcpyKind kind, hipStream_t s) {
  constexpr size_t ROW = 64 << 10;
  const size_t rows = bytes / ROW, body = rows * ROW;
  if (rows > 0) {
    const hipError_t e = hipMemcpy2DAsync(dst, ROW, src, ROW, ROW, rows, kind, s);
    if (e != hipSuccess) return e;
  }
  if (bytes > body) return hipMemcpyAsync((char*)dst + body, (const char*)src + body, bytes - body, kind, s);
  return hipSuccess;
}

// elements [first, first + count) of an fp32 accumulator -> the same elements of the host landing buffer, in the drain
// format, on the copy stream
static int drain_copy(l2l_ctx* c, void* host, const float* acc, long long first, long long count) {
  if (c->drain_dtype == L2L_F32) {
    if (c->copy_rows) HIP_TRY(c, memcpy_rows_async((float*)host + first, acc + first, count * 4, hipMemcpyDeviceToHost, c->xs));
    else HIP_TRY(c, hipMemcpyAsync((float*)host + first, acc + first, count * 4, hipMemcpyDeviceToHost, c->xs));
    return L2L_OK;
  }
  if ((size_t)count > c->drain_stage_elems) return fail(c, L2L_E_STATE, "drain: %lld elements exceed the 16-bit staging buffer", count);
  const unsigned blocks = (unsigned)std::min<long long>((count / 4 + 255) / 256 + 1, 2048);
  if (c->drain_dtype == L2L_BF16) hipLaunchKernelGGL(narrow_kernel<bf16>, dim3(blocks), dim3(256), 0, c->xs, acc + first, (bf16*)c->drain_stage, count);
  else hipLaunchKernelGGL(narrow_kernel<fp16>, dim3(blocks), dim3(256), 0, c->xs, acc + first, (fp16*)c->drain_stage, count);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(c, L2L_E_HIP, "narrow launch: %s", hipGetErrorString(e));
  if (c->copy_rows) HIP_TRY(c, memcpy_rows_async((char*)host + first * 2, c->drain_stage, count * 2, hipMemcpyDeviceToHost, c->xs));
  else HIP_TRY(c, hipMemcpyAsync((char*)host + first * 2, c->drain_stage, count * 2, hipMemcpyDeviceToHost, c->xs));
  return L2L_OK;
}
static double drain_bytes(const l2l_ctx* c, long long count) { return (double)count * (c->drain_dtype == L2L_F32 ? 4 : 2); }

int l2l_set_drain_dtype(l2l_ctx* c, int dtype) {
  if (!c) return L2L_E_ARG;
  if (dtype != L2L_F32 && dtype != L2L_BF16 && dtype != L2L_FP16) return fail(c, L2L_E_ARG, "l2l_set_drain_dtype: unknown dtype %d", dtype);
  if (dtype != L2L_F32 && !c->drain_stage) {
    const size_t n = (size_t)std::max<long long>(c->lay.total, c->cfg.vocab > 0 ? c->lay.etotal : 0);
    L2L_TRY(dev_alloc(c, &c->drain_stage, n * 2));
    c->drain_stage_elems = n;
  }
  c->drain_dtype = dtype;
  return L2L_OK;
}

int l2l_grad_drain(l2l_ctx* c, int layer, void* host_grads) {
  if (!c) return L2L_E_ARG;
  if (!host_grads) return fail(c, L2L_E_ARG, "l2l_grad_drain: null host pointer");
  for (int a = 0; a < 2; ++a) {
    if (c->gacc_state[a] == 1 && c->gacc_layer[a] == layer) {
      HIP_TRY(c, hipStreamWaitEvent(c->xs, c->gacc_ready[a], 0));
      const CopyMark mark = copy_begin(c);
      L2L_TRY(drain_copy(c, host_grads, c->gacc[a], 0, c->lay.total));
      HIP_TRY(c, hipEventRecord(c->gacc_landed[a], c->xs));
      L2L_TRY(fill_zero_copy_stream(c, c->gacc[a], c->lay.total * 4));   // "erased from the device" (Section 2.1)
      copy_end(c, mark, drain_bytes(c, c->lay.total));
      HIP_TRY(c, hipEventRecord(c->gacc_drained[a], c->xs));
      c->gacc_state[a] = 2;
      return L2L_OK;
    }
  }
  return fail(c, L2L_E_STATE, "l2l_grad_drain: no un-drained gradients for layer %d", layer);
}

int l2l_drain_wait(l2l_ctx* c, int layer) {
  if (!c) return L2L_E_ARG;
  for (int a = 0; a < 2; ++a) {
    if (c->gacc_state[a] == 2 && c->gacc_layer[a] == layer) {
      HIP_TRY(c, hipEventSynchronize(c->gacc_landed[a]));
      return L2L_OK;
    }
  }
  return fail(c, L2L_E_STATE, "l2l_drain_wait: no drain in flight for layer %d", layer);
}

// ---- embedding and head ----------------------------------------------------------------------------
static int need_vocab(l2l_ctx* c, const char* who) {
  if (!c) return L2L_E_ARG;
  if (c->cfg.vocab <= 0) return fail(c, L2L_E_STATE, "%s: context was created with vocab = 0", who);
  return L2L_OK;
}

int l2l_embed_stage(l2l_ctx* c, const void* host) {
  L2L_TRY(need_vocab(c, "l2l_embed_stage"));
  if (!host) return fail(c, L2L_E_ARG, "l2l_embed_stage: null host pointer");
  if (c->emb_staged) HIP_TRY(c, hipStreamWaitEvent(c->xs, c->emb_released_ev, 0));
  const CopyMark mark = copy_begin(c);
  HIP_TRY(c, hipMemcpyAsync(c->emb, host, c->lay.etotal * esize(c->cfg.dtype), hipMemcpyHostToDevice, c->xs));
  copy_end(c, mark, (double)c->lay.etotal * esize(c->cfg.dtype));
  HIP_TRY(c, hipEventRecord(c->emb_staged_ev, c->xs));
  c->emb_staged = 1;
  return L2L_OK;
}


int l2l_embed_stage_part(l2l_ctx* c, const void* host, long long first, long long count) {
  L2L_TRY(need_vocab(c, "l2l_embed_stage_part"));
  if (!host) return fail(c, L2L_E_ARG, "l2l_embed_stage_part: null host pointer");
  if (first < 0 || count <= 0 || first + count > c->lay.etotal)
    return fail(c, L2L_E_ARG, "l2l_embed_stage_part: elements %lld..%lld outside the block of %lld", first, first + count, c->lay.etotal);
  if (c->emb_staged) HIP_TRY(c, hipStreamWaitEvent(c->xs, c->emb_released_ev, 0));
  const size_t es = esize(c->cfg.dtype);
  const CopyMark mark = copy_begin(c);
  HIP_TRY(c, hipMemcpyAsync((char*)c->emb + first * es, (const char*)host + first * es, count * es, hipMemcpyHostToDevice, c->xs));
  copy_end(c, mark, (double)count * es);
  HIP_TRY(c, hipEventRecord(c->emb_staged_ev, c->xs));
  c->emb_staged = 1;
  return L2L_OK;
}

int l2l_embed_fwd(l2l_ctx* c, const int32_t* tokens, void* x_out) {
  L2L_TRY(need_vocab(c, "l2l_embed_fwd"));
  if (!tokens || !x_out) return fail(c, L2L_E_ARG, "l2l_embed_fwd: null pointer");
  if (!c->emb_staged) return fail(c, L2L_E_STATE, "l2l_embed_fwd: embedding block never staged");
  if (c->egacc_state == 1) return fail(c, L2L_E_STATE, "l2l_embed_fwd: embedding gradients of the previous step were never drained");
  HIP_TRY(c, hipStreamWaitEvent(c->cs, c->emb_staged_ev, 0));
  if (c->egacc_state == 2) HIP_TRY(c, hipStreamWaitEvent(c->cs, c->egacc_drained, 0));
  c->egacc_state = 0;   // the accumulator is zero: cleared at creation and after every drain
  if (c->cfg.dtype == L2L_BF16) L2L_TRY(embed_fwd_t<bf16>(c, tokens, x_out));
  else if (c->cfg.dtype == L2L_FP16) L2L_TRY(embed_fwd_t<fp16>(c, tokens, x_out));
  else L2L_TRY(embed_fwd_t<float>(c, tokens, x_out));
  HIP_TRY(c, hipEventRecord(c->emb_released_ev, c->cs));
  return L2L_OK;
}


int l2l_head_loss(l2l_ctx* c, const void* x_last, const int32_t* labels, void* dy_out, float* loss_out) {
  L2L_TRY(need_vocab(c, "l2l_head_loss"));
  if (!x_last || !labels || !dy_out || !loss_out) return fail(c, L2L_E_ARG, "l2l_head_loss: null pointer");
  if (!c->emb_staged) return fail(c, L2L_E_STATE, "l2l_head_loss: embedding block never staged");
  HIP_TRY(c, hipStreamWaitEvent(c->cs, c->emb_staged_ev, 0));
  if (c->cfg.dtype == L2L_BF16) L2L_TRY(head_loss_t<bf16>(c, x_last, labels, dy_out, loss_out));
  else if (c->cfg.dtype == L2L_FP16) L2L_TRY(head_loss_t<fp16>(c, x_last, labels, dy_out, loss_out));
  else L2L_TRY(head_loss_t<float>(c, x_last, labels, dy_out, loss_out));
  HIP_TRY(c, hipEventRecord(c->emb_released_ev, c->cs));
  return L2L_OK;
}


int l2l_embed_bwd(l2l_ctx* c, const int32_t* tokens, const void* dy) {
  L2L_TRY(need_vocab(c, "l2l_embed_bwd"));
  if (!tokens || !dy) return fail(c, L2L_E_ARG, "l2l_embed_bwd: null pointer");
  if (!c->emb_staged) return fail(c, L2L_E_STATE, "l2l_embed_bwd: embedding block never staged");
  if (c->cfg.dtype == L2L_BF16) L2L_TRY(embed_bwd_t<bf16>(c, tokens, dy));
  else if (c->cfg.dtype == L2L_FP16) L2L_TRY(embed_bwd_t<fp16>(c, tokens, dy));
  else L2L_TRY(embed_bwd_t<float>(c, tokens, dy));
  HIP_TRY(c, hipEventRecord(c->emb_released_ev, c->cs));
  HIP_TRY(c, hipEventRecord(c->egacc_ready, c->cs));
  c->egacc_state = 1;
  return L2L_OK;
}

int l2l_embed_grad_drain(l2l_ctx* c, void* host_grads) {
  L2L_TRY(need_vocab(c, "l2l_embed_grad_drain"));
  if (!host_grads) return fail(c, L2L_E_ARG, "l2l_embed_grad_drain: null host pointer");
  if (c->egacc_state != 1) return fail(c, L2L_E_STATE, "l2l_embed_grad_drain: no un-drained embedding gradients");
  if (c->egacc_part_next != 0) return fail(c, L2L_E_STATE, "l2l_embed_grad_drain: a drain in pieces is under way");
  HIP_TRY(c, hipStreamWaitEvent(c->xs, c->egacc_ready, 0));
  const CopyMark mark = copy_begin(c);
  L2L_TRY(drain_copy(c, host_grads, c->egacc, 0, c->lay.etotal));
  HIP_TRY(c, hipEventRecord(c->egacc_landed, c->xs));
  L2L_TRY(fill_zero_copy_stream(c, c->egacc, c->lay.etotal * 4));
  copy_end(c, mark, drain_bytes(c, c->lay.etotal));
  HIP_TRY(c, hipEventRecord(c->egacc_drained, c->xs));
  c->egacc_state = 2;
  return L2L_OK;
}

int l2l_embed_grad_drain_part(l2l_ctx* c, void* host_grads, long long first, long long count) {
  L2L_TRY(need_vocab(c, "l2l_embed_grad_drain_part"));
  if (!host_grads) return fail(c, L2L_E_ARG, "l2l_embed_grad_drain_part: null host pointer");
  if (c->egacc_state != 1) return fail(c, L2L_E_STATE, "l2l_embed_grad_drain_part: no un-drained embedding gradients");
  if (first != c->egacc_part_next || count <= 0 || first + count > c->lay.etotal)
    return fail(c, L2L_E_ARG, "l2l_embed_grad_drain_part: piece %lld..%lld, expected one starting at %lld within %lld elements", first,
                first + count, c->egacc_part_next, c->lay.etotal);
  if (c->drain_dtype != L2L_F32 && first % 4) return fail(c, L2L_E_ARG, "l2l_embed_grad_drain_part: 16-bit drains take pieces that start at multiples of 4 elements");
  if (first == 0) HIP_TRY(c, hipStreamWaitEvent(c->xs, c->egacc_ready, 0));
  const CopyMark mark = copy_begin(c);
  L2L_TRY(drain_copy(c, host_grads, c->egacc, first, count));
  c->egacc_part_next = first + count;
  if (c->egacc_part_next == c->lay.etotal) {   // the block is out: clear and release the accumulator
    HIP_TRY(c, hipEventRecord(c->egacc_landed, c->xs));
    L2L_TRY(fill_zero_copy_stream(c, c->egacc, c->lay.etotal * 4));
    copy_end(c, mark, drain_bytes(c, count));
    HIP_TRY(c, hipEventRecord(c->egacc_drained, c->xs));
    c->egacc_state = 2;
    c->egacc_part_next = 0;
  } else {
    copy_end(c, mark, drain_bytes(c, count));
  }
  return L2L_OK;
}

int l2l_embed_drain_wait(l2l_ctx* c) {
  L2L_TRY(need_vocab(c, "l2l_embed_drain_wait"));
  if (c->egacc_state != 2) return fail(c, L2L_E_STATE, "l2l_embed_drain_wait: no drain in flight");
  HIP_TRY(c, hipEventSynchronize(c->egacc_landed));
  return L2L_OK;
}

int l2l_cls_stage(l2l_ctx* c, const void* host_params, int classes) {
  if (!c) return L2L_E_ARG;
  if (!host_params) return fail(c, L2L_E_ARG, "l2l_cls_stage: null host pointer");
  if (classes < 2) return fail(c, L2L_E_ARG, "l2l_cls_stage: %d classes", classes);
  if (c->cls_classes && c->cls_classes != classes)
    return fail(c, L2L_E_ARG, "l2l_cls_stage: the head was set up for %d classes, not %d", c->cls_classes, classes);
  const size_t es = esize(c->cfg.dtype);
  if (!c->cls_classes) {   // first use: the head's buffers
    const ClsLayout L = make_cls_layout(&c->cfg, classes);
    for (int i = 0; i < N_CLS_T; ++i) { c->cls_off[i] = L.off[i]; c->cls_size[i] = L.size[i]; }
    c->cls_total = L.total;
    c->cls_cp = up(classes, 8);
    const long long nseq = (long long)c->cfg.ubatch * c->cfg.num_ubatches, H = c->cfg.hidden;
    L2L_TRY(dev_alloc(c, &c->cls_w, L.total * es));
    L2L_TRY(dev_alloc(c, (void**)&c->cls_g, L.total * 4));
    HIP_TRY(c, hipMemset(c->cls_g, 0, L.total * 4));
    void** rows[] = {&c->cls_x, &c->cls_u, &c->cls_p, &c->cls_dp, &c->cls_du, &c->cls_dx};
    for (void** p : rows) L2L_TRY(dev_alloc(c, p, nseq * H * es));
    L2L_TRY(dev_alloc(c, (void**)&c->cls_z, nseq * c->cls_cp * 4));
    L2L_TRY(dev_alloc(c, &c->cls_dz, nseq * c->cls_cp * es));
    hipEvent_t* evs[] = {&c->cls_staged_ev, &c->cls_released_ev, &c->cls_ready, &c->cls_landed, &c->cls_drained};
    for (hipEvent_t* e : evs) HIP_TRY(c, hipEventCreateWithFlags(e, hipEventDisableTiming));
    c->cls_classes = classes;
  }
  if (c->cls_staged) HIP_TRY(c, hipStreamWaitEvent(c->xs, c->cls_released_ev, 0));
  const CopyMark mark = copy_begin(c);
  HIP_TRY(c, hipMemcpyAsync(c->cls_w, host_params, c->cls_total * es, hipMemcpyHostToDevice, c->xs));
  copy_end(c, mark, (double)c->cls_total * es);
  HIP_TRY(c, hipEventRecord(c->cls_staged_ev, c->xs));
  c->cls_staged = 1;
  return L2L_OK;
}

int l2l_cls_head_loss(l2l_ctx* c, const void* x_last, const int32_t* seq_labels, void* dy_out, float* loss_out) {
  if (!c) return L2L_E_ARG;
  if (!x_last || !seq_labels || !dy_out || !loss_out) return fail(c, L2L_E_ARG, "l2l_cls_head_loss: null pointer");
  if (!c->cls_staged) return fail(c, L2L_E_STATE, "l2l_cls_head_loss: head parameters never staged");
  if (c->cls_state == 1) return fail(c, L2L_E_STATE, "l2l_cls_head_loss: the head's gradients of the previous step were never drained");
  HIP_TRY(c, hipStreamWaitEvent(c->cs, c->cls_staged_ev, 0));
  if (c->cls_state == 2) HIP_TRY(c, hipStreamWaitEvent(c->cs, c->cls_drained, 0));
  if (c->cfg.dtype == L2L_BF16) L2L_TRY(cls_head_t<bf16>(c, x_last, seq_labels, dy_out, loss_out));
  else if (c->cfg.dtype == L2L_FP16) L2L_TRY(cls_head_t<fp16>(c, x_last, seq_labels, dy_out, loss_out));
  else L2L_TRY(cls_head_t<float>(c, x_last, seq_labels, dy_out, loss_out));
  HIP_TRY(c, hipEventRecord(c->cls_released_ev, c->cs));
  HIP_TRY(c, hipEventRecord(c->cls_ready, c->cs));
  c->cls_state = 1;
  return L2L_OK;
}

int l2l_cls_grad_drain(l2l_ctx* c, void* host_grads) {
  if (!c) return L2L_E_ARG;
  if (!host_grads) return fail(c, L2L_E_ARG, "l2l_cls_grad_drain: null host pointer");
  if (c->cls_state != 1) return fail(c, L2L_E_STATE, "l2l_cls_grad_drain: no un-drained head gradients");
  HIP_TRY(c, hipStreamWaitEvent(c->xs, c->cls_ready, 0));
  const CopyMark mark = copy_begin(c);
  L2L_TRY(drain_copy(c, host_grads, c->cls_g, 0, c->cls_total));
  HIP_TRY(c, hipEventRecord(c->cls_landed, c->xs));
  L2L_TRY(fill_zero_copy_stream(c, c->cls_g, c->cls_total * 4));
  copy_end(c, mark, drain_bytes(c, c->cls_total));
  HIP_TRY(c, hipEventRecord(c->cls_drained, c->xs));
  c->cls_state = 2;
  return L2L_OK;
}

int l2l_cls_drain_wait(l2l_ctx* c) {
  if (!c) return L2L_E_ARG;
  if (c->cls_state != 2) return fail(c, L2L_E_STATE, "l2l_cls_drain_wait: no drain in flight");
  HIP_TRY(c, hipEventSynchronize(c->cls_landed));
  return L2L_OK;
}

int l2l_set_loss_scale(l2l_ctx* c, float scale) {
  if (!c) return L2L_E_ARG;
  if (!(scale > 0.f) || !std::isfinite(scale)) return fail(c, L2L_E_ARG, "l2l_set_loss_scale: scale must be positive and finite");
  c->loss_scale = scale;
  return L2L_OK;
}

int l2l_stream_create_cu_masked(int cus_per_32, void** out) {
  if (!out || cus_per_32 < 1 || cus_per_32 > 32) return L2L_E_ARG;
  *out = nullptr;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    (void)hipGetLastError();
    return L2L_E_HIP;
  }
  const int words = (prop.multiProcessorCount + 31) / 32;
  std::vector<uint32_t> mask((size_t)words, cus_per_32 == 32 ? 0xFFFFFFFFu : ((1u << cus_per_32) - 1u));
  hipStream_t s = nullptr;
  const hipError_t err = hipExtStreamCreateWithCUMask(&s, (uint32_t)words, mask.data());
  if (err != hipSuccess) {
    fprintf(stderr, "l2l_stream_create_cu_masked: %s (%d CUs, %d mask words)\n", hipGetErrorString(err), prop.multiProcessorCount, words);
    (void)hipGetLastError();
    return L2L_E_HIP;
  }
  *out = (void*)s;
  return L2L_OK;
}

int l2l_memcpy_rows_async(void* dst, const void* src, size_t bytes, int to_host, void* stream) {
  if (!dst || !src) return L2L_E_ARG;
  if (bytes == 0) return L2L_OK;
  if (memcpy_rows_async(dst, src, bytes, to_host ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice, (hipStream_t)stream) != hipSuccess) {
    (void)hipGetLastError();
    return L2L_E_HIP;
  }
  return L2L_OK;
}

int l2l_stream_destroy(void* stream) {
  if (!stream) return L2L_E_ARG;
  if (hipStreamDestroy((hipStream_t)stream) != hipSuccess) {
    (void)hipGetLastError();
    return L2L_E_HIP;
  }
  return L2L_OK;
}

// ---- profiling -----------------------------------------------------------------------------------
static void prof_resolve(l2l_ctx* c) {
  for (auto& r : c->prof) {
    (void)hipEventSynchronize(r.b);
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
      float t0 = 0.f;
      if (c->prof_base && hipEventElapsedTime(&t0, c->prof_base, r.a) == hipSuccess)
        (r.cls == L2L_PROF_COPY ? c->iv_copy : c->iv_compute).push_back({t0, t0 + ms});
      if (r.shape >= 0 && r.shape < (int)c->prof_shapes.size()) {
        c->prof_shapes[r.shape].launches += 1;
        c->prof_shapes[r.shape].ms += ms;
      }
      c->prof_n[r.cls] += 1;
      c->prof_ms[r.cls] += ms;
      c->prof_fl[r.cls] += r.flops;
      c->prof_by[r.cls] += r.bytes;
    }
    c->ev_pool.push_back(r.a);
    c->ev_pool.push_back(r.b);
  }
  c->prof.clear();
  (void)hipGetLastError();
}

int l2l_profile(l2l_ctx* c, int on) {
  if (!c) return L2L_E_ARG;
  prof_resolve(c);
  for (int i = 0; i < L2L_PROF_CLASSES; ++i) { c->prof_n[i] = 0; c->prof_ms[i] = c->prof_fl[i] = c->prof_by[i] = 0; }
  c->iv_compute.clear();
  c->iv_copy.clear();
  c->prof_shapes.clear();
  c->prof_on = on;
  if (on) {
    if (!c->prof_base) HIP_TRY(c, hipEventCreate(&c->prof_base));
    HIP_TRY(c, hipEventRecord(c->prof_base, c->cs));
  }
  return L2L_OK;
}

int l2l_profile_overlap(l2l_ctx* c, double merge_gap_ms, double* compute_busy_ms, double* copy_busy_ms, double* copy_hidden_ms,
                        double* span_ms) {
  if (!c || !(merge_gap_ms >= 0.0)) return L2L_E_ARG;
  prof_resolve(c);
  typedef std::vector<std::pair<float, float>> Iv;
  const auto merged = [](Iv v, float gap) {
    std::sort(v.begin(), v.end());
    Iv out;
    for (const auto& p : v) {
      if (!out.empty() && p.first <= out.back().second + gap) out.back().second = std::max(out.back().second, p.second);
      else out.push_back(p);
    }
    return out;
  };
  const auto length = [](const Iv& v) {
    double s = 0.0;
    for (const auto& p : v) s += (double)p.second - p.first;
    return s;
  };
  const Iv a = merged(c->iv_compute, (float)merge_gap_ms), b = merged(c->iv_copy, 0.f);
  double both = 0.0;
  for (size_t i = 0, j = 0; i < a.size() && j < b.size();) {
    const float lo = std::max(a[i].first, b[j].first), hi = std::min(a[i].second, b[j].second);
    if (lo < hi) both += (double)hi - lo;
    if (a[i].second < b[j].second) ++i; else ++j;
  }
  double first = 1e300, last = -1e300;
  for (const Iv* v : {&a, &b})
    for (const auto& p : *v) { first = std::min<double>(first, p.first); last = std::max<double>(last, p.second); }
  if (compute_busy_ms) *compute_busy_ms = length(a);
  if (copy_busy_ms) *copy_busy_ms = length(b);
  if (copy_hidden_ms) *copy_hidden_ms = both;
  if (span_ms) *span_ms = last > first ? last - first : 0.0;
  return L2L_OK;
}

int l2l_profile_gemm_table(l2l_ctx* c, char* buf, size_t cap) {
  if (!c || !buf || cap == 0) return L2L_E_ARG;
  prof_resolve(c);
  size_t at = 0;
  buf[0] = 0;
  for (const ProfShape& p : c->prof_shapes) {
    const int n = snprintf(buf + at, cap - at, "%d %d %d %d %d %d %d %d %lld %.6f\n", p.M, p.N, p.K, p.a_kc, p.b_kc, p.epi, p.out_f32,
                           p.pass, p.launches, p.ms);
    if (n < 0 || (size_t)n >= cap - at) return fail(c, L2L_E_ARG, "l2l_profile_gemm_table: %zu bytes are too few", cap);
    at += (size_t)n;
  }
  return L2L_OK;
}

int l2l_profile_read(l2l_ctx* c, int cls, long long* launches, double* ms, double* flops, double* bytes) {
  if (!c) return L2L_E_ARG;
  if (cls < 0 || cls >= L2L_PROF_CLASSES) return fail(c, L2L_E_ARG, "l2l_profile_read: class %d", cls);
  prof_resolve(c);
  if (launches) *launches = c->prof_n[cls];
  if (ms) *ms = c->prof_ms[cls];
  if (flops) *flops = c->prof_fl[cls];
  if (bytes) *bytes = c->prof_by[cls];
  return L2L_OK;
}

// ---- single operations ---------------------------------------------------------------------------
int l2l_op_gemm_ex(l2l_ctx* c, int in_dtype, int out_f32, int a_kc, int b_kc, int M, int N, int K, const void* A, long long lda,
                   const void* B, long long ldb, void* C, long long ldc, float alpha, const void* bias, const void* resid,
                   long long ldr, int epi, const void* aux, void* aux_out, long long ldaux, float* colsum, long long colsum_rows,
                   int* colsum_rows_used, int impl) {
  if (!c) return L2L_E_ARG;
  if (!A || !B || !C) return fail(c, L2L_E_ARG, "l2l_op_gemm: null pointer");
  if (M < 0 || N < 0 || K < 0 || lda <= 0 || ldb <= 0 || ldc < N) return fail(c, L2L_E_ARG, "l2l_op_gemm: bad shape");
  if (in_dtype != L2L_F32 && in_dtype != L2L_BF16 && in_dtype != L2L_FP16) return fail(c, L2L_E_ARG, "l2l_op_gemm: bad dtype");
  if (in_dtype == L2L_F32) out_f32 = 1;
  if (epi & ~(L2L_EPI_GELU | L2L_EPI_GELUGRAD | L2L_EPI_ACCUM | L2L_EPI_COLSUM | L2L_EPI_KEEPGRAD | L2L_EPI_MULAUX))
    return fail(c, L2L_E_ARG, "l2l_op_gemm: unknown epilogue flag in %d", epi);
  if ((epi & L2L_EPI_KEEPGRAD) && (!(epi & L2L_EPI_GELU) || !aux_out)) return fail(c, L2L_E_ARG, "l2l_op_gemm: keeping gelu' goes with GELU and a buffer for it");
  if ((epi & L2L_EPI_MULAUX) && (!aux || ldaux < N || (epi & (L2L_EPI_GELU | L2L_EPI_GELUGRAD))))
    return fail(c, L2L_E_ARG, "l2l_op_gemm: the element-wise factor needs its buffer and row stride, and excludes GELU and GELU'");
  if ((epi & L2L_EPI_ACCUM) && !out_f32) return fail(c, L2L_E_ARG, "l2l_op_gemm: accumulate needs an fp32 output");
  if (impl < 0 || (impl > 2 && impl < 100)) return fail(c, L2L_E_ARG, "l2l_op_gemm: impl %d", impl);
  if (resid && ldr < N) return fail(c, L2L_E_ARG, "l2l_op_gemm: residual row stride %lld < N", ldr);
  if ((epi & L2L_EPI_GELUGRAD) && (!aux || ldaux < N)) return fail(c, L2L_E_ARG, "l2l_op_gemm: GELU' needs the pre-activation and its row stride");
  if ((epi & L2L_EPI_GELU) && aux_out && ldaux < N) return fail(c, L2L_E_ARG, "l2l_op_gemm: pre-activation row stride %lld < N", ldaux);
  if ((epi & L2L_EPI_GELU) && (epi & L2L_EPI_GELUGRAD)) return fail(c, L2L_E_ARG, "l2l_op_gemm: GELU and GELU' share the pre-activation stride: one of them per call");
  GemmArgs g = gemm_args(M, N, K, A, lda, a_kc != 0, B, ldb, b_kc != 0, C, ldc);
  g.alpha = alpha;
  if (bias) { g.epi |= EPI_BIAS; g.bias = bias; }
  if (epi & L2L_EPI_GELU) { g.epi |= EPI_GELU; g.aux_out = aux_out; g.ldaux = ldaux; }
  if (epi & L2L_EPI_KEEPGRAD) g.epi |= EPI_KEEPGRAD;
  if (epi & L2L_EPI_MULAUX) { g.epi |= EPI_MULAUX; g.aux = aux; g.ldaux = ldaux; }
  if (epi & L2L_EPI_GELUGRAD) { g.epi |= EPI_GELUGRAD; g.aux = aux; g.ldaux = ldaux; }
  if (resid) { g.epi |= EPI_RESID; g.resid = resid; g.ldr = ldr; }
  if (epi & L2L_EPI_ACCUM) g.epi |= EPI_ACCUM;
  if (colsum_rows_used) *colsum_rows_used = 0;
  if (epi & L2L_EPI_COLSUM) {
    int rows = 0;
    g.colsum = colsum;
    if (!colsum || impl != 0 || M == 0 || N == 0 || !colsum_in_gemm_ok(in_dtype, out_f32 != 0, g, &rows))
      return fail(c, L2L_E_ARG, "l2l_op_gemm: column sums are not available for this shape, layout or implementation");
    if (rows > colsum_rows) return fail(c, L2L_E_ARG, "l2l_op_gemm: column sums need %d rows, the buffer has %lld", rows, colsum_rows);
    if (colsum_rows_used) *colsum_rows_used = rows;
    g.epi |= EPI_COLSUM;
  }
  return gemm(c, in_dtype, out_f32 != 0, g, impl);
}

int l2l_op_gemm(l2l_ctx* c, int in_dtype, int out_f32, int a_kc, int b_kc, int M, int N, int K, const void* A, long long lda,
                const void* B, long long ldb, void* C, long long ldc, float alpha, const void* bias, const void* resid, int gelu,
                int accumulate, int impl) {
  return l2l_op_gemm_ex(c, in_dtype, out_f32, a_kc, b_kc, M, N, K, A, lda, B, ldb, C, ldc, alpha, bias, resid, ldc,
                        (gelu ? L2L_EPI_GELU : 0) | (accumulate ? L2L_EPI_ACCUM : 0), nullptr, nullptr, 0, nullptr, 0, nullptr, impl);
}

// ---- an entry point that allocates nothing --------------------------------------------------------
// C += A B like l2l_op_gemm(..., out_f32 = 1, accumulate = 1) on the K-split path, whose kernels keep the splits'
// partial results in a workspace: here that workspace is a file-scope device array instead of context memory, so the
// call needs no context and makes no allocation.  Every GPU the library runs on holds its own copy of the array until
// the process ends; calls on one GPU share it, so calls that overlap there race.
constexpr size_t kNoallocScratchFloats = (size_t)8 << 20;   // 32 MiB
static __device__ __align__(256) float scratch[kNoallocScratchFloats];

namespace {
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};   // per device: the array's address there, from hipGetSymbolAddress
int g_num_cus[kMaxDevices] = {};
std::mutex g_scratch_mu;
thread_local char g_noalloc_err[256] = "no error";

int noalloc_fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_noalloc_err, sizeof(g_noalloc_err), fmt, ap);
  va_end(ap);
  return code;
}

// the current device's copy of `scratch` (looked up once per device, with that device current)
int noalloc_scratch(float** ptr, int* cus) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { (void)hipGetLastError(); return noalloc_fail(L2L_E_HIP, "hipGetDevice: %s", hipGetErrorString(e)); }
  if (dev < 0 || dev >= kMaxDevices) return noalloc_fail(L2L_E_ARG, "device %d: the library keeps scratch addresses for devices 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> l(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { (void)hipGetLastError(); return noalloc_fail(L2L_E_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e)); }
    int n = 0;
    e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) { (void)hipGetLastError(); n = 0; }
    g_num_cus[dev] = n;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  *cus = g_num_cus[dev];
  return L2L_OK;
}
}  // namespace

size_t l2l_noalloc_scratch_bytes(void) { return kNoallocScratchFloats * sizeof(float); }
const char* l2l_noalloc_last_error(void) { return g_noalloc_err; }

int l2l_op_gemm_accum_noalloc(void* stream, int in_dtype, int a_kc, int b_kc, int M, int N, int K, const void* A, long long lda,
                              const void* B, long long ldb, float* C, long long ldc) {
  if (!A || !B || !C) return noalloc_fail(L2L_E_ARG, "l2l_op_gemm_accum_noalloc: null pointer");
  if (in_dtype != L2L_BF16 && in_dtype != L2L_FP16) return noalloc_fail(L2L_E_ARG, "l2l_op_gemm_accum_noalloc: operands are bf16 or fp16");
  if (M < 0 || N < 0 || K < 0 || lda <= 0 || ldb <= 0 || ldc < N) return noalloc_fail(L2L_E_ARG, "l2l_op_gemm_accum_noalloc: bad shape");
  if (M == 0 || N == 0 || K == 0) return L2L_OK;   // nothing to add
  GemmArgs g = gemm_args(M, N, K, A, lda, a_kc != 0, B, ldb, b_kc != 0, C, ldc);
  g.epi = EPI_ACCUM;
  if (!mfma_ok(g)) return noalloc_fail(L2L_E_ARG, "l2l_op_gemm_accum_noalloc: operand alignment, row pitch or extent not supported by the MFMA kernels");
  if ((g.M + 63) / 64 > 65535) return noalloc_fail(L2L_E_ARG, "l2l_op_gemm_accum_noalloc: grid too large");
  int v, splits;
  pick_tile(g, true, &v, &splits);
  if (kTiles[v].direct && !g.a_kc && g.b_kc) v = 3;
  float* ws = nullptr;
  int cus = 0;
  L2L_TRY(noalloc_scratch(&ws, &cus));
  g.resident = cus;
  const hipStream_t s = (hipStream_t)stream;
  const int how = launch_split_through_workspace(v, g, s, splits, true, in_dtype == L2L_FP16, ws, kNoallocScratchFloats);
  if (how == SPLIT_NO_ROOM)
    return noalloc_fail(L2L_E_ARG, "l2l_op_gemm_accum_noalloc: %d x %d outputs in %d K-splits need %zu bytes of scratch, the library holds %zu",
                        M, N, splits, (size_t)splits * M * N * 4, kNoallocScratchFloats * sizeof(float));
  if (how == SPLIT_NOT_APPLICABLE) launch_mfma_variant(v, g, s, splits, true, in_dtype == L2L_FP16);   // no split, or splits adding with atomics: no scratch
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return noalloc_fail(L2L_E_HIP, "kernel launch: %s", hipGetErrorString(e));
  return L2L_OK;
}

int l2l_op_layernorm(l2l_ctx* c, int dtype, int rows, int n, const void* x, const void* gamma, const void* beta, float eps, void* y,
                     float* mean, float* rstd) {
  if (!c) return L2L_E_ARG;
  if (!x || !gamma || !beta || !y) return fail(c, L2L_E_ARG, "l2l_op_layernorm: null pointer");
  if (rows < 0 || n <= 0 || n % 8) return fail(c, L2L_E_ARG, "l2l_op_layernorm: n must be a positive multiple of 8");
  if ((mean == nullptr) != (rstd == nullptr)) return fail(c, L2L_E_ARG, "l2l_op_layernorm: mean and rstd go together");
  if (dtype == L2L_BF16) return ln_fwd<bf16>(c, x, gamma, beta, y, mean, rstd, rows, n, eps);
  if (dtype == L2L_FP16) return ln_fwd<fp16>(c, x, gamma, beta, y, mean, rstd, rows, n, eps);
  if (dtype == L2L_F32) return ln_fwd<float>(c, x, gamma, beta, y, mean, rstd, rows, n, eps);
  return fail(c, L2L_E_ARG, "l2l_op_layernorm: bad dtype");
}

}  // extern "C"
