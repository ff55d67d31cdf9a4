/*
 * l2l.h -- C ABI of the L2L (layer-to-layer) relay-execution device library for MI355X (gfx950).
 *
 * The library runs the hot path of L2L execution (Algorithm 2, Section 2.1-2.2 of the paper): one
 * transformer encoder layer at a time is resident on the device and runs its forward pass -- and its
 * backward pass with the layer forward recomputed from the stashed boundary activation -- across
 * all U micro-batches of the minibatch, while the next layer's parameters stream in from the host
 * eager param-server (EPS) and the finished layer's gradients stream out.
 *
 * Conventions
 *  - Every function returns L2L_OK (0) or a negative l2l_status; nothing throws or aborts.
 *    l2l_last_error() gives a human-readable message for the last failure on that context.
 *  - "device pointer" = memory of the GPU the context was created on (e.g. a torch tensor's
 *    data_ptr()); "host pointer" = CPU memory, pinned where stated.  The caller owns every buffer it
 *    passes in; the context owns the two parameter slots, the gradient accumulators and the
 *    per-launch workspace.
 *  - All device work is enqueued on the two streams given to l2l_create: kernels on
 *    `compute_stream`, host<->device copies on `copy_stream`; ordering between them is by events
 *    inside the library.  No call blocks the host except l2l_sync, l2l_drain_wait, l2l_embed_drain_wait
 *    and l2l_create/l2l_destroy.
 *  - Tensors are row-major, token-major.  T = ubatch * seq tokens per micro-batch.  In dtype
 *    L2L_BF16 activations and parameters are bfloat16 with fp32 accumulation everywhere, in
 *    L2L_FP16 IEEE half (the FP16 of the paper's cross mixed precision, Section 2.3; use it with a
 *    loss scale, l2l_set_loss_scale); in L2L_F32 everything is fp32.  Gradients of parameters are
 *    always accumulated in fp32.
 *
 * Packed parameter block of one encoder layer (one contiguous DMA, Section 2.1 "receives each
 * layer's weights from EPS one at a time"), in elements of the configured dtype, every sub-block
 * starting at a multiple of 128 elements:
 *     Wqkv[H,3H] | bqkv[3H] | Wo[H,H] | bo[H] | g1[H] | be1[H] | W1[H,F] | b1[F] | W2[F,H] | b2[H] | g2[H] | be2[H]
 * Weight matrices are [in, out] row-major (y = x W + b).  The Q, K and V projections are the three
 * H-wide column groups of Wqkv; head h owns columns h*d .. h*d+d-1 of its group.  The gradient block
 * uses the same order and offsets in fp32.  Padding elements must be zero in parameters and are
 * zero in gradients.
 *
 * Packed embedding / head block:  E[V,H] | Ppos[S,H] | ge[H] | be[H] | bv[V]   (same alignment rule).
 */
#ifndef L2L_H
#define L2L_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  L2L_OK = 0,
  L2L_E_ARG = -1,    /* null pointer, bad index, unsupported shape */
  L2L_E_STATE = -2,  /* call out of order (slot never staged, nothing to drain, ...) */
  L2L_E_HIP = -3,    /* a HIP runtime call failed; message carries the HIP error string */
  L2L_E_NOMEM = -4
} l2l_status;

enum { L2L_F32 = 0, L2L_BF16 = 1, L2L_FP16 = 2 };

typedef struct l2l_ctx l2l_ctx;

typedef struct {
  int hidden;        /* H; multiple of 8 */
  int heads;         /* A; H % A == 0 and d = H / A a multiple of 8 */
  int ffn;           /* F; multiple of 8 */
  int seq;           /* S; multiple of 8 */
  int ubatch;        /* ub: sequences per micro-batch */
  int num_ubatches;  /* U */
  int dtype;         /* L2L_F32, L2L_BF16 or L2L_FP16 */
  float ln_eps;      /* LayerNorm epsilon */
  int vocab;         /* V; 0 = no embedding / head buffers */
  int ubatch_group;  /* micro-batches handed to one kernel launch (rows are independent, so this
                        changes launch shape and workspace size only); 0 = library default */
} l2l_config;

/* ---- sizes (host-only, usable without a GPU) --------------------------------------------------- */
/* Number of tensors in the layer block (12) / embedding block (5). */
int    l2l_layer_tensor_count(void);
int    l2l_embed_tensor_count(void);
/* Element offset / element count / name of tensor `i` inside the packed block. Negative or NULL on
   a bad index or config. */
long long   l2l_layer_tensor_offset(const l2l_config*, int i);
long long   l2l_layer_tensor_size(const l2l_config*, int i);
const char* l2l_layer_tensor_name(int i);
long long   l2l_embed_tensor_offset(const l2l_config*, int i);
long long   l2l_embed_tensor_size(const l2l_config*, int i);
const char* l2l_embed_tensor_name(int i);
/* P_l = 4H^2 + 2HF + 9H + F (unpadded parameter count of a layer). */
size_t l2l_layer_param_count(const l2l_config*);
/* Elements / bytes of the packed (padded) blocks. grad bytes are fp32. */
size_t l2l_layer_packed_elems(const l2l_config*);
size_t l2l_layer_param_bytes(const l2l_config*);
size_t l2l_layer_grad_bytes(const l2l_config*);
size_t l2l_embed_packed_elems(const l2l_config*);
size_t l2l_embed_param_bytes(const l2l_config*);
size_t l2l_embed_grad_bytes(const l2l_config*);
/* Returns L2L_OK if the config is supported, else L2L_E_ARG. */
int    l2l_config_check(const l2l_config*);

/* ---- context ----------------------------------------------------------------------------------- */
/* compute_stream / copy_stream: hipStream_t handles (may be the same; NULL = the null stream).
   Allocates slots, accumulators and workspace on the current device.
   Tuning and test switches are taken from the environment here, once, and from nowhere else:
     L2L_NO_FUSED_ATTENTION=1  attention as batched GEMMs + softmax kernels with the score matrices in memory
     L2L_HEAD_ROWS=n           labelled rows per pass of the LM head (default min(U T, 8192))
     L2L_SPLIT_WS_MB=n         room for the partial results of K-split GEMMs (default: what the layer's dW GEMMs need)
     L2L_SPLIT_ATOMICS=1       K-split GEMMs add their partial results with fp32 atomics instead
     L2L_FORCE_SPLITS=n        split factor of the accumulating fp32 GEMMs (default: by shape)
     L2L_COPY_ROWS=0           gradient drains issued as plain copies (the runtime's copy kernel) instead of rows of 64 KiB (DMA engine)
     L2L_NO_WEIGHT_TRANSPOSE=1 forward GEMMs read the weights as stored, as a K-strided operand (no [out,in] copies per stage)
     L2L_GEMM_RESIDENT=0       one workgroup per GEMM tile instead of one resident workgroup per compute unit */
int  l2l_create(const l2l_config*, void* compute_stream, void* copy_stream, l2l_ctx** out);
int  l2l_destroy(l2l_ctx*);
/* Device bytes owned by the context (slots + accumulators + workspace): depth-independent. */
size_t l2l_device_bytes(const l2l_ctx*);
const char* l2l_last_error(const l2l_ctx*);
/* Host blocks until both streams are idle.  L2L_E_ARG if, since the last call, a kernel met a token id or label
   outside its range (ids in [0, V), labels < V resp. < num_classes): such ids are clamped on the device, never
   followed out of a table, and the results computed from them mean nothing. */
int  l2l_sync(l2l_ctx*);

/* A HIP stream whose kernels run on a subset of the compute units only: of every 32 consecutive bits of
   the CU mask the first `cus_per_32` (1..32) are set, which spreads the subset over all XCDs whichever
   way the runtime enumerates them.  Meant for the copy stream: on systems where the runtime moves
   host<->device copies with a copy kernel, that kernel otherwise takes workgroup slots on every CU and
   kernels launched while it runs wait for it (the transfers of Section 2.2 are supposed to hide behind
   compute, not in front of it).  *out receives a hipStream_t; release it with l2l_stream_destroy.
   L2L_E_ARG for a bad count or a null pointer, L2L_E_HIP if the runtime refuses. */
int  l2l_stream_create_cu_masked(int cus_per_32, void** out);
int  l2l_stream_destroy(void* stream);
/* Asynchronous copy between pinned host memory and device memory on `stream` (a hipStream_t), issued as rows of
   64 KiB so that the runtime carries it out with a DMA engine in either direction (a plain device-to-host
   hipMemcpyAsync is carried out by a copy kernel here, whose workgroups occupy compute units for the length of the
   transfer).  For the stash offload and reload of Section 2.1's constant-memory mode, which move a layer boundary
   activation per layer visit beside the layer's kernels.  to_host: 1 = device to host, 0 = host to device.
   L2L_E_ARG for null pointers, L2L_E_HIP if the runtime refuses. */
int  l2l_memcpy_rows_async(void* dst, const void* src, size_t bytes, int to_host, void* stream);

/* ---- the four calls of the relay (Algorithm 2; Section 2.1) -------------------------------------- */

/* Param stage: asynchronous host->device copy, on copy_stream, of one layer's packed parameters
   (l2l_layer_param_bytes bytes, host pointer, pinned for the copy to overlap compute) into device
   slot 0 or 1.  The copy is ordered after every kernel that still reads the slot. `layer` >= 0 is a
   tag used to match later fwd/bwd calls. */
int l2l_param_stage(l2l_ctx*, int layer, const void* host_params, int slot);

/* Layer forward over all U micro-batches (inner loop of Algorithm 2's forward phase).
   x_stash: device, U contiguous [ub, S, H] blocks = the layer's input (stash of layer-1's output).
   y_out:   device, same shape = this layer's boundary output (the next stash entry).
   Ordered after the slot's stage; x_stash and y_out must not overlap. */
int l2l_layer_fwd(l2l_ctx*, int layer, int slot, const void* x_stash, void* y_out);

/* Layer backward over all U micro-batches with layer-forward recompute (Section 2.1).
   x_stash: as above.  dy_dx: device, U x [ub,S,H]; holds dL/dY on entry and dL/dX on return
   (in place).  The layer's parameter gradients are summed over the U micro-batches into a
   context-owned fp32 accumulator that starts from zero at this call. */
int l2l_layer_bwd(l2l_ctx*, int layer, int slot, const void* x_stash, void* dy_dx);

/* The same two calls with LayerNorm 2's row statistics kept across the passes.  The backward pass needs of the
   layer's last LayerNorm only its normalised input xhat and 1 / sigma per row; xhat can be taken back out of the
   layer's OUTPUT (y = g2 xhat + be2), which Section 2.1 stashes anyway as the next layer's input, so with 1 / sigma
   kept from the forward pass (4 bytes per token: 0.2 % of the stash at H = 1024) the recompute pass can leave out the
   FFN2 product, a twelfth of the layer's GEMM work.  Results equal l2l_layer_bwd's up to rounding (xhat comes from
   the rounded y instead of the rounded LayerNorm input).
   rstd_out / rstd: device float[U * T], caller-owned like the stash.  y_stash: device, U x [ub,S,H], what
   l2l_layer_fwd_stats wrote to y_out.  The caller uses the pair only while no |g2| is tiny (xhat = (y - be2) / g2; the
   step driver checks the master weights and falls back to l2l_layer_bwd otherwise).  Where LayerNorm backward runs in
   its two-kernel form (H > 2048) l2l_layer_bwd_stats recomputes in full, like l2l_layer_bwd. */
int l2l_layer_fwd_stats(l2l_ctx*, int layer, int slot, const void* x_stash, void* y_out, float* rstd_out);
int l2l_layer_bwd_stats(l2l_ctx*, int layer, int slot, const void* x_stash, const void* y_stash, const float* rstd, void* dy_dx);

/* Grad drain: asynchronous device->host copy, on copy_stream, of the gradients accumulated by the
   last l2l_layer_bwd(layer) (l2l_layer_grad_bytes bytes, fp32, packed order; half of that, rounded to the
   16-bit format, after l2l_set_drain_dtype) into host memory
   (pinned to overlap), ordered after that backward.  The accumulator is reusable once the copy
   lands; two accumulators alternate so the next layer's backward need not wait. */
int l2l_grad_drain(l2l_ctx*, int layer, void* host_grads);
int l2l_drain_wait(l2l_ctx*, int layer);   /* host blocks until that drain has landed */

/* ---- first and last resident "layers": embedding and tied LM head (Section 2.1: "a 3 layer model") */
/* Async H2D of the packed embedding block (pinned host pointer) on copy_stream. */
int l2l_embed_stage(l2l_ctx*, const void* host_embed_params);
/* The same for elements [first, first + count) of the packed block only (host_embed_params still points at
   element 0).  Lets the host ship the block piece by piece while its optimizer is still working on the rest
   (the embedding block is the last to be updated in a step and the first to be needed in the next: Section 2.2's
   eager update has nothing left to hide it behind).  The caller stages every element before l2l_embed_fwd.
   L2L_E_ARG for a range outside the block. */
int l2l_embed_stage_part(l2l_ctx*, const void* host_embed_params, long long first, long long count);
/* x0[u][b,s] = LN_e(E[tok] + Ppos[s]).  tokens: device int32 [U, ub, S]; x_out: device U x [ub,S,H].
   Zeroes the embedding-block gradient accumulator (start of a step). */
int l2l_embed_fwd(l2l_ctx*, const int32_t* tokens, void* x_out);
/* Tied head + cross-entropy, forward and backward, over all micro-batches:
   z = x E^T + bv at positions with label >= 0; loss = -(1/N) sum log softmax(z)[label], N = labelled
   positions of the whole minibatch.  labels: device int32 [U, ub, S] (-1 = ignore).
   dy_out: device U x [ub,S,H], receives dL/dx (zero at unlabelled positions).
   loss_out: device float[1].  Adds dE and dbv into the embedding-block accumulator. */
int l2l_head_loss(l2l_ctx*, const void* x_last, const int32_t* labels, void* dy_out, float* loss_out);
/* ---- sequence-classification head (the task head of the paper's GLUE fine-tuning runs, Sections 3.1 and 3.5,
   Table 7; the paper does not write it out, this is the usual BERT one): pooled = tanh(x0 Wp + bp) on the first
   token x0 of each sequence, z = pooled Wc + bc, cross-entropy over the sequences with label >= 0,
   normalised by their count over the whole mini-batch.  An alternative to l2l_head_loss; it needs no
   vocabulary.  Packed block (elements of the configured dtype, sub-blocks at multiples of 128):
       Wp[H,H] | bp[H] | Wc[H,C] | bc[C]          (gradient block: same layout, fp32)               */
int    l2l_cls_tensor_count(void);
const char* l2l_cls_tensor_name(int i);
long long   l2l_cls_tensor_offset(const l2l_config*, int num_classes, int i);   /* -1 on bad arguments */
long long   l2l_cls_tensor_size(const l2l_config*, int num_classes, int i);
size_t l2l_cls_packed_elems(const l2l_config*, int num_classes);                /* 0 on bad arguments */
/* Async H2D of the head's packed parameters (pinned host memory) on the copy stream.  The first call
   fixes num_classes (>= 2) for the context and allocates the head's buffers. */
int l2l_cls_stage(l2l_ctx*, const void* host_params, int num_classes);
/* Forward and backward of the head over all U x ub sequences.  x_last: device U x [ub,S,H];
   seq_labels: device int32 [U x ub], -1 = no label; dy_out: device U x [ub,S,H], receives dL/dx
   (non-zero only in the first-token rows of labelled sequences); loss_out: device float[1].
   Adds the four tensors' gradients into the head's fp32 accumulator.  The loss scale applies. */
int l2l_cls_head_loss(l2l_ctx*, const void* x_last, const int32_t* seq_labels, void* dy_out, float* loss_out);
/* Async D2H of the head's gradients (fp32, packed) into pinned host memory, then clears them. */
int l2l_cls_grad_drain(l2l_ctx*, void* host_grads);
int l2l_cls_drain_wait(l2l_ctx*);

/* Loss scaling (Section 2.3: FP16 on the device needs it, the gradient of the loss being ~1/(N V) per
   logit, below half precision's range): from the next l2l_head_loss on, the gradient of the loss is
   multiplied by `scale` before it is rounded to the device dtype, so every activation and parameter
   gradient downstream carries that factor (the reported loss does not); the host divides it out of the
   drained gradients (eps_grad_unscale).  Default 1.  L2L_E_ARG unless 0 < scale < inf. */
int l2l_set_loss_scale(l2l_ctx*, float scale);

/* Format in which the gradient drains (l2l_grad_drain, l2l_embed_grad_drain and its piecewise form, l2l_cls_grad_drain)
   write to host memory: L2L_F32 (default: the accumulators as they are) or L2L_BF16 / L2L_FP16 (rounded to nearest
   even on the device first, half the bytes over the host link; the paper's device holds and sends 16-bit values,
   Section 2.3).  The gradients still accumulate in fp32 on the device.  With a 16-bit format `host_grads` of the
   drain calls points at 16-bit elements, and element offsets count those.  Call between steps (no drain in flight).
   L2L_E_ARG for another value, L2L_E_NOMEM if the staging buffer cannot be allocated. */
int l2l_set_drain_dtype(l2l_ctx*, int dtype);
/* Backward of l2l_embed_fwd: adds dE (scatter-add over token ids), dPpos, dge, dbe into the
   embedding-block accumulator.  dy: device U x [ub,S,H] (read only). */
int l2l_embed_bwd(l2l_ctx*, const int32_t* tokens, const void* dy);
/* Async D2H of the embedding-block gradients (fp32, packed) into host memory, after the above. */
int l2l_embed_grad_drain(l2l_ctx*, void* host_grads);
int l2l_embed_drain_wait(l2l_ctx*);
/* The same drain in pieces: elements [first, first + count) of the packed gradients go to host_grads + first
   (host_grads points at element 0 of the landing buffer).  Pieces are issued in ascending order without gaps; the
   piece that ends the block also clears and releases the accumulator.  With 16-bit drains pieces start at
   multiples of 4 elements.  L2L_E_ARG for a piece out of order, misaligned or outside the block, L2L_E_STATE
   without un-drained gradients. */
int l2l_embed_grad_drain_part(l2l_ctx*, void* host_grads, long long first, long long count);

/* ---- profiling: HIP-event timing of kernel classes on the compute stream ----------------------
   (the measurements behind the roofline and overlap figures: Section 2.2's cost model speaks of a layer's compute
   time C and transfer time X; these calls measure both per class, and how much of X ran under C)
   GEMM = the layer's dense projections (QKV, out-proj, FFN1, FFN2 and their dX / dW GEMMs);
   ATTN = the per-(sequence, head) score/context products and softmax; ROWWISE = LayerNorm, embedding;
   COLSUM = bias / gain gradient reductions; OTHER = head, cross-entropy, fills. */
enum { L2L_PROF_GEMM = 0, L2L_PROF_ATTN = 1, L2L_PROF_ROWWISE = 2, L2L_PROF_COLSUM = 3, L2L_PROF_OTHER = 4,
       L2L_PROF_COPY = 5,   /* copy stream: stages (with the weight transposes), drains (with the clearing) */
       L2L_PROF_CLASSES = 6 };
/* on = 1: every launch is bracketed by events; on = 2: only the GEMM class (less perturbation);
   on = 0: off.  Counters are reset by every call. */
int l2l_profile(l2l_ctx*, int on);
/* Resolves pending events and returns, for one class: launches, total milliseconds, total
   algorithmic flops and bytes of those launches. */
int l2l_profile_read(l2l_ctx*, int cls, long long* launches, double* ms, double* flops, double* bytes);
/* The GEMM class by launch shape, since the last l2l_profile(ctx, 1 or 2): one text line per distinct shape,
   "M N K a_kc b_kc epi out_f32 pass launches total_ms" (epi: the library's epilogue flag set: bias 1, GELU 2, GELU' 4,
   residual 8, accumulate 16, column sums 32; pass: 0 forward pass, 1 recompute, 2 backward, 3 single operations), in
   order of first use, into buf (cap bytes, NUL-terminated).
   L2L_E_ARG if buf is too small. */
int l2l_profile_gemm_table(l2l_ctx*, char* buf, size_t cap);
/* Overlap of the two streams over everything recorded since l2l_profile(ctx, 1): the time the compute
   stream had a kernel running (union of the bracketed intervals), the time the copy stream was busy,
   the part of the latter that fell inside the former (the transfers Section 2.2 wants hidden), and the
   span from the first start to the last end; all in ms.  Compute intervals closer together than
   merge_gap_ms are joined first (the launch gap between two back-to-back kernels, which the event
   brackets themselves widen, is not time the copy stream could have avoided); 0 joins nothing.
   Any pointer may be null. */
int l2l_profile_overlap(l2l_ctx*, double merge_gap_ms, double* compute_busy_ms, double* copy_busy_ms, double* copy_hidden_ms,
                        double* span_ms);

/* ---- single operations, for kernel-level parity tests and micro-benchmarks ---------------------
   The paper names no kernels; these expose the two building blocks of the encoder layer it executes (a projection
   with its fused epilogue, a LayerNorm: Section 2.1's "encoder layer") one at a time, so that each compiled kernel
   variant can be checked against its definition without the rest of the layer around it. */
/* C[M,N] = epilogue(alpha * A B), device pointers, on compute_stream.
   a_kc: 1 = A stored [M,K] (K contiguous, row stride lda); 0 = A stored [K,M] (row stride lda).
   b_kc: 1 = B stored [N,K] (row stride ldb); 0 = B stored [K,N].
   in_dtype: dtype of A, B, bias, resid;  out_f32: 1 = C is fp32, else in_dtype.
   bias: [N] or NULL; resid: [M,N] with row stride ldc or NULL; accumulate: C += result (needs out_f32).
   gelu: apply GELU after the bias.  impl: 0 = library's choice, 1 = force the plain kernel,
   2 = force the MFMA kernel (L2L_E_ARG if the shape does not allow it); 100 + v = MFMA tile variant v
   (for tuning). */
int l2l_op_gemm(l2l_ctx*, int in_dtype, int out_f32, int a_kc, int b_kc, int M, int N, int K,
                const void* A, long long lda, const void* B, long long ldb, void* C, long long ldc,
                float alpha, const void* bias, const void* resid, int gelu, int accumulate, int impl);
/* The same with every epilogue the layer uses.  epi: OR of the L2L_EPI_ flags.
   resid: [M,N] with row stride ldr, or NULL.
   L2L_EPI_GELU: GELU after the bias; aux_out (or NULL) receives the pre-activation, [M,N] in in_dtype, row stride ldaux.
   L2L_EPI_GELUGRAD: the result is multiplied by gelu'(aux), aux: [M,N] in in_dtype, row stride ldaux (the FFN2
     backward GEMM that turns dG into dU1).  Not together with L2L_EPI_GELU.
   L2L_EPI_KEEPGRAD (with L2L_EPI_GELU and aux_out): aux_out receives gelu'(u) instead of u -- what the recompute
     pass's FFN1 GEMM leaves for the backward pass.
   L2L_EPI_MULAUX: the result is multiplied element-wise by aux ([M,N] in in_dtype, row stride ldaux): the FFN2
     backward GEMM with gelu'(U1) kept that way.  Not together with L2L_EPI_GELU or L2L_EPI_GELUGRAD.
   L2L_EPI_ACCUM: C += result (fp32 C).
   L2L_EPI_COLSUM: also leaves partial column sums of the stored values: colsum is device fp32 [colsum_rows][N];
     *colsum_rows_used (host int, may be NULL) receives how many rows were written; their sum over rows is the column
     sum of C (the bias gradient db1 = colsum(dU1) without a pass over dU1).  Only where the direct-to-LDS MFMA
     kernel takes the launch with 16-byte aligned rows (impl = 0, 16-bit output): otherwise L2L_E_ARG. */
enum { L2L_EPI_GELU = 1, L2L_EPI_GELUGRAD = 2, L2L_EPI_ACCUM = 4, L2L_EPI_COLSUM = 8, L2L_EPI_KEEPGRAD = 16, L2L_EPI_MULAUX = 32 };
int l2l_op_gemm_ex(l2l_ctx*, int in_dtype, int out_f32, int a_kc, int b_kc, int M, int N, int K,
                   const void* A, long long lda, const void* B, long long ldb, void* C, long long ldc,
                   float alpha, const void* bias, const void* resid, long long ldr, int epi,
                   const void* aux, void* aux_out, long long ldaux,
                   float* colsum, long long colsum_rows, int* colsum_rows_used, int impl);
/* For callers that cannot allocate -- code under HIP graph capture, tight serving loops, harnesses that forbid
   hipMalloc: C[M,N] += A B with fp32 C, i.e. l2l_op_gemm(..., out_f32 = 1, accumulate = 1) on its default
   implementation, without a context.  Where that call splits the contraction over K and keeps the splits' partial
   results in context memory, this one keeps them in a device array that is part of the library itself
   (l2l_noalloc_scratch_bytes() bytes = 32 MiB, present once on every GPU the library runs on until the process
   ends); it calls no allocating routine.  stream: hipStream_t (NULL = the null stream) on the current device.
   in_dtype: L2L_BF16 or L2L_FP16; A, B, C, strides and a_kc / b_kc as in l2l_op_gemm; operands must satisfy the MFMA
   kernels' rules (16-byte aligned bases, row pitches that are multiples of 8 elements and cover the extent rounded up
   to 8, panels below 2 GiB), else L2L_E_ARG.  L2L_E_ARG with a message naming the sizes when the K-split the shape
   calls for needs more than the array holds (splits x M x N floats).  The array keeps the last call's contents;
   nothing in it has to start from zero (every element a call reads was written by that call).  All calls on one GPU
   share the array: calls that overlap in time on one GPU race.  The message of the last failure of this call on the
   calling thread: l2l_noalloc_last_error(). */
int    l2l_op_gemm_accum_noalloc(void* stream, int in_dtype, int a_kc, int b_kc, int M, int N, int K,
                                 const void* A, long long lda, const void* B, long long ldb, float* C, long long ldc);
size_t l2l_noalloc_scratch_bytes(void);
const char* l2l_noalloc_last_error(void);
/* y = LN(x) rows of length n; mean/rstd: device float[rows] or NULL. */
int l2l_op_layernorm(l2l_ctx*, int dtype, int rows, int n, const void* x, const void* gamma,
                     const void* beta, float eps, void* y, float* mean, float* rstd);

/* ---- host EPS (Section 2.1, 2.3): fp32 master weights + Adam on host cores ---------------------- */
typedef struct eps_store eps_store;
/* n_blocks parameter blocks with elems[i] packed elements each.  ship_dtype: dtype of the copy that
   is shipped to the device.  Allocates, per block: fp32 master, m, v (pageable) and the shipping
   copy + fp32 gradient landing buffer (pinned).  threads: worker threads for Adam (<=0: all cores). */
int   eps_create(int n_blocks, const size_t* elems, int ship_dtype, int threads, eps_store** out);
int   eps_destroy(eps_store*);
float* eps_master(eps_store*, int block);      /* fp32 master weights (host) */
void*  eps_ship(eps_store*, int block);        /* pinned shipping copy in ship_dtype */
float* eps_grad(eps_store*, int block);        /* pinned fp32 gradient landing buffer */
float* eps_moment(eps_store*, int block, int which); /* Adam m (0) or v (1) */
/* master -> shipping copy (round to nearest even for bf16) for blocks [first, last]. */
int   eps_refresh_ship(eps_store*, int first, int last);
/* One bias-corrected Adam step (no weight decay) on blocks [first, last] from their landing
   buffers, then refreshes their shipping copies.  t >= 1 is the step number. */
int   eps_adam_step(eps_store*, int first, int last, int t, double lr, double beta1, double beta2, double eps_a);
/* The same update for elements [first_elem, first_elem + count) of one block only (its gradients landed, the rest may
   still be on their way). */
int   eps_adam_step_range(eps_store*, int block, long long first_elem, long long count, int t, double lr, double beta1,
                          double beta2, double eps);
/* Multiplies the landing buffers of blocks [first, last] by inv_scale (1 / loss scale) and sets
   *nonfinite to 1 if any of them holds an inf or NaN (an overflow on the device: the caller then skips
   the update and lowers the scale), else 0.  nonfinite may be null. */
int   eps_grad_unscale(eps_store*, int first, int last, double inv_scale, int* nonfinite);
/* The same for elements [first_elem, first_elem + count) of one block (a piece of it that has landed). */
int   eps_grad_unscale_range(eps_store*, int block, long long first_elem, long long count, double inv_scale, int* nonfinite);
/* 16-bit gradient landing buffers (for l2l_set_drain_dtype): eps_enable_grad16 allocates one per block (pinned, 2 bytes
   per element, once), eps_grad16 returns a block's, eps_grad_widen converts what landed there (dtype L2L_BF16 or
   L2L_FP16) into the fp32 gradient buffers of blocks [first, last], which the optimizer steps read; the _range form
   does elements [first_elem, first_elem + count) of one block. */
int   eps_enable_grad16(eps_store*);
void* eps_grad16(eps_store*, int block);
int   eps_grad_widen(eps_store*, int first, int last, int dtype);
int   eps_grad_widen_range(eps_store*, int block, long long first_elem, long long count, int dtype);
/* eps_adam_step_range with the gradients taken from the block's 16-bit landing buffer (grad_dtype L2L_BF16 or L2L_FP16)
   and widened on the fly: the same arithmetic as eps_grad_widen_range followed by eps_adam_step_range, without the
   extra pass over host memory (the fp32 gradient buffer is left as it was). */
int   eps_adam_step_range16(eps_store*, int block, long long first_elem, long long count, int t, double lr, double beta1,
                            double beta2, double eps, int grad_dtype);
/* One LAMB step (the optimizer of Table 1; update rule of the LAMB publication the paper cites, with
   bias correction): per tensor, u = mhat / (sqrt(vhat) + eps_a) + weight_decay * w and
   w -= lr * (||w|| / ||u||) * u, the ratio taken as 1 where either norm is zero.  The tensors of a
   block are the n_seg element ranges [seg_begin[i], seg_end[i]) (host arrays, the same for every block
   in [first, last]; elements outside every range, i.e. the packing's padding, are left alone).
   seg_decay[i] scales weight_decay for range i (null: 1 for all; pass 0 for biases and LayerNorm
   parameters to exempt them).  Norms are accumulated in double.  Refreshes the shipping copies.
   L2L_E_ARG on overlapping, unordered or out-of-range segments. */
int   eps_lamb_step(eps_store*, int first, int last, int t, double lr, double beta1, double beta2, double eps_a,
                    double weight_decay, int n_seg, const long long* seg_begin, const long long* seg_end,
                    const double* seg_decay);
size_t eps_host_bytes(const eps_store*);
/* 1 if the shipping and landing buffers are pinned (a GPU was visible at eps_create), else 0: without
   a GPU the store still works as host logic on ordinary memory. */
int   eps_is_pinned(const eps_store*);

#ifdef __cplusplus
}
#endif
#endif /* L2L_H */
