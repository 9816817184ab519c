/*
 * ae_attn.h -- C ABI of the fused parallel-pattern attention forward operator
 * for AMD MI355X (gfx950).
 *
 * The operator is the parallel pattern of the paper's unified attention
 * template (Section 4.1, "Attention Patterns and Templates"): relevance
 * scoring S = Q K^T, a customizable function on the scores made of an
 * elementwise `modification` (which may be annotated as a mask) and a
 * `row-wise normalization` (Section 4.1, "Customizable functions and
 * flexibility"), then aggregation O = P V.  The score matrix never reaches
 * device memory: the normalization runs in its online form (prologue / per
 * key-block update / epilogue, Section 4.1 "online row-norm interface").
 * The customization points are closed enums here instead of a DSL.
 *
 * All entry points are host functions.  They return a status code, never
 * throw and never abort.  Q, K, V, O are DEVICE pointers owned by the caller;
 * everything else is host memory.
 */
#ifndef AE_ATTN_H
#define AE_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ae_attn ae_attn_t; /* opaque; host memory only */

/* The HIP runtime's stream type, declared here as the runtime declares it so
 * that this header needs no HIP include (a repeated identical typedef is legal
 * in C11 and C++).  NULL is the default stream.                               */
typedef struct ihipStream_t *hipStream_t;

typedef enum {
  AE_OK = 0,
  AE_ERR_INVALID_ARG = 1, /* null/misaligned pointer, bad size, bad parameter  */
  AE_ERR_UNSUPPORTED = 2, /* well-formed, but no kernel for this combination    */
  AE_ERR_HIP = 3,         /* the HIP runtime reported an error on launch        */
  AE_ERR_NOMEM = 4        /* host allocation of the handle failed               */
} ae_status_t;

/* Elementwise modification of the scaled scores s' = scale * s
 * (Section 4.1, "Examples of Attention variants").                           */
typedef enum {
  AE_MOD_NONE = 0,       /* s'                                                 */
  AE_MOD_BIAS = 1,       /* s' + bias            (constant additive bias)      */
  AE_MOD_HEAD_DECAY = 2, /* s' * gamma[h_q]^(i + L_k - L_q - j): the retention
                            mask of RetNet parallel attention; needs CAUSAL    */
  AE_MOD_RELU = 3,       /* max(s', 0)           (ReLU attention)              */
  AE_MOD_BIAS_TENSOR = 4 /* s' + bias[b, h_q, i, j]: an additive bias per
                            (query, key) pair (relative position, ALiBi ...),
                            a device tensor passed to ae_attn_forward_bias     */
} ae_score_mod_t;

/* Row-wise normalization of the modified scores over the visible keys.      */
typedef enum {
  AE_NORM_SOFTMAX = 0,    /* exp(x - rowmax) / rowsum, computed online         */
  AE_NORM_SIGMOID = 1,    /* 1 / (1 + exp(-x)), no row reduction               */
  AE_NORM_ABSSUM = 2,     /* x / max(sum_j |x|, 1)   (reduceAbssum, clamp 1)   */
  AE_NORM_ABS_OF_SUM = 3, /* x / max(|sum_j x|, 1)   (alternative reading)     */
  AE_NORM_NONE = 4        /* x                                                 */
} ae_norm_t;

/* Mask annotation of the modification.  A masked (query, key) pair
 * contributes nothing: its weight is 0 and it takes no part in any row
 * reduction.  A query row with no visible key produces a zero output row.    */
typedef enum {
  AE_MASK_NONE = 0,
  AE_MASK_CAUSAL = 1, /* key j visible to query i iff j <= i + (L_k - L_q)     */
  AE_MASK_SLIDING_WINDOW = 2 /* causal, and only the `window` nearest keys:
                                i + (L_k - L_q) - window < j <= i + (L_k - L_q)  */
} ae_mask_t;

/* Element type of O.  The kernel computes the normalised rows in fp32 either
 * way; AE_OUT_BF16 rounds them to bf16 (nearest even) when they are stored.   */
typedef enum { AE_OUT_F32 = 0, AE_OUT_BF16 = 1 } ae_out_dtype_t;

#define AE_MAX_DECAY_HEADS 256
#define AE_KV_SPLITS_AUTO (-1) /* ae_attn_desc_t.kv_splits: let the library decide */

/*
 * Problem descriptor (host memory, copied by ae_attn_create).
 *
 * Layouts (bf16 inputs, fp32 or bf16 output, innermost dimension contiguous):
 *   Q [B, H_q,  L_q, D_qk]   K [B, H_kv, L_k, D_qk]
 *   V [B, H_kv, L_k, D_v ]   O [B, H_q,  L_q, D_v ]
 * Query head h_q reads key/value head h_q / (H_q / H_kv) (contiguous groups).
 * Strides are in ELEMENTS, ordered {batch, head, row}; an all-zero triple
 * means "contiguous [B, H, L, D]".  Row strides of Q, K, V must be multiples
 * of 8 elements and that of O a multiple of 4, so that every row starts on a
 * 16-byte boundary.
 */
typedef struct {
  int32_t B, H_q, H_kv, L_q, L_k, D_qk, D_v;
  ae_score_mod_t score_mod;
  float bias;          /* used by AE_MOD_BIAS                                   */
  const float *gamma;  /* host array [H_q], each finite and > 0; read only by
                          AE_MOD_HEAD_DECAY (H_q <= AE_MAX_DECAY_HEADS)         */
  ae_norm_t norm;
  ae_mask_t mask;
  float scale;         /* finite and non-zero; multiplies the scores            */
  ae_out_dtype_t out_dtype;
  int32_t window;      /* keys per query, >= 1; read only by
                          AE_MASK_SLIDING_WINDOW                                */
  int32_t kv_splits;   /* 0 or 1: every workgroup walks all keys of its rows.
                          n > 1 (at most 256): the keys are cut into n ranges
                          walked by different workgroups, whose partial results
                          a second kernel combines -- for few query rows and
                          many keys (decoding).  AE_NORM_SOFTMAX with
                          AE_MASK_NONE or AE_MASK_CAUSAL only; such a handle
                          runs through ae_attn_forward_split.
                          AE_KV_SPLITS_AUTO: the library picks (it splits only
                          where it may and where the query tiles leave most of
                          the device idle); ask ae_attn_workspace_bytes whether
                          it did.                                               */
  int64_t q_stride[3], k_stride[3], v_stride[3], o_stride[3];
  int64_t bias_stride[3]; /* AE_MOD_BIAS_TENSOR: element strides {batch, head,
                          row} of the bf16 bias tensor [B, H_q, L_q, L_k] (last
                          dimension contiguous).  All zero: contiguous.  A batch
                          or head stride of 0 beside a non-zero row stride shares
                          the tensor over that dimension.  The row stride must be
                          >= L_k, every stride a multiple of 8; rows are read in
                          pieces of 8 elements, so the last row must be backed by
                          memory up to the next multiple of 8 as well.          */
} ae_attn_desc_t;

/* Instantiates the parallel pattern of Section 4.1 ("Attention Patterns and
 * Templates") for one problem: the descriptor fixes the two customizable
 * functions (modification with its mask annotation, row-wise normalization) and
 * the shapes; the tile shape comes from a table keyed by (D_qk, D_v, mask), the
 * static stand-in for the enumerate-and-profile tile scheduling of Section 4.3
 * (Algorithm 1).  Validates the descriptor, picks the kernel and its tile shape
 * for (D_qk, D_v, mask, norm, score_mod) and returns a handle in *out.  Touches
 * no device.  Supported head dims (D_qk/D_v): 64/64, 128/128, 128/256, 192/128;
 * and, for the retention variants only (HEAD_DECAY with ABSSUM, ABS_OF_SUM or
 * NONE, CAUSAL; Table 2, "Retention Parallel"): 256/128 and 256/512, the latter
 * evaluated as four launches over 128 value columns each (no split keys).
 * Supported (score_mod, norm) pairs: NONE or BIAS with every norm;
 * HEAD_DECAY with ABSSUM, ABS_OF_SUM or NONE (CAUSAL mask only); RELU with NONE.
 * AE_MASK_SLIDING_WINDOW: score_mod NONE or BIAS with SOFTMAX, SIGMOID or NONE.
 * AE_MOD_BIAS_TENSOR: with SOFTMAX, SIGMOID or NONE, masks NONE or CAUSAL, head
 * dims 64/64, 128/128 or 192/128, no split keys.
 * One (batch, head) slab of Q, K, V (and of the bias tensor) must span less than
 * 4 GiB: rows x row stride x 2 bytes (AE_ERR_UNSUPPORTED otherwise).
 * Errors: AE_ERR_INVALID_ARG, AE_ERR_UNSUPPORTED, AE_ERR_NOMEM; *out is set
 * to NULL on error.                                                           */
ae_status_t ae_attn_create(const ae_attn_desc_t *desc, ae_attn_t **out);

/* The parallel pattern itself (Section 4.1, "Attention Patterns and
 * Templates": Q@K, the customizable function on the scores, then S@V; the
 * normalization in the online form of the row-norm interface, Section 4.1),
 * as one fused kernel.
 * Enqueues O = rownorm(mod(scale * Q K^T)) V on `stream` (may be NULL for the
 * default stream) of the current device and returns without synchronising.  Q, K, V, O: device pointers, 16-byte aligned, sized as the
 * descriptor says; O must not alias the inputs.  The handle is not modified:
 * concurrent calls on one handle from several threads or streams are allowed.
 * Allocates no device memory.  Errors: AE_ERR_INVALID_ARG (nothing is
 * launched), AE_ERR_HIP.                                                       */
ae_status_t ae_attn_forward(const ae_attn_t *h, const void *Q, const void *K,
                            const void *V, void *O, hipStream_t stream);

/* ae_attn_forward that also writes, per query row, the final result of the row
 * reduction its normalization keeps (the online row-norm interface's final row
 * scales, Section 4.1) -- what a backward pass recomputes the weights from:
 *   AE_NORM_SOFTMAX     ln sum_j exp(x_ij)  over the visible keys (-inf if none),
 *   AE_NORM_ABSSUM      sum_j |x_ij|        (before the clamp at 1),
 *   AE_NORM_ABS_OF_SUM  sum_j x_ij          (signed, before |.| and the clamp),
 * with x the modified scores.  stats: device pointer, fp32 [B, H_q, L_q]
 * contiguous, 4-byte aligned, not aliasing the other buffers.  Same launch, same
 * ownership and error rules as ae_attn_forward; AE_ERR_UNSUPPORTED for
 * normalizations without a row reduction (SIGMOID, NONE).                      */
ae_status_t ae_attn_forward_stats(const ae_attn_t *h, const void *Q,
                                  const void *K, const void *V, void *O,
                                  void *stats, hipStream_t stream);

/* Forward for a handle created with AE_MOD_BIAS_TENSOR: ae_attn_forward with the
 * additive bias tensor (device, bf16, 16-byte aligned, laid out as
 * desc.bias_stride says, read only) and optionally the row statistic (stats may be
 * NULL; see ae_attn_forward_stats).  One kernel, nothing allocated.  Errors as
 * ae_attn_forward; AE_ERR_INVALID_ARG for a handle of another score_mod.        */
ae_status_t ae_attn_forward_bias(const ae_attn_t *h, const void *Q, const void *K,
                                 const void *V, const void *bias, void *O,
                                 void *stats, hipStream_t stream);

/* Bytes of device workspace that ae_attn_forward_split needs for this handle:
 * the partial output rows and their log-sum-exp, fp32,
 * n * B * H_q * L_q * (D_v + 1) elements for n ranges of keys (0 if the keys
 * are not split).                                                              */
ae_status_t ae_attn_workspace_bytes(const ae_attn_t *h, size_t *bytes);

/* Forward for a handle created with kv_splits > 1 (it also serves any other
 * handle, ignoring the workspace): the attention kernel writes per-range
 * partial results to `workspace`, a second kernel combines them into O (and
 * into `stats`, which may be NULL; see ae_attn_forward_stats).  workspace:
 * device pointer owned by the caller, 16-byte aligned, at least
 * ae_attn_workspace_bytes() bytes, not aliasing the other buffers; its contents
 * need not be initialised and are overwritten.  Both kernels are enqueued on
 * `stream`; nothing is allocated.  Calls that share a workspace must not
 * overlap in time.  Errors as ae_attn_forward.                                 */
ae_status_t ae_attn_forward_split(const ae_attn_t *h, const void *Q,
                                  const void *K, const void *V, void *O,
                                  void *stats, void *workspace,
                                  size_t workspace_bytes, hipStream_t stream);

/* ae_attn_forward_split for callers that cannot allocate device memory or pass
 * a workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  The same two kernels; the partial rows and their
 * log-sum-exp live in a static device array of the library
 * (AE_ATTN_STATIC_SCRATCH_BYTES per device that runs the library, held until
 * the process ends) instead of a workspace.  The call allocates nothing and
 * frees nothing.  A handle whose ae_attn_workspace_bytes() exceeds
 * AE_ATTN_STATIC_SCRATCH_BYTES is refused with AE_ERR_UNSUPPORTED (nothing is
 * launched); a handle without split keys runs as ae_attn_forward[_stats].
 * Every call on one device shares that device's array, which keeps the last
 * call's contents (nothing in it needs clearing: each call overwrites what it
 * reads): calls that overlap in time on one device -- different streams or
 * threads -- race; serialise them.  Q, K, V, O, stats, stream and errors as
 * ae_attn_forward_split; AE_ERR_HIP also if the array's address cannot be
 * looked up on the current device.                                            */
#define AE_ATTN_STATIC_SCRATCH_BYTES (4u << 20)
ae_status_t ae_attn_forward_split_static(const ae_attn_t *h, const void *Q,
                                         const void *K, const void *V, void *O,
                                         void *stats, hipStream_t stream);

/* Bytes of device workspace that ae_attn_backward needs for this handle: one
 * fp32 value per query row (B * H_q * L_q elements) for the normalizations that
 * keep a row statistic (SOFTMAX, ABSSUM, ABS_OF_SUM), 0 for the others.                                                                  */
ae_status_t ae_attn_backward_workspace_bytes(const ae_attn_t *h, size_t *bytes);

/* Backward pass of the operator (the backward graph of Section 4.1's online
 * row-norm interface: derived from the forward definition, reading the final row
 * scales): for an upstream gradient dO, the gradients of sum(O * dO) with
 * respect to Q, K and V,
 *   dV = P^T dO,  dS' = P * (dO V^T - delta)  (softmax; delta_i = dO_i . O_i)
 *                     = dO V^T * P * (1 - P)  (sigmoid)
 *                     = dO V^T [* step(S')]   (no normalization [with ReLU])
 *                     = (dO V^T - g * [r > 1] * delta) / max(r, 1)
 *                       (abs-sum family; r the row statistic, g = sign(S') or
 *                       the sign of the row sum),
 *   dQ = scale * dS' K,  dK = scale * dS'^T Q,
 * with the weights P recomputed from Q, K and the forward pass's row statistic;
 * dK and dV of a k/v head are summed over the query heads that share it.
 * Supported: every (score_mod, norm) pair, mask and pair of head dims that
 * ae_attn_create accepts (AE_MOD_BIAS_TENSOR through ae_attn_backward_bias);
 * per-head decay multiplies dS' as it multiplies S'; kv_splits plays no part.
 *   Q, K, V   device, bf16, laid out as the descriptor says (the forward inputs);
 *   O         device, the forward output, dtype and strides as the descriptor
 *             says (read where a row statistic exists; may be NULL otherwise);
 *   dO        device, bf16, contiguous [B, H_q, L_q, D_v];
 *   stats     device, fp32 [B, H_q, L_q] as written by ae_attn_forward_stats
 *             (where one exists; may be NULL otherwise);
 *   dQ, dK, dV  device, fp32, contiguous, shaped like Q, K, V; every element is
 *             written (rows that see no key get zeros);
 *   workspace device, owned by the caller, 16-byte aligned, at least
 *             ae_attn_backward_workspace_bytes() bytes, overwritten.
 * All pointers 16-byte aligned (stats: 4); outputs must not alias anything.  Up
 * to three kernels are enqueued on `stream`; nothing is allocated, the call does
 * not synchronise, the handle is not modified.  Calls that share a workspace
 * must not overlap in time.  Errors: AE_ERR_INVALID_ARG, AE_ERR_UNSUPPORTED
 * (nothing is launched), AE_ERR_HIP.                                            */
ae_status_t ae_attn_backward(const ae_attn_t *h, const void *Q, const void *K,
                             const void *V, const void *O, const void *dO,
                             const void *stats, void *dQ, void *dK, void *dV,
                             void *workspace, size_t workspace_bytes,
                             hipStream_t stream);

/* ae_attn_backward for a handle created with AE_MOD_BIAS_TENSOR: the same, with
 * the bias tensor of the forward pass (device, bf16, 16-byte aligned, read only).
 * dBias (may be NULL): device, bf16, [B, H_q, L_q, dbias_row_stride], 8-byte
 * aligned, row stride a multiple of 4 elements and >= L_k: receives the gradient
 * with respect to the bias, which is dS', per batch element and query head -- for
 * a bias shared over batch or heads the caller sums over the sharers.  Entries
 * hidden by the mask are NOT written (their gradient is 0): clear the buffer
 * before the call where a mask is in use.                                       */
ae_status_t ae_attn_backward_bias(const ae_attn_t *h, const void *Q, const void *K,
                                  const void *V, const void *bias, const void *O,
                                  const void *dO, const void *stats, void *dQ,
                                  void *dK, void *dV, void *dBias,
                                  int64_t dbias_row_stride, void *workspace,
                                  size_t workspace_bytes, hipStream_t stream);

/* Frees the handle made by ae_attn_create (host memory only; no device work is
 * waited for: kernels already enqueued keep running, their arguments were
 * copied at launch).  NULL is a no-op.                                        */
ae_status_t ae_attn_destroy(ae_attn_t *h);

/* Tile shape and launch geometry chosen at create time (for harnesses).
 * Any output pointer may be NULL.                                             */
ae_status_t ae_attn_query(const ae_attn_t *h, int32_t *block_m, int32_t *block_n,
                          int32_t *lds_bytes, int32_t *grid_size, int32_t *block_threads);

/* Name of the device kernel a handle launches (for matching profiler rows);
 * owned by the library, valid for the life of the process.                    */
const char *ae_attn_kernel_name(const ae_attn_t *h);

/* Measurement aid, not part of the operator: enqueues a kernel that does nothing
 * but bf16 MFMAs (v_mfma_f32_32x32x16_bf16, operands in registers, values that
 * toggle like data), `iters` x 16 per wavefront, 8 wavefronts per workgroup, and
 * stores *flop = the floating-point operations it performs.  Timed by the
 * caller, it gives the rate the matrix pipes sustain under the board's power
 * limit -- the practical ceiling next to the nominal peak.  sink: device buffer of
 * at least workgroups * 512 floats (written, contents meaningless).
 * Errors: AE_ERR_INVALID_ARG, AE_ERR_HIP.                                      */
ae_status_t ae_calib_mfma_bf16(void *sink, size_t sink_bytes, int32_t workgroups,
                               int32_t iters, double *flop, hipStream_t stream);

/* Message of the calling thread's most recent failing call ("" if none).     */
const char *ae_attn_last_error(void);

/* Library version as major * 100 + minor.                                     */
int32_t ae_attn_version(void);

/* ---- Recurrent pattern: chunk-parallel retention ------------------------------
 *
 * The paper's second pattern (Section 4.1, "Attention Patterns and Templates":
 * K@V first, then Q@h, iterated over a compressed state h; Table 2, "Retention
 * Recurrent"), with a constant decay per head as the state modification
 * (Section 4.1, h_mod: h x decay):
 *     h_t = gamma[head] * h_{t-1} + k_t^T v_t   (h_0 = 0, h: [D_qk x D_v])
 *     o_t = scale * q_t h_t
 * evaluated chunk by chunk so that the matrix units do the work (Section 4.2,
 * kernel templates for recurrent patterns): one kernel walks the chunks and
 * leaves the state in front of each (bf16, [D_qk x D_v]); the parallel-pattern
 * kernel then starts every chunk's rows from the read-out of that state and
 * walks the chunk's own keys on top of it.  The work grows linearly with L.
 * Where B x H is at least 192 the call runs instead as ONE kernel that walks the
 * chunks of a (batch, head) in order with the state on chip (the kernel behind
 * ae_gated_forward, with the head's constant decay): same result up to rounding
 * order, Q, K, V read once; the workspace is then not touched (but must still
 * be passed: the choice is the library's).
 *
 * Layouts: Q, K [B, H, L, D_qk] and V [B, H, L, D_v] bf16, O [B, H, L, D_v]
 * fp32 (or bf16, desc.out_dtype), all contiguous, device memory, 16-byte aligned; the caller owns them.
 * gamma: host array [H], each in (0, 1] (read by create only).  chunk: 64, 128
 * or 256 tokens (256 fills the parallel kernel's 256-row tile).  Head dims
 * 64/64 and 128/128; H <= AE_MAX_DECAY_HEADS.
 * The workspace (device memory, 256-byte aligned, owned by the caller, size
 * from ae_recurrent_workspace_bytes) holds the state in front of every chunk:
 * 2 bytes x B x H x chunks x D_qk x D_v.
 * ae_recurrent_forward_state also takes the state in front of the first token
 * (h_in, fp32 [B, H, D_qk, D_v], device memory, 16-byte aligned; NULL: zero)
 * and hands back the one after the last token (h_out, same layout; NULL: not
 * computed), so that a sequence can be processed in pieces (prefill, then more
 * tokens): the pieces' outputs equal those of one call up to rounding.  h_out
 * may be the buffer h_in points to.  Calls that share a
 * workspace must not overlap.  Nothing allocates device memory; all kernels are
 * enqueued on `stream` (a hipStream_t, NULL = default stream) and the call
 * returns without waiting.
 * Errors: AE_ERR_INVALID_ARG (nothing is launched), AE_ERR_UNSUPPORTED,
 * AE_ERR_NOMEM (create), AE_ERR_HIP.                                            */
typedef struct ae_recurrent ae_recurrent_t;
typedef struct {
  int32_t B, H, L, D_qk, D_v;
  int32_t chunk;
  float scale;        /* finite and non-zero */
  const float *gamma; /* host array [H] */
  ae_out_dtype_t out_dtype; /* element type of O: AE_OUT_F32 (0), or AE_OUT_BF16 (fp32 rows rounded when stored) */
} ae_recurrent_desc_t;

ae_status_t ae_recurrent_create(const ae_recurrent_desc_t *desc, ae_recurrent_t **out);
ae_status_t ae_recurrent_workspace_bytes(const ae_recurrent_t *h, size_t *bytes);
ae_status_t ae_recurrent_forward(const ae_recurrent_t *h, const void *Q, const void *K, const void *V, void *O,
                                 void *workspace, size_t workspace_bytes, hipStream_t stream);
ae_status_t ae_recurrent_forward_state(const ae_recurrent_t *h, const void *Q, const void *K, const void *V,
                                       const void *h_in, void *O, void *h_out, void *workspace,
                                       size_t workspace_bytes, hipStream_t stream);
/* One token of the recurrence as Section 4.1 states it (K@V into the state,
 * then Q@h), for decoding: state <- gamma * state + k^T v, o = scale * q state.
 * q, k bf16 [B, H, D_qk], v bf16 [B, H, D_v], state fp32 [B, H, D_qk, D_v]
 * (updated in place; the layout of h_in / h_out above), o fp32 [B, H, D_v]; all
 * contiguous device memory, 16-byte aligned.  Uses B, H, the head dims, gamma
 * and scale of the handle (L and chunk play no part).  No workspace.             */
ae_status_t ae_recurrent_step(const ae_recurrent_t *h, const void *q, const void *k, const void *v, void *state,
                              void *o, hipStream_t stream);
ae_status_t ae_recurrent_destroy(ae_recurrent_t *h); /* NULL is allowed */

/* ---- Recurrent pattern with per-token gates: gated retention, Mamba2 SSM -----------
 *
 * The recurrent pattern (Section 4.1, "Attention Patterns and Templates") with
 * the key and state modifications of Section 4.1's Mamba2 example (k_mod = k x
 * gate, h_mod = h x decay x gate; Table 2 rows "Mamba2 SSM", "Gated Retention"):
 *     h_t = a_t * h_{t-1} + (g_t * k_t)^T v_t        a_t = exp(log_decay_t)
 *     o_t = scale * q_t h_t
 * per batch entry and value head, h: [D_qk x D_v], h before the first token =
 * h_in (zero if NULL).  The paper's "decay x gate" on the state is ONE factor
 * a_t in (0, 1] per token here, passed as its natural logarithm (<= 0):
 *   gated retention   log_decay = ln of the token's gate, key_gate = NULL;
 *   Mamba2 SSM        q = C, k = B, v = x, log_decay = dt * A, key_gate = dt,
 *                     H_qk = the number of B/C groups;
 *   retention         log_decay = ln gamma[head] for every token.
 * One kernel walks each (batch, head) in chunks of 64 tokens (Section 4.2: chunk
 * parallelism) with the state on chip: Q, K, V are read once, O is written
 * once, no workspace exists and nothing is allocated.
 *
 *   Q, K       device, bf16, contiguous [B, H_qk, L, D_qk]; value head h reads
 *              q/k head h / (H / H_qk) (H_qk divides H; H_qk = H: one each);
 *   V          device, bf16, contiguous [B, H, L, D_v];
 *   log_decay  device, fp32, contiguous [B, H, L], every value <= 0 (not checked:
 *              a positive value makes a_t > 1 and the chunk arithmetic may
 *              overflow);
 *   key_gate   device, fp32 [B, H, L], or NULL for all ones;
 *   h_in       device, fp32 [B, H, D_qk, D_v], or NULL; h_out the same layout or
 *              NULL (not written); h_out may be the buffer h_in points to;
 *   O          device, [B, H, L, D_v], fp32 or (desc.out_dtype) bf16.
 * Q, K, V, O and the states 16-byte aligned, the gates 4-byte; O and h_out must
 * not alias the inputs.  D_qk and D_v each 64 or 128.  The launch is enqueued on
 * `stream`; the call returns without waiting.  Errors: AE_ERR_INVALID_ARG
 * (nothing is launched), AE_ERR_UNSUPPORTED, AE_ERR_NOMEM (create), AE_ERR_HIP. */
typedef struct ae_gated ae_gated_t;
typedef struct {
  int32_t B, H, H_qk, L, D_qk, D_v;
  float scale;              /* finite and non-zero */
  ae_out_dtype_t out_dtype; /* element type of O */
} ae_gated_desc_t;

ae_status_t ae_gated_create(const ae_gated_desc_t *desc, ae_gated_t **out);
ae_status_t ae_gated_forward(const ae_gated_t *h, const void *Q, const void *K, const void *V,
                             const void *log_decay, const void *key_gate, const void *h_in,
                             void *O, void *h_out, hipStream_t stream);

/* The same call for few (batch, head) pairs and long sequences.  One workgroup
 * walks a (batch, head) from the first token to the last, so B x H of them keep
 * B x H compute units busy, however long L is.  Where that leaves most of the
 * chip idle (create decides: fewer than 192 workgroups and L >= 1024) this entry
 * point cuts every walk into segments (Section 4.2: parallelism over chunks of
 * the sequence): all segments are walked side by side for their final states from
 * a zero start, a small kernel chains those into the state in front of every
 * segment (h_s+1 = exp(sum of the segment's log-decays) h_s + the segment's own
 * state), and the segments are walked again, side by side, for the outputs.
 * Same result as ae_gated_forward up to rounding order.
 *   workspace  device, 256-byte aligned, ae_gated_workspace_bytes (0 where create
 *              chose not to cut: then it may be NULL and the call is
 *              ae_gated_forward); owned by the caller; calls sharing it must not
 *              overlap.  Everything else as ae_gated_forward.  Three launches.   */
ae_status_t ae_gated_workspace_bytes(const ae_gated_t *h, size_t *bytes);
ae_status_t ae_gated_forward_segmented(const ae_gated_t *h, const void *Q, const void *K, const void *V,
                                       const void *log_decay, const void *key_gate, const void *h_in,
                                       void *O, void *h_out, void *workspace, size_t workspace_bytes,
                                       hipStream_t stream);

/* Backward pass of the recurrence above: the paper evaluates the recurrent
 * pattern forward and backward (Section 6.1; Table 2) and takes the backward
 * graph from automatic differentiation of the forward one (Section 5.1); here
 * the chain rule is written out.  With A_ij the product of the decays a_t of
 * the tokens j < t <= i, and for an upstream gradient dO of the outputs (the
 * state in front of the first token is zero, no gradient enters the final
 * state):
 *     dq_i = scale sum_{j <= i} A_ij g_j (dO_i . v_j) k_j
 *     dk_j = g_j x_j,  x_j = scale sum_{i >= j} A_ij (dO_i . v_j) q_i,   dkey_gate_j = k_j . x_j
 *     dv_j = g_j scale sum_{i >= j} A_ij (q_i . k_j) dO_i
 *     dlog_decay_t = sum_{i >= t} (q_i . dq_i - k_i . dk_i)
 * (the last line because the cumulative log-decay B_i enters weight (i, j) as
 * exp(B_i - B_j) and the sums are linear in q_i and in k_j).  Each of the first
 * three sums is the forward recurrence on other operands -- queries dO, keys V,
 * values K; and, walking the tokens backwards, queries V, keys dO, values Q;
 * queries K, keys Q, values dO -- so the forward kernel computes them, chunk by
 * chunk with the state on chip; two small kernels form the dot products, the
 * sums over the value heads of a q/k head, and the suffix sums.
 *
 *   Q, K, V, log_decay, key_gate   as in ae_gated_forward;
 *   dO         device, bf16, contiguous [B, H, L, D_v];
 *   dQ, dK     device, fp32, contiguous [B, H_qk, L, D_qk] (summed over the value
 *              heads of each q/k head);  dV  device, fp32, contiguous [B, H, L, D_v];
 *   dlog_decay device, fp32 [B, H, L];  dkey_gate the same, required exactly when
 *              key_gate is given, else NULL;
 *   workspace  device, 256-byte aligned, ae_gated_backward_workspace_bytes: 4 B per
 *              (batch, head, token), plus 8 D_qk B per (batch, head, token) when
 *              H_qk < H (the gradients of q and of the gated key per value head,
 *              which a small kernel sums over each group), plus the segments'
 *              states where the walks are cut (see ae_gated_forward_segmented).
 *              Owned by the caller; calls sharing it must not overlap.
 * Tensors 16-byte aligned, gates and their gradients 4-byte; outputs must alias
 * neither inputs nor each other.  Uses B, H, H_qk, L, the head dims and scale of
 * the handle (out_dtype plays no part: gradients are fp32).  Five launches on
 * `stream`, no allocation, no wait.  Errors as ae_gated_forward.                */
ae_status_t ae_gated_backward_workspace_bytes(const ae_gated_t *h, size_t *bytes);
ae_status_t ae_gated_backward(const ae_gated_t *h, const void *Q, const void *K, const void *V,
                              const void *log_decay, const void *key_gate, const void *dO,
                              void *dQ, void *dK, void *dV, void *dlog_decay, void *dkey_gate,
                              void *workspace, size_t workspace_bytes, hipStream_t stream);
ae_status_t ae_gated_destroy(ae_gated_t *h); /* NULL is allowed */

#ifdef __cplusplus
}
#endif
#endif /* AE_ATTN_H */
