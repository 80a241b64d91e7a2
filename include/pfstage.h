/*
 * pfstage.h - C boundary of the PipeFusion patch-stage library for AMD MI355X (gfx950).
 *
 * One pf_stage object is "the work one GPU does as one pipeline stage": a contiguous stack of
 * DiT blocks (PipeFusion, Sec. 3.3: the model is cut along the data flow into sets of consecutive
 * layers) together with, for every one of those layers, a K/V buffer that spans the FULL token
 * sequence (Sec. 3.4, Table 1: memory (1/N)(KV)L per device).  pf_stage_patch_forward runs the
 * stack on the tokens of one of the M patches: each layer computes fresh Q/K/V for the patch,
 * writes the fresh K/V into its buffer at the patch's rows, and attends the patch's queries over
 * the whole buffer, whose other rows still hold what earlier calls left there - the previous
 * diffusion step's values for patches not yet visited in this step (Sec. 3.3, micro-step example).
 *
 * General conventions
 *  - Every pointer named "device" is GPU memory owned by the caller (e.g. a torch tensor) and must
 *    stay valid until pf_stage_destroy.  The library never allocates or frees device memory and
 *    never synchronises: all work is enqueued on the HIP stream given at creation and results are
 *    valid once that stream has been synchronised by the caller.
 *  - All matrices are row-major.  Weight matrices are stored [out_features, in_features]
 *    (y = x W^T + b), i.e. the contraction index is contiguous for both GEMM operands.
 *  - dtype selects the storage/arithmetic type of weights, biases, projections, K/V and attention
 *    operands: PF_F32 (fp32 everywhere) or PF_BF16 (bf16 operands, fp32 accumulation, fp32 softmax
 *    statistics, LayerNorm statistics, GELU and residual arithmetic).
 *  - The residual stream crosses the boundary in fp32 for both dtypes: x_patch, y_patch, joint text
 *    rows and the conditioning vector are float arrays.
 *  - Every call returns a pf_status; argument and state errors are detected on the host before
 *    anything is launched.  Nothing throws or aborts.  pf_last_error gives a readable message.
 *  - A stage is used by one host thread at a time.
 */
#ifndef PFSTAGE_H
#define PFSTAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pf_stage pf_stage; /* opaque */

typedef enum {
  PF_OK = 0,
  PF_ERR_NULL = -1,      /* a required pointer is NULL */
  PF_ERR_CONFIG = -2,    /* inconsistent pf_config (hidden != heads*head_dim, M does not divide L, ...) */
  PF_ERR_SHAPE = -3,     /* a size argument does not fit the kernels' requirements */
  PF_ERR_DTYPE = -4,     /* unknown dtype */
  PF_ERR_STATE = -5,     /* pf_stage_patch_forward before pf_kv_init */
  PF_ERR_RANGE = -6,     /* patch or layer index out of range */
  PF_ERR_WORKSPACE = -7, /* kv buffer or workspace too small or misaligned */
  PF_ERR_DEVICE = -8     /* a HIP launch reported an error */
} pf_status;

typedef enum { PF_F32 = 0, PF_BF16 = 1 } pf_dtype;

typedef enum {
  PF_BLOCK_ADALN_ZERO = 0,         /* DiT block, modulation = Linear(SiLU(c)) per layer            */
  PF_BLOCK_ADALN_SINGLE_XATTN = 1, /* PixArt-like: shared 6d modulation + per-layer table, and a   */
                                   /* cross-attention to text tokens after the self-attention      */
  PF_BLOCK_MMDIT_JOINT = 2,        /* SD3-like: text and image streams with separate weights, one  */
                                   /* joint attention over [text rows; image rows]                 */
  PF_BLOCK_SINGLE_STREAM = 3       /* Flux-like single stream: attention and MLP in parallel,      */
                                   /* shared weights for text and image rows, 2-D RoPE on q and k  */
} pf_block_kind;

typedef enum {
  PF_PATH_AUTO = 0, /* MFMA kernels for bf16, plain SIMT kernels for fp32 */
  PF_PATH_SIMT = 1, /* force the plain SIMT kernels (debugging aid; still GPU code) */
  /* pf_op_attention / pf_op_attention_static only: as PF_PATH_AUTO, but q already carries the factor
   * log2(e) / sqrt(head_dim), the form in which a stage's QKV projection hands the queries to its self-attention
   * (the scores are then exponents of 2).  bf16 with head_dim 64, 72 or 128 only: PF_ERR_SHAPE otherwise. */
  PF_PATH_AUTO_PRESCALED_Q = 2
} pf_kernel_path;

typedef struct {
  int32_t kind;        /* pf_block_kind */
  int32_t dtype;       /* pf_dtype */
  int32_t n_layers;    /* blocks in this stage, >= 1 */
  int32_t hidden;      /* d = n_heads * head_dim, multiple of 8 */
  int32_t n_heads;     /* H */
  int32_t head_dim;    /* dh: multiple of 8, <= 128 (multiple of 4 is required for RoPE) */
  int32_t mlp_dim;     /* F, multiple of 8 */
  int32_t seq_img;     /* L: image tokens of the whole sequence = grid_h * grid_w */
  int32_t n_patches;   /* M: must divide L; a patch is n = L/M consecutive tokens (Sec. 3.3) */
  int32_t text_len;    /* T: joint text rows (kinds 2, 3) or cross-attention keys (kind 1); else 0 */
  int32_t cross_dim;   /* kind 1: feature width of the text tokens, multiple of 8; else 0 */
  int32_t grid_h, grid_w; /* token grid; image token t sits at (t / grid_w, t % grid_w) (RoPE) */
  float ln_eps;        /* LayerNorm epsilon (biased variance, no learned affine) */
  float rope_theta;    /* kind 3: RoPE base */
  int32_t gelu_tanh;   /* 1: tanh form of GELU, 0: erf form */
  int32_t kernel_path; /* pf_kernel_path */
  int32_t batch;       /* B: images per call, 0 or 1 = one, at most PF_MAX_BATCH.  B = 2 is one image run with and
                          without its condition for classifier-free guidance (Sec. 4.1, CFG parallel, keeps the two on separate device
                          groups; on one device they share the weights and every GEMM).  Each image has K/V buffers of its
                          own.  With B > 1 every per-call array gains a leading image axis: x_patch / y_patch [B, n, d],
                          x_prev / y_prev [B, L, d], cond [B, d or 6d], text / text_out [B, T, ...]. */
  int32_t qk_norm;     /* 1: q and k of every head are RMS-normalised over the head's channels (learned scale
                          q_norm_w / k_norm_w, eps = ln_eps) right after the projection and before any RoPE, as the
                          Flux-family blocks do (the paper names the models, Sec. 4, not this detail).  head_dim must
                          be a power of two.  0: off */
  int32_t joint_rope;  /* kind 2 only, 1: RoPE on q and k of the image rows exactly as in kind 3 (text rows are not
                          rotated): the two-stream block of Flux-like models.  0: off */
  int32_t txt_pre_only_last; /* kind 2 only, 1: in the stage's LAST layer the text stream only supplies keys and
                          values - the final joint block of an MMDiT, whose text output nobody reads (the stage that
                          holds the model's last block sets it).  That layer's txt weights are w_mod [2d, d] / b_mod
                          [2d] (chunks shift, scale), w_qkv / b_qkv (the q rows are not used) and the q / k norm
                          scales; its other txt pointers may be NULL.  The text rows leave the layer unchanged.  0: off */
} pf_config;

#define PF_MAX_BATCH 8

/*
 * Weights of one layer (one stream).  Device pointers, dtype elements, [out, in] row-major.
 *   kinds 0, 2: w_mod [6d, d], b_mod [6d]      modulation = w_mod * SiLU(c) + b_mod
 *   kind 1    : w_mod [6, d] table, b_mod NULL modulation = table + c6  (c6 is the caller's 6d vector)
 *   kind 3    : w_mod [3d, d], b_mod [3d]
 *   modulation chunks, each d wide: [shift1, scale1, gate1, shift2, scale2, gate2] (kind 3:
 *   [shift, scale, gate]).  LN(x)*(1+scale)+shift feeds a branch, gate multiplies its output.
 *   w_qkv [3d, d], b_qkv [3d]: rows [0,d) produce q, [d,2d) k, [2d,3d) v; head h owns channels
 *                              [h*dh, (h+1)*dh) of each.
 *   w_o [d, d], b_o [d]       (unused by kind 3)
 *   w_up [F, d], b_up [F]
 *   w_down [d, F], b_down [d] (kind 3: [d, d+F], acting on the concatenation [attention | GELU(mlp)])
 *   kind 1 only: xattn_wq [d, d], xattn_bq [d]; xattn_wkv [2d, cross_dim], xattn_bkv [2d] (keys then
 *                values); xattn_wo [d, d], xattn_bo [d].  Cross-attention reads the un-normalised
 *                residual, has no modulation and no gate, and sits between self-attention and MLP.
 *   qk_norm only: q_norm_w [dh], k_norm_w [dh]: scales of the per-head RMSNorm (shared by the heads; kind 2: one
 *                pair per stream).
 *   kind 2 only: txt points to a second pf_layer_weights (host memory, copied at creation) holding the
 *                text stream's weights in the same layout.
 */
typedef struct pf_layer_weights {
  const void *w_mod, *b_mod;
  const void *w_qkv, *b_qkv;
  const void *w_o, *b_o;
  const void *w_up, *b_up;
  const void *w_down, *b_down;
  const void *xattn_wq, *xattn_bq, *xattn_wkv, *xattn_bkv, *xattn_wo, *xattn_bo;
  const void *q_norm_w, *k_norm_w;
  const struct pf_layer_weights *txt;
} pf_layer_weights;

/*
 * Per-call conditioning (device pointers).
 *   cond    : float [d] (kinds 0, 2, 3) or float [6d] (kind 1): timestep/conditioning embedding.
 *   text    : kind 1: dtype [T, cross_dim] text features, read by pf_kv_init only (may be NULL in
 *             pf_stage_patch_forward).  kinds 2, 3: float [T, d] text rows of the residual stream, or
 *             NULL: then only the n image rows are processed and the text K/V already in the buffer
 *             is attended to.
 *   text_out: kinds 2, 3 with text != NULL: float [T, d] receives the text rows after the stage
 *             (may alias text).  Otherwise ignored.
 *   same_cond: pf_stage_patch_forward only.  Non-zero: `cond` holds the same values as in the previous call
 *             on this stage (pf_kv_init's warm-up pass included) - the M patch calls of one diffusion step
 *             share the timestep embedding (Sec. 3.3) - so the stage keeps the modulation vectors it derived
 *             then and does not read `cond` (it may be NULL).  Vectors that the previous calls did not derive
 *             (the text stream's, when no text rows rode along) are derived from `cond`, which must then not
 *             be NULL.  Zero: they are derived anew.  The claim is the caller's; it is not checked.
 */
typedef struct {
  const float *cond;
  const void *text;
  float *text_out;
  int32_t same_cond;
} pf_cond;

/* Size of the caller-allocated K/V buffer / workspace for this configuration, in bytes
 * (0 if the configuration is invalid).  Both must be 256-byte aligned. */
size_t pf_stage_kv_bytes(const pf_config *cfg);
size_t pf_stage_workspace_bytes(const pf_config *cfg);

/*
 * Create a stage (Sec. 3.3: one partition of consecutive layers).  `layers` is a host array of
 * n_layers entries whose members are device pointers; the array itself is copied.  kv_buffer and
 * workspace are device memory of at least pf_stage_kv_bytes / pf_stage_workspace_bytes bytes.
 * hip_stream is a hipStream_t (NULL = the default stream).  No device work is enqueued.
 * Errors: PF_ERR_NULL, PF_ERR_CONFIG, PF_ERR_DTYPE, PF_ERR_WORKSPACE.
 */
pf_status pf_stage_create(const pf_config *cfg, const pf_layer_weights *layers, void *kv_buffer,
                          size_t kv_bytes, void *workspace, size_t ws_bytes, void *hip_stream,
                          pf_stage **out);

/*
 * Fill the K/V buffers.
 *   x_prev != NULL: float [L, d] device.  Runs the stage synchronously on the whole sequence of the
 *     previous diffusion step with no stale activations - the warm-up step of Sec. 3.3 - writing every
 *     row of every layer's buffer.  cond_prev->cond is required; kinds 2, 3 also need cond_prev->text
 *     (the text rows are part of the joint sequence; text_out may be NULL).  y_prev, if not NULL,
 *     receives the warm-up pass's output [L, d] (float).
 *   x_prev == NULL: every buffer row is set to zero (App. B: zero-initialised buffer, no warm-up).
 *   kind 1: cond_prev->text is required in both cases; the text keys/values of each layer's
 *     cross-attention are computed here once and kept (text does not change between steps).
 * Padding rows of the buffers are zeroed.  Afterwards the stage is ready for patch calls.
 */
pf_status pf_kv_init(pf_stage *stage, const float *x_prev, const pf_cond *cond_prev, float *y_prev);

/*
 * One pipeline micro-step (Sec. 3.3: one device works on one patch with its own layers; the example of micro-step 5 fixes
 * which rows are fresh) of this stage on patch `patch_idx` (0 <= patch_idx < M):
 * x_patch float [n, d] device in, y_patch float [n, d] device out (may alias).  For every layer:
 * modulation, LayerNorm+modulate, QKV projection (RoPE for kind 3), write of the patch's K/V into buffer
 * rows [off, off+n) BEFORE attention (all other rows are left exactly as they are), attention of the
 * patch's queries over all buffer rows, gated out-projection, (kind 1: cross-attention), gated GELU MLP.
 * Calls may come in any patch order.  Errors: PF_ERR_NULL, PF_ERR_STATE, PF_ERR_RANGE, PF_ERR_DEVICE.
 */
pf_status pf_stage_patch_forward(pf_stage *stage, const float *x_patch, const pf_cond *cond,
                                 int patch_idx, float *y_patch);

/*
 * Read-only view of one layer's buffer: the K/V activations of the whole token sequence, which every device keeps for
 * its own layers (Sec. 3.3; Sec. 3.4, Table 1: (1/N)(KV)L per device).  Borrowed pointers into kv_buffer, valid until
 * destroy; contents valid after a stream synchronise.  Element (row r, head h, channel c) of K lives at
 *   (char*)k + elem_bytes * (r*k_row_stride + h*k_head_stride + c*k_col_stride), likewise for V.
 * Rows [0, text_rows) are the joint text rows (kinds 2, 3), rows [text_rows, rows) the image tokens.
 * K of kind 3 is stored after RoPE.  V is kept transposed (row stride 1) so that the attention kernel
 * reads the contraction index contiguously.
 */
typedef struct {
  const void *k, *v;
  int32_t rows, rows_padded, text_rows, elem_bytes;
  int64_t k_row_stride, k_head_stride, k_col_stride;
  int64_t v_row_stride, v_head_stride, v_col_stride;
} pf_kv_view_t;

pf_status pf_kv_view(const pf_stage *stage, int layer, pf_kv_view_t *out);   /* image 0 */
/* The same for image `image` (0 <= image < B) of a batched stage; cross != 0 selects the cached cross-attention
 * keys/values (kind 1).  Errors: PF_ERR_NULL, PF_ERR_RANGE, PF_ERR_CONFIG. */
pf_status pf_kv_view_image(const pf_stage *stage, int layer, int image, int cross, pf_kv_view_t *out);
/* kind 1: the cached text keys/values of a layer's cross-attention (rows = T). */
pf_status pf_xattn_kv_view(const pf_stage *stage, int layer, pf_kv_view_t *out);

/* Host-only query: how an attention launch of `nq` query rows per image over the self (cross = 0) or cross-attention
 * (cross = 1, kind 1) keys would be split over the key range, the bytes of partial results that split writes
 * and the bytes of workspace reserved for them (ws_needed <= ws_reserved always holds). */
pf_status pf_stage_attention_plan(const pf_stage *stage, int nq, int cross, int *splits, size_t *ws_needed,
                                  size_t *ws_reserved);

/* Change the stream later work is enqueued on (e.g. a capturing stream). */
pf_status pf_stage_set_stream(pf_stage *stage, void *hip_stream);

/*
 * Per-kernel-class timing with HIP events on the stage's stream.  After pf_stage_profile(stage, 1) an event
 * is recorded before the first launch of every call and after each launch (consecutive launches share the
 * event between them); pf_stage_profile_read synchronises the stream, adds up the elapsed time per class
 * since the last read and resets.  Classes: see pf_kernel_class.  An event costs a microsecond or two per
 * launch: use a separate pass from the one that measures whole-call throughput.  ms and launches are host
 * arrays of PF_KC_COUNT entries.
 */
typedef enum {
  PF_KC_MODULATION = 0, PF_KC_LN_MODULATE, PF_KC_GEMM_QKV, PF_KC_KV_SCATTER, PF_KC_ATTENTION,
  PF_KC_ATTN_COMBINE, PF_KC_GEMM_OUT, PF_KC_GEMM_XATTN, PF_KC_XATTN, PF_KC_GEMM_UP, PF_KC_GEMM_DOWN,
  PF_KC_COPY, PF_KC_COUNT
} pf_kernel_class;
pf_status pf_stage_profile(pf_stage *stage, int enable);
pf_status pf_stage_profile_read(pf_stage *stage, double *ms, int64_t *launches);

void pf_stage_destroy(pf_stage *stage); /* NULL-safe */
const char *pf_status_str(pf_status s);
const char *pf_last_error(const pf_stage *stage); /* "" if none; NULL stage: last creation error */

/* ------------------------------------------------------------------------------------------------
 * Single-operator entry points: the kernels of the path, callable on their own for unit parity tests
 * and per-kernel roofline measurement.  All pointers are device memory; `stream` is a hipStream_t.
 * They validate shapes on the host and return PF_ERR_* without launching when something does not fit.
 * ---------------------------------------------------------------------------------------------- */

/* mod[j] = b[j] + sum_i w[j][i] * SiLU(c[i])  (table_mode = 0), or mod[j] = w[j] + c[j] (table_mode = 1,
 * adaLN-single).  w, b in dtype; c, mod float; out_dim entries. */
pf_status pf_op_modulation(int dtype, const void *w, const void *b, const float *c, float *mod,
                           int out_dim, int in_dim, int table_mode, void *stream);

/* out[r][:] = LN(x[r][:]) * (1 + scale) + shift for r < rows (normalize = 1), or a plain conversion of x
 * to dtype (normalize = 0; shift/scale ignored).  x float [rows, d] with row stride ldx, out dtype
 * [rows, d] with row stride ldo. */
pf_status pf_op_ln_modulate(int dtype, const float *x, int64_t ldx, const float *shift, const float *scale,
                            float eps, void *out, int64_t ldo, int rows, int d, int normalize, void *stream);

/*
 * C = epilogue(A W^T + bias).  A dtype [M, K] (row stride lda), W dtype [N, K] (row stride ldw), bias dtype [N].
 *   epilogue 0: C (dtype, row stride ldc) = acc + bias, with GELU applied to columns >= gelu_from
 *               (gelu_from >= N: no GELU).
 *   epilogue 1: X (float, row stride ldc, pointer C) = R + gate ⊙ (acc + bias); R float with row stride ldr
 *               (may be X itself), gate float [N] or NULL (= 1).  If C2 != NULL the new X is also stored
 *               rounded to dtype in C2 (row stride ldc2).
 * K must be a multiple of 8, lda/ldw multiples of 8 elements, A and W 16-byte aligned.
 */
pf_status pf_op_gemm(int dtype, int path, const void *A, int64_t lda, const void *W, int64_t ldw,
                     const void *bias, void *C, int64_t ldc, int M, int N, int K, int epilogue,
                     int gelu_from, int gelu_tanh, const float *gate, const float *R, int64_t ldr,
                     void *C2, int64_t ldc2, void *stream);

/* out[i] = x[i] + alpha * y[i] for i < n (float, device; out may alias x): the element-wise sampler update that sits
 * between the last stage of diffusion step t and the first stage of step t-1 (Sec. 2, Eq. 1; Euler form).  n = 0 is a
 * no-op (pointers may then be NULL); n < 0 gives PF_ERR_SHAPE, a NULL pointer with n > 0 PF_ERR_NULL. */
pf_status pf_op_axpy(const float *x, const float *y, float alpha, float *out, int64_t n, void *stream);
/* out[i] = a * x[i] + b * y[i]: the same update for samplers whose rule is linear in x_t and the network output with a
 * coefficient on x_t (deterministic DDIM-type rules).  Same argument rules as pf_op_axpy. */
pf_status pf_op_axpby(const float *x, const float *y, float a, float b, float *out, int64_t n, void *stream);

/* Name of the kernel instance the library's tile heuristic runs for a GEMM of this shape (static string; matches the
 * template instance seen in a rocprofv3 kernel trace).  Used by the benchmark to group GEMM launches by kernel. */
const char *pf_gemm_kernel_name(int dtype, int path, int M, int N, int K);
/* Likewise for an attention launch of nq query rows per image (q_prescaled: the stage's self-attention, whose queries
 * carry the softmax factor; 0: plain queries).  The string is per-thread storage, valid until the next call. */
const char *pf_attention_kernel_name(int dtype, int path, int head_dim, int nq, int q_prescaled);

/*
 * Write rows of fresh keys/values into a layer's buffer.  qkv dtype [rows, 3d] (row stride ld): q | k | v.
 * Row i goes to buffer row row0 + i of K [H][rows_padded][dh] and of V^T [H][dh][rows_padded]; no other
 * buffer element is written.  With rope != 0 the q and k channels of the rows are first rotated in place
 * in qkv (token index tok0 + i on a grid of width grid_w; tok0 < 0: no rotation, used for text rows),
 * and the rotated k is what reaches the buffer.  With q_norm_w / k_norm_w != NULL (dtype [head_dim], both or
 * neither; head_dim a power of two) q and k of every head are first RMS-normalised over the head's channels,
 * x / sqrt(mean x^2 + norm_eps) * w, before any rotation, also in place.
 */
pf_status pf_op_kv_scatter(int dtype, void *qkv, int64_t ld, void *kbuf, void *vtbuf, int rows_padded,
                           int n_heads, int head_dim, int row0, int rows, int rope, int tok0, int grid_w,
                           float rope_theta, const void *q_norm_w, const void *k_norm_w, float norm_eps,
                           void *stream);

/*
 * out[i][h*dh + c] = sum_j softmax_j(q_i . k_j / sqrt(dh)) v_j[c] over the first `kv_rows` buffer rows.
 * q dtype [nq, H*dh] (row stride ldq), K [H][rows_padded][dh], V^T [H][dh][rows_padded], out dtype (row
 * stride ldo).  splits >= 1 partitions the key range over workgroups; partial results go through
 * `ws` (float, at least pf_op_attention_ws_bytes bytes; may be NULL when splits == 1 on the SIMT path).
 * path PF_PATH_AUTO_PRESCALED_Q: q holds q * log2(e) / sqrt(dh) instead of q (same result up to the rounding
 * of q); a stage config's kernel_path does not take that value (PF_ERR_CONFIG).
 */
size_t pf_op_attention_ws_bytes(int nq, int n_heads, int head_dim, int splits);
pf_status pf_op_attention(int dtype, int path, const void *q, int64_t ldq, const void *kbuf,
                          const void *vtbuf, int kv_rows, int rows_padded, int n_heads, int head_dim,
                          void *out, int64_t ldo, int nq, int splits, void *ws, size_t ws_bytes,
                          void *stream);

/*
 * pf_op_attention for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels and same results as
 * pf_op_attention with the same `splits`; the split partial results go into an array that is part of the library's
 * device image (PF_STATIC_SCRATCH_BYTES per GPU, held until the process ends) instead of a workspace argument.  The
 * call allocates and frees nothing and synchronises nothing; q, kbuf, vtbuf and out are the caller's, as before.
 *   - pf_op_attention_ws_bytes(nq, n_heads, head_dim, splits) > PF_STATIC_SCRATCH_BYTES: PF_ERR_WORKSPACE, nothing is
 *     launched, pf_last_error(NULL) says how many bytes were needed.  Other argument errors as pf_op_attention.
 *   - All calls on one GPU share that GPU's array: two calls whose work overlaps in time on one GPU (different
 *     streams, or several host threads) race on it.  Calls on one stream are ordered and safe.  Nothing in the array
 *     needs clearing between calls: a call reads only what it wrote itself.
 *   - The array's device address is looked up on the first call on each device (hipGetSymbolAddress), which is host
 *     work only; a caller that captures a graph may want to make one plain call first.
 */
#define PF_STATIC_SCRATCH_BYTES (32u << 20)
size_t pf_static_scratch_bytes(void);
pf_status pf_op_attention_static(int dtype, int path, const void *q, int64_t ldq, const void *kbuf,
                                 const void *vtbuf, int kv_rows, int rows_padded, int n_heads, int head_dim,
                                 void *out, int64_t ldo, int nq, int splits, void *stream);

/*
 * Measurement aid (no part of the method): enqueues a register-only loop of bf16 32x32x16 MFMAs - `workgroups` workgroups
 * of four waves, `iters` x 32 MFMAs per wave - and stores the launch's flop count in *flops (host).  out: device float
 * [workgroups * 256], overwritten.  Timed by the benchmark (events on `stream`) it gives the matrix rate the chip sustains
 * at the clock it holds under such a load: the measured ceiling beside the data-sheet peak, this library's own yardstick.
 */
pf_status pf_probe_mfma_loop(float *out, int workgroups, int iters, double *flops, void *stream);

/* pf_op_gemm with the tile configuration of the bf16 MFMA kernel chosen by the caller for this one launch: tile = 0 lets
 * the library's heuristic pick (then it is pf_op_gemm), 1 .. pf_gemm_tile_count() pins one of the configurations the
 * heuristic chooses from (the unit tests run every one of them on ragged shapes).  Nothing outlives the call.  tile > 0
 * needs dtype PF_BF16, path PF_PATH_AUTO and K a multiple of 64 (PF_ERR_SHAPE otherwise); tile out of range: PF_ERR_RANGE. */
int pf_gemm_tile_count(void);
pf_status pf_op_gemm_tile(int tile, int dtype, int path, const void *A, int64_t lda, const void *W, int64_t ldw,
                          const void *bias, void *C, int64_t ldc, int M, int N, int K, int epilogue, int gelu_from,
                          int gelu_tanh, const float *gate, const float *R, int64_t ldr, void *C2, int64_t ldc2,
                          void *stream);

/*
 * Host-only view of the bf16 MFMA GEMM's workgroup -> output tile map (for tests of the map; no device work).  A launch
 * on an M x N output with tile_m x tile_n tiles has *grid workgroups; workgroup ids are dealt round-robin to the 8 XCDs
 * and every XCD works on one rectangular block of the tile grid.  Returns 1 and the tile indices (row block *tm, column
 * block *tn) when workgroup `workgroup` computes a tile, 0 when it is one of the surplus ids of the padded grid (or
 * >= *grid; *tm = *tn = -1), PF_ERR_NULL / PF_ERR_RANGE (negative) on bad arguments.  All pointers are host pointers.
 */
int pf_gemm_tile_map(int M, int N, int tile_m, int tile_n, unsigned workgroup, unsigned *grid, int *tm, int *tn);

#ifdef __cplusplus
}
#endif
#endif /* PFSTAGE_H */
