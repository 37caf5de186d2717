/*
 * tcmv.h - C ABI of the MI355X (gfx950) vision preprocess + ViT-encode library.
 *
 * The paper ("TCM-Serve: Modality-aware Scheduling for Multimodal LLM
 * Inference") splits a multimodal request into inference stages (Sec. 2.1,
 * Fig. 1): vision preprocessing, vision encoding, then the LLM.  Its Workload
 * Profiler (Sec. 3.2) times preprocessing and encoding separately, and its
 * characterisation (Sec. 2.2; the split of the time to first token in Sec. 3.3,
 * Fig. 6) attributes the extra latency of image and video requests to these two
 * stages.  This library is
 * those two stages plus the projection of visual tokens to the LLM width:
 *
 *     tcmv_preprocess     raw uint8 frames  -> normalised patch rows
 *     tcmv_encode         patch rows        -> ViT encoder output (visual tokens)
 *     tcmv_merge_project  encoder output    -> merged tokens at the LLM width
 *
 * General rules
 *  - Every pointer whose name starts with d_ (and every pointer inside
 *    tcmv_weights and tcmv_item) is a DEVICE pointer owned by the caller; all
 *    other pointers are host pointers.  The library never allocates or frees
 *    device memory: frames, patch rows, activations, workspaces, weights and the
 *    device copy of a plan's index metadata (a few ints per token, see
 *    tcmv_plan_upload) all belong to the caller.
 *  - Kernels and copies are enqueued on the caller's hipStream_t (passed as
 *    void*, NULL = default stream); no call synchronises the stream or the device.
 *  - Every function returns TCMV_OK (0) or a negative TCMV_E_* code; the text of
 *    the last error of a context is available from tcmv_last_error.  No C++
 *    exception crosses this boundary.
 *  - Matrices are row-major and contiguous.  Linear weights are stored
 *    [out_features, in_features] (the contraction dimension is contiguous):
 *    y = x * W^T + b.
 *  - A context is not thread-safe; use one per thread.  Plans are immutable and
 *    may be used for any number of stage calls.
 *
 * Element types
 *  dtype TCMV_BF16: matrices (w_pe, w_qkv, w_o, w_1, w_2, w_m1, w_m2) are bf16;
 *    biases, LayerNorm gamma/beta, cls and position tables are fp32; patch rows
 *    are bf16; the encoder output (d_hidden) is fp32; the projector output is bf16.
 *  dtype TCMV_F32: everything is fp32.
 *
 * Token order (Sec. 2.2: an image is cut into a grid of patches of one fixed
 * size, which is why its token count hardly varies): frames are grouped by
 * `tpatch` (a still image is repeated),
 * giving a grid (gt, gh, gw) = (n_frames/tpatch or 1, dst_h/patch, dst_w/patch).
 * merge == 1: rows ordered (t, h, w).  merge == 2: rows ordered
 * (t, h/2, w/2, h%2, w%2) so every 2x2 merge group is four consecutive rows.
 * With attention windows (tcmv_model_desc.window) the same order is used inside
 * each window and windows follow each other; tcmv_plan_row_map returns the
 * (t, h, w) of every row.
 * Inside a patch row element k = ((c*tpatch + tt)*patch + py)*patch + px; rows
 * are zero-padded from K = 3*tpatch*patch^2 to k_pad (see tcmv_k_pad).
 */
#ifndef TCMV_H
#define TCMV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tcmv_ctx tcmv_ctx;   /* opaque; freed by tcmv_destroy      */
typedef struct tcmv_plan tcmv_plan; /* opaque; freed by tcmv_plan_destroy */

enum {
  TCMV_OK = 0,
  TCMV_E_INVALID_ARG = -1,         /* NULL pointer, negative size, unknown enum value      */
  TCMV_E_BAD_SHAPE = -2,           /* a shape the method does not define (see plan_create)  */
  TCMV_E_WORKSPACE_TOO_SMALL = -3, /* workspace_bytes below what tcmv_plan_query reports    */
  TCMV_E_NO_WEIGHTS = -4,          /* encode / merge_project before tcmv_set_weights        */
  TCMV_E_HIP = -5,                 /* a HIP runtime call failed; text in tcmv_last_error    */
  TCMV_E_UNSUPPORTED = -6          /* valid request outside what the kernels implement      */
};

typedef enum { TCMV_F32 = 0, TCMV_BF16 = 1 } tcmv_dtype;
typedef enum { TCMV_POS_NONE = 0, TCMV_POS_LEARNED_1D = 1, TCMV_POS_SEPARABLE_2D = 2, TCMV_POS_ROTARY_2D = 3 } tcmv_pos;
typedef enum { TCMV_NORM_LAYER = 0, TCMV_NORM_RMS = 1 } tcmv_norm;
typedef enum { TCMV_TEXT = 0, TCMV_IMAGE = 1, TCMV_VIDEO = 2 } tcmv_modality;

/* Encoder description.  d % heads == 0; head size d/heads must be a multiple
 * of 16 and at most 128 (TCMV_F32) or one of 32, 64, 80, 96 (TCMV_BF16); d, mlp
 * and heads*head size multiples of 64, out_dim of 8 for TCMV_BF16. */
typedef struct {
  int dtype;       /* tcmv_dtype */
  int layers, d, heads, mlp;
  int patch, tpatch, merge; /* merge: 1, or 2 for the 2x2 spatial merge      */
  int out_dim;     /* width after the projector; 0 = no projector             */
  int use_cls;     /* 1: a learned CLS row is row 0 of every segment          */
  int pos;         /* tcmv_pos */
  int max_pos;     /* rows of pos0 (and pos1): max rows per segment for
                      LEARNED_1D, max grid side for SEPARABLE_2D              */
  int final_ln;    /* 1: LayerNorm after the last block                       */
  float ln_eps;
  float mean[3], std[3]; /* per-channel normalisation x = (v/255 - mean)/std  */
  /* Encoder-family switches (the vision encoders of the paper's Table 1 differ in
   * these).  All zero = the plain pre-LN block above.  Non-zero values need
   * TCMV_BF16 and use_cls == 0. */
  int norm;        /* tcmv_norm: RMSNorm x/sqrt(mean(x^2)+eps)*gamma replaces every
                      LayerNorm (beta pointers are ignored)                      */
  int mlp_gated;   /* 1: h = silu(x Wg^T + bg) * (x Wu^T + bu), out = h W_2^T + b_2;
                      w_1 is then [2*mlp, d] with row 2j = Wg row j and row
                      2j+1 = Wu row j, b_1 [2*mlp] in the same order             */
  int window;      /* > 0 (a multiple of merge): token rows are ordered window by
                      window (window x window patches, clipped at the right and
                      bottom edges, raster order of windows inside a frame group,
                      the usual merge-group order inside a window) and layers
                      attend inside a window                                     */
  int full_every;  /* with window > 0: layers l with (l+1) % full_every == 0 attend
                      over the whole segment; 0 = every layer is windowed        */
  float rope_theta; /* TCMV_POS_ROTARY_2D: element pairs (2p, 2p+1) of every head of q
                      and k are rotated; the first dh/4 pairs by
                      h * theta^(-p/(dh/4)), the others by w * theta^(-(p-dh/4)/(dh/4)),
                      (h, w) = patch coordinate of the token; dh % 4 == 0        */
  int head_dim;    /* 0: every head is d/heads wide.  > 0 (TCMV_BF16 only): size of a head
                      as stored; q, k, v are then heads*head_dim wide each: w_qkv
                      [3*heads*head_dim, d], b_qkv [3*heads*head_dim], w_o
                      [d, heads*head_dim].  A model whose head size the kernels do not
                      have (72, say) is run by zero-padding every head to the next
                      size they have and giving the true scale in attn_scale        */
  float attn_scale; /* 0: scores are scaled by 1/sqrt(head size); > 0: by this value */
} tcmv_model_desc;

/* One request (Sec. 4.1, Workloads: every request carries one text, one image
 * or one video).  Text requests carry no frames (n_frames == 0), produce no
 * tokens and launch nothing (Sec. 3.3: these two stages cost a text request
 * next to nothing).  An image is n_frames == 1; a video needs n_frames to
 * be a multiple of tpatch.  d_frames: uint8 RGB interleaved
 * [n_frames, src_h, src_w, 3]; when (src_h, src_w) != (dst_h, dst_w) the frames
 * are resampled (integer bilinear, half-pixel centres, edge clamp, no
 * antialias).  dst_h and dst_w must be positive multiples of patch*merge. */
typedef struct {
  int modality; /* tcmv_modality */
  int n_frames, src_h, src_w, dst_h, dst_w;
  const uint8_t *d_frames;
} tcmv_item;

/* Parameters (device pointers, borrowed).  layer[l*12 + j], j in the order
 * ln1_g, ln1_b, w_qkv [3d,d], b_qkv, w_o [d,d], b_o, ln2_g, ln2_b, w_1 [mlp,d],
 * b_1, w_2 [d,mlp], b_2.  w_pe is [d, k_pad] with zero columns beyond K.
 * w_qkv rows: first d rows produce q, next d rows k, last d rows v; head j owns
 * rows [j*dh, (j+1)*dh) of each third.  cls [d]; pos0/pos1 [max_pos, d].
 * lnf_*: final LayerNorm.  lnm_*, w_m1 [m2*d, m2*d], w_m2 [out_dim, m2*d]:
 * projector (m2 = merge^2).  Unused entries may be NULL. */
typedef struct {
  const void *w_pe, *b_pe, *cls, *pos0, *pos1;
  const void *const *layer; /* host array of layers*12 device pointers */
  const void *lnf_g, *lnf_b, *lnm_g, *lnm_b, *w_m1, *b_m1, *w_m2, *b_m2;
} tcmv_weights;

/* Sizes of one plan.  n_patch_rows: rows of the patch matrix; n_tokens: rows of
 * the encoder output (= n_patch_rows + one CLS row per non-empty segment);
 * n_out_tokens = n_tokens / merge^2 when a projector exists, else 0. */
typedef struct {
  int64_t n_patch_rows, n_tokens, n_out_tokens;
  int64_t k, k_pad;
  size_t patches_bytes;          /* size of d_patches  [n_patch_rows, k_pad]          */
  size_t hidden_bytes;           /* size of d_hidden   [n_tokens, d] fp32             */
  size_t out_bytes;              /* size of d_out      [n_out_tokens, out_dim]        */
  size_t encode_workspace_bytes; /* minimum workspace for tcmv_encode                 */
  size_t merge_workspace_bytes;  /* minimum workspace for tcmv_merge_project          */
  int n_items, n_segments;       /* n_segments: items with at least one token         */
  size_t meta_bytes;             /* size of the plan's index metadata (tcmv_plan_upload); 0 for a plan without tokens */
} tcmv_plan_info;

/* major*100 + minor; 110 added the encoder-family fields at the end of tcmv_model_desc,
 * 120 head_dim and attn_scale behind them; 200: the caller owns the device copy of the plan
 * metadata (tcmv_plan_upload, d_meta argument of the stage calls, meta_bytes) and the index
 * data of tcmv_op_attention. */
int tcmv_version(void);
const char *tcmv_error_name(int code);

/* Padded patch-row length for a model: K rounded up to a multiple of 64 for
 * TCMV_BF16, to an even number for TCMV_F32.  Negative on an invalid description. */
int64_t tcmv_k_pad(const tcmv_model_desc *desc);

/* One context per vision encoder (Table 1 of the paper lists the encoder families of
 * its models; the description selects one).  Validates the description
 * (TCMV_E_INVALID_ARG / TCMV_E_UNSUPPORTED) and creates a context.  Host only: works
 * without a GPU. */
int tcmv_create(const tcmv_model_desc *desc, tcmv_ctx **out);
void tcmv_destroy(tcmv_ctx *ctx);
/* Text of the last error of a context; with ctx == NULL, the reason of the last
 * failed tcmv_create on the calling thread.  Valid until the next call. */
const char *tcmv_last_error(const tcmv_ctx *ctx);

/* Borrows the device pointers (the caller keeps them alive and unchanged while
 * the context uses them).  Checks only for NULLs of required entries. */
int tcmv_set_weights(tcmv_ctx *ctx, const tcmv_weights *w);

/* One plan per batch of requests (Sec. 4.1, Workloads: one text, image or video per
 * request; Sec. 2.2: an image becomes a grid of fixed-size patches, a video a
 * sequence of sampled frames).  Host only (no GPU needed; d_frames is not
 * dereferenced).  Computes grids, token order, cumulative segment lengths, per-row
 * index maps and the attention work list.  TCMV_E_BAD_SHAPE: dst not a positive multiple of patch*merge,
 * video length not a multiple of tpatch, src size < 1 for an item with frames,
 * a segment longer than max_pos rows (LEARNED_1D) or a grid side above max_pos
 * (SEPARABLE_2D), a grid side above 255, or so many tokens that tokens x widest
 * activation row (max of 3d, mlp, merge^2 d, k_pad) reaches 2^32, or tokens x 2 x
 * attention width, or the transposed values (heads x head size rows of padded token
 * columns; with attention windows every window is padded to 64 columns) reach 2^31
 * elements (the kernels keep element offsets in 32 bits, the attention kernel byte
 * offsets; about 838 000 tokens at d = 1280, mlp = 5120).  Zero items,
 * or only text items, give a valid empty plan.  Plans are immutable; the d_frames
 * pointers are recorded in the plan's metadata. */
int tcmv_plan_create(tcmv_ctx *ctx, const tcmv_item *items, int n_items, tcmv_plan **out);
void tcmv_plan_destroy(tcmv_plan *plan);
int tcmv_plan_query(const tcmv_plan *plan, tcmv_plan_info *info);
/* The kernels read a plan's index metadata (row maps, work lists, the 3 x 256
 * normalisation table, request descriptors) from a DEVICE buffer of meta_bytes bytes
 * that the caller owns, 256-byte aligned, and hands to the stage calls as d_meta.
 * tcmv_plan_meta returns the plan's host copy (lives as long as the plan) and its
 * size, for callers that copy it themselves; tcmv_plan_upload enqueues the copy
 * host -> d_meta on `stream` (hipMemcpyAsync from the plan's host copy: the plan must
 * stay alive until the stream has passed the copy; TCMV_E_WORKSPACE_TOO_SMALL when
 * meta_bytes is below tcmv_plan_info.meta_bytes).  One upload serves any number of
 * stage calls. */
const void *tcmv_plan_meta(const tcmv_plan *plan, size_t *bytes);
int tcmv_plan_upload(const tcmv_plan *plan, void *d_meta, size_t meta_bytes, void *stream);
/* cu_seqlens: host array of n_items+1 cumulative token counts (rows of the
 * encoder output per request; equal neighbours for text requests).  The pointer
 * lives as long as the plan. */
const int64_t *tcmv_plan_cu_seqlens(const tcmv_plan *plan);
/* Host copies of the per-row index maps, for inspection and tests.  which = 0:
 * (t,h,w) of each patch row packed as t<<16 | h<<8 | w; 1: encoder-output row
 * that each patch row lands in; 2: position index of each patch row (row inside
 * the segment for LEARNED_1D, h | w<<16 for SEPARABLE_2D, 0 otherwise).
 * Returns the number of entries, or a negative error. */
int64_t tcmv_plan_row_map(const tcmv_plan *plan, int which, const int32_t **out);

/* Stage 1 (Sec. 2.1: visual inputs are first preprocessed into pixels or frames;
 * Sec. 3.2 times this stage per request): resize + normalise + patchify in one
 * pass.  d_meta: the device copy of the plan's metadata.  d_patches
 * [n_patch_rows, k_pad], bf16 or fp32 by dtype, 16-byte aligned; every element is
 * written (padding columns with zeros).
 * Integer / table arithmetic only: results are bit-exact by definition. */
int tcmv_preprocess(tcmv_ctx *ctx, const tcmv_plan *plan, const void *d_meta, void *d_patches, void *stream);

/* Stage 2 (Sec. 2.1: the preprocessed input is then encoded into embeddings;
 * Sec. 3.2 times this stage per request): patch embedding (+CLS, +position),
 * `layers` pre-LN transformer blocks with bidirectional attention restricted to
 * each request's own tokens, optional final LayerNorm.  d_meta as above.
 * d_hidden [n_tokens, d] fp32 receives the result.  d_workspace: scratch of at
 * least encode_workspace_bytes, 256-byte aligned, contents undefined after. */
int tcmv_encode(tcmv_ctx *ctx, const tcmv_plan *plan, const void *d_meta, const void *d_patches, void *d_hidden,
                void *d_workspace, size_t workspace_bytes, void *stream);

/* Stage 3 (Sec. 2.1 and Fig. 1: the encoder's embeddings reach the LLM backend in
 * one common format, next to the text embeddings, i.e. at the LLM's hidden size):
 * LayerNorm, concatenate each merge^2 consecutive rows, two-layer MLP with GELU to
 * out_dim.  d_out [n_out_tokens, out_dim] in the model dtype.
 * TCMV_E_UNSUPPORTED when out_dim == 0. */
int tcmv_merge_project(tcmv_ctx *ctx, const tcmv_plan *plan, const void *d_hidden, void *d_out,
                       void *d_workspace, size_t workspace_bytes, void *stream);

/* ---- per-kernel timing ------------------------------------------------------
 * tcmv_profile_enable(ctx, classes): classes is a bit mask over the kernel classes
 * below (bit TCMV_K_x), a negative value selects all of them, 0 switches timing off.
 * The three stage calls then bracket every launch of a selected class with a pair
 * of HIP events on the caller's stream (host-side objects, no device memory).
 * tcmv_profile_read waits for the recorded events, adds the elapsed
 * milliseconds and launch counts per kernel class to ms[] / launches[] (arrays
 * of TCMV_K_COUNT entries, overwritten) and forgets the events. */
enum {
  TCMV_K_PREPROCESS = 0, TCMV_K_EMBED_GEMM, TCMV_K_LAYERNORM, TCMV_K_QKV_GEMM, TCMV_K_ATTENTION,
  TCMV_K_OUT_GEMM, TCMV_K_FC1_GEMM, TCMV_K_FC2_GEMM, TCMV_K_MERGE_GEMM, TCMV_K_OTHER, TCMV_K_COUNT
};
int tcmv_profile_enable(tcmv_ctx *ctx, int classes);
int tcmv_profile_read(tcmv_ctx *ctx, double *ms, int64_t *launches);

/* ---- single operators (the kernels the stages are built from), exposed so
 * that each can be checked and timed alone.  All pointers are device pointers.
 * dtype selects the bf16 MFMA path or the fp32 path. ---------------------- */

/* y = LN(x) * gamma + beta over the last dimension (biased variance).
 * x [rows, d] fp32; y [rows, d] bf16 (TCMV_BF16) or fp32 (TCMV_F32).
 * d_beta == NULL selects RMSNorm: y = x / sqrt(mean(x^2) + eps) * gamma. */
int tcmv_op_layernorm(int dtype, const float *d_x, const float *d_gamma, const float *d_beta,
                      void *d_y, int64_t rows, int d, float eps, void *stream);

/* Bandwidth reference, no part of the path: reads in_bytes from d_in once and
 * writes out_bytes to d_out once (the words written are the XOR of words read, so the
 * reads cannot be dropped).  Timed beside a bandwidth-bound kernel with the same byte
 * counts it shows what that kernel could reach at best at its size.  Sizes and
 * pointers must be multiples of 16 (else TCMV_E_INVALID_ARG); either size may be 0. */
int tcmv_op_stream(const void *d_in, size_t in_bytes, void *d_out, size_t out_bytes, void *stream);

/* C = epilogue(A * W^T + bias).  A [m, k], W [n, k], both bf16 (k % 64 == 0,
 * n % 8 == 0) or fp32.  epilogue: 0: store (bf16 / fp32 by dtype);
 * 1: GELU (erf form; the bf16 path evaluates it to within 3.5e-5 absolute, and
 * the bf16 result is within one unit in the last place of the rounded exact value
 * or within 2^-22 of it) then store; 2: d_c is fp32 [m, n] and is incremented
 * (residual add); 5 (TCMV_BF16 only): gated product, output column j =
 * silu(column 2j) * column 2j+1, d_c is bf16 [m, n/2].  bias fp32 [n] or NULL. */
int tcmv_op_gemm(int dtype, int epilogue, const void *d_a, const void *d_w, const float *d_bias,
                 void *d_c, int64_t m, int n, int k, void *stream);

/* Block-diagonal bidirectional attention.  d_qkv [T, 3*d] (q | k | v thirds,
 * head j = columns [j*dh, (j+1)*dh) of each third), bf16 or fp32; cu_seqlens:
 * HOST array of n_seg+1 row offsets; d_out [T, d] same type as the input.
 * The kernels read index data (row maps, work list) that depends on cu_seqlens only:
 * tcmv_op_attention_index writes it into a HOST buffer of at least
 * tcmv_op_attention_index_bytes bytes; the caller copies it to the device (d_index,
 * 256-byte aligned) and may reuse it for any number of calls with the same shape.
 * d_workspace / workspace_bytes: scratch, 256-byte aligned, size from
 * tcmv_op_attention_workspace (0 from the size queries = invalid arguments). */
size_t tcmv_op_attention_workspace(int dtype, const int64_t *cu_seqlens, int n_seg, int d, int heads);
size_t tcmv_op_attention_index_bytes(int dtype, const int64_t *cu_seqlens, int n_seg, int d, int heads);
int tcmv_op_attention_index(int dtype, const int64_t *cu_seqlens, int n_seg, int d, int heads, void *h_index,
                            size_t index_bytes);
int tcmv_op_attention(int dtype, const void *d_qkv, const int64_t *cu_seqlens, int n_seg, int d, int heads,
                      const void *d_index, void *d_out, void *d_workspace, size_t workspace_bytes, void *stream);

/* tcmv_op_attention for callers that cannot allocate device memory (code under HIP
 * graph capture, serving loops and harnesses that forbid hipMalloc): same arguments
 * and same result, but no workspace argument.  The scratch lives in a fixed array of
 * TCMV_NOALLOC_SCRATCH_BYTES in device memory that every GPU the library runs on
 * holds until the process ends; the call allocates and frees nothing.  Shapes whose
 * scratch (tcmv_op_attention_workspace) exceeds that size return
 * TCMV_E_WORKSPACE_TOO_SMALL.  All calls on one GPU share the array: calls that
 * overlap on one GPU (two streams, two threads) race; calls on one stream do not. */
#define TCMV_NOALLOC_SCRATCH_BYTES (16u << 20)
int tcmv_op_attention_noalloc(int dtype, const void *d_qkv, const int64_t *cu_seqlens, int n_seg, int d, int heads,
                              const void *d_index, void *d_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TCMV_H */
