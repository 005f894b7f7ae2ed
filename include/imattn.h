/*
 * imattn.h -- C ABI of the Interlaced-Mask (IM) attention library for AMD
 * Instinct MI355X (gfx950).
 *
 * The library computes multi-head attention over the concatenation
 * V_m = [V_t; V_v; V_a] of the modality sequences with ONE set of projection
 * weights for all modalities, under a block pattern of live (all-zero, "O") and
 * masked (all-minus-infinity, "J") modality blocks -- the Interlaced Mask of the
 * GsiT paper (Sec. 5 "All-Modal-In-One Fusion", Eq. "ifm" and the IEM equation;
 * Eq. "allmodalinone fusion").  Nothing is loaded or multiplied for a masked
 * block: this is the role the paper gives its "Decomposition" step (Sec. 6
 * "Inner Decomposition for Efficiency").
 *
 * General conventions
 *   - Pointers named in "device" lists are device (HBM) pointers owned by the
 *     caller; the im_shape_t, size outputs and im_work_item_t arrays are host
 *     memory.  The library never allocates or frees device memory and keeps no
 *     device state between calls.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*;
 *     NULL = the default stream).  No call synchronises the device.
 *   - Arrays are dense row-major.  Activations are [B, T_m, d] with
 *     T_m = sum(seg_len) and the segments stored one after the other in the
 *     order given by seg_len (the paper's order is text, vision, audio).
 *   - Weights are [d_in, d_out] and applied as y = x W (Sec. 3 writes
 *     W in R^{d x d^f}); biases are [d_out] or NULL.
 *   - dtype IM_DTYPE_F32: every float array is fp32.
 *     dtype IM_DTYPE_BF16: activations, weights and biases are bfloat16; all
 *     accumulation is fp32; weight/bias GRADIENTS are written in fp32.
 *   - Return value: IM_OK, or a negative error code.  Shape, pointer, alignment
 *     and workspace-size validation precedes any launch (a call rejected with
 *     IM_ERR_INVALID / UNSUPPORTED / WORKSPACE has enqueued nothing); IM_ERR_HIP
 *     reports a launch error collected after the call's kernels were enqueued.
 *     im_last_error() returns a thread-local description of the last failure.
 *   - Limits: batch <= 65535.  With dtype IM_DTYPE_BF16 and a head dimension of
 *     8, 16 or 64 (d_model a multiple of 64: the matrix-core kernels) x, the
 *     weights, dy, y, dx, saved and workspace must be 16-byte aligned.
 *   - Numerical conventions: a key is padding if key_pad[b, c] != 0 or if its
 *     position inside its segment is >= valid_len[b, segment]; padded keys get
 *     weight exactly 0.  Padded QUERY rows are computed like any other row.  A
 *     query row with no live, valid key has attention output 0 (y = b_o) and
 *     contributes 0 to every gradient.  A row with several live blocks is
 *     normalised by ONE softmax over all its live keys (the additive -inf
 *     definition; Sec. "Information Disorder" under "Further Analysis").
 */
#ifndef IMATTN_H
#define IMATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IM_MAX_SEG 8

#define IM_DTYPE_F32 0
#define IM_DTYPE_BF16 1

#define IM_OK 0
#define IM_ERR_INVALID (-1)     /* null required pointer, bad shape, live_mask bits out of range */
#define IM_ERR_UNSUPPORTED (-2) /* dtype / head dimension / model dimension the library has no kernel for */
#define IM_ERR_WORKSPACE (-3)   /* workspace_bytes smaller than im_attention_sizes / gsit_layer_sizes reports */
#define IM_ERR_HIP (-4)         /* a HIP runtime call failed; text in im_last_error() */

/* Named 3x3 patterns for segment order (t, v, a) = (0, 1, 2).
 * Bit (i * n_seg + j) set <=> block (query segment i, key segment j) is O (live).
 * IFM forward / backward: Sec. 5 Eq. "ifm"; IEM: the M_intra equation after it. */
#define IM_IFM_FORWARD 0x062ull  /* live (t,v), (v,a), (a,t) */
#define IM_IFM_BACKWARD 0x08Cull /* live (t,a), (v,t), (a,v) */
#define IM_IEM 0x111ull          /* live (t,t), (v,v), (a,a) */
#define IM_DENSE3 0x1FFull       /* ordinary self-attention over V_m */
/* The other structures of the ablation (Sec. "Ablation Study"; App. "Graph Structures"), each a pair of
 * masks, and Self-Only, whose rows have two live blocks each and share one softmax across them
 * (Sec. "Information Disorder").  Structure-1's first set follows the text's edge list. */
#define IM_STRUCTURE1_A 0x0A4ull /* live (t,a), (v,a), (a,v) */
#define IM_STRUCTURE1_B 0x04Aull /* live (t,v), (v,t), (a,t) */
#define IM_STRUCTURE2_A 0x08Aull /* live (t,v), (v,t), (a,v) */
#define IM_STRUCTURE2_B 0x064ull /* live (t,a), (v,a), (a,t) */
#define IM_STRUCTURE3_A 0x0A2ull /* live (t,v), (v,a), (a,v) */
#define IM_STRUCTURE3_B 0x04Cull /* live (t,a), (v,t), (a,t) */
#define IM_SELF_ONLY 0x0EEull    /* every block but the diagonal */

/* The problem statement: per-modality lengths, model width, heads, block pattern. */
typedef struct im_shape {
  int32_t batch;               /* B >= 1 */
  int32_t n_seg;               /* number of modality segments, 1..IM_MAX_SEG (3 in the paper) */
  int32_t seg_len[IM_MAX_SEG]; /* padded length T_s >= 1 of each segment, concatenation order */
  int32_t d_model;             /* d */
  int32_t n_heads;             /* H, d % H == 0; head dimension dh = d / H */
  uint64_t live_mask;          /* the IM: bit (i*n_seg + j) <=> block (query seg i, key seg j) live */
  float scale;                 /* multiplies Q K^T before the softmax (App. B "apply scaling and softmax"); finite, >= 0; usually 1/sqrt(dh) */
  int32_t dtype;               /* IM_DTYPE_F32 or IM_DTYPE_BF16 */
  /* Packed rows (no padding rows in memory; the datasets' sequences are far shorter than their
   * maxima, Table "Dataset statistics and data forms", average vs. maximum length).  NULL: every
   * [rows, .] tensor is [B, T_m, .] as described at the entry points.  Non-NULL: device int32
   * [B * n_seg + 1], cu_rows[0] = 0, non-decreasing; segment s of batch element b occupies rows
   * cu_rows[b*n_seg+s] .. cu_rows[b*n_seg+s+1]-1 of [total_rows, .] tensors, its length may be
   * anything in 0..seg_len[s] (seg_len then only bounds the lengths).  valid_len must be NULL
   * (the lengths are in cu_rows); key_pad, if given, is [total_rows].  Supported by
   * im_attention_* and gsit_layer_*; the whole-model call needs padded rows. */
  const int32_t* cu_rows;
  int64_t total_rows;          /* = cu_rows[B * n_seg] (host copy), >= 1; ignored when cu_rows is NULL */
} im_shape_t;

/* One unit of the live-block schedule (host side; see im_schedule_build). */
typedef struct im_work_item {
  int32_t q_seg;     /* query segment i */
  int32_t q_start;   /* first query row of the tile inside segment i */
  int32_t q_rows;    /* rows in the tile (<= tile_rows) */
  int32_t n_key_seg; /* number of live key segments for this query segment */
  int32_t key_seg[IM_MAX_SEG]; /* their indices j, ascending */
  int64_t pairs;     /* q_rows * sum_j T_j : (query, key) pairs this item covers (padded lengths) */
} im_work_item_t;

/* Sec. 6 "Decomposition": enumerate, for ONE (batch element, head), the query
 * tiles and the live key segments each must visit; nothing is emitted for a
 * masked block.  Items are ordered by query segment, the segments by decreasing
 * number of live keys per query row (heaviest rows first; inside a segment by
 * row, so a ragged last tile has fewer pairs than its predecessors).  Pure
 * host function, no GPU needed.  items may be NULL to only count.  *n_pairs
 * receives sum(pairs) = sum over live (i,j) of T_i T_j (App. B, attention cost
 * "w/ Decomposition").  Returns IM_ERR_INVALID if max_items is too small. */
int im_schedule_build(const im_shape_t* shape, int32_t tile_rows, im_work_item_t* items, int32_t max_items,
                      int32_t* n_items, int64_t* n_pairs);

/* Bytes of the `saved` buffer (forward -> backward) and of the largest
 * workspace any of im_attention_fwd / im_attention_bwd needs for this shape. */
int im_attention_sizes(const im_shape_t* shape, size_t* saved_bytes, size_t* workspace_bytes);

/* y = IMAttention(x): shared Q/K/V projection (Sec. 3; App. A Eq. "adjmat_all"),
 * scores and row softmax on the live blocks only (App. A Eq. "sbg_sbg0",
 * Sec. 5), aggregation P V with heads concatenated (App. A Eq. "sbg_sbg1"), output
 * projection.
 * device in : x [B,T_m,d]; wq, wk, wv, wo [d,d]; bq, bk, bv, bo [d] or NULL;
 *             valid_len int32 [B,n_seg] or NULL; key_pad uint8 [B,T_m] or NULL
 *             (both given: a key is padding if either says so).
 * device out: y [B,T_m,d]; saved (saved_bytes; opaque: projected Q, K, V, the
 *             attention output before W_o and the per-row log-sum-exp) or NULL
 *             for inference; workspace (scratch, contents undefined afterwards). */
int im_attention_fwd(const im_shape_t* shape, const void* x, const void* wq, const void* wk, const void* wv,
                     const void* wo, const void* bq, const void* bk, const void* bv, const void* bo,
                     const int32_t* valid_len, const uint8_t* key_pad, void* y, void* saved, void* workspace,
                     size_t workspace_bytes, void* hip_stream);

/* Gradients of im_attention_fwd given dy [B,T_m,d] and the `saved` buffer of the
 * forward call with the same arguments (the paper states no backward; this is
 * the chain rule of the definition above, restricted to live blocks).
 * device out (overwritten, not accumulated): dx [B,T_m,d] (activation dtype);
 *   dwq, dwk, dwv, dwo fp32 [d,d]; dbq, dbk, dbv, dbo fp32 [d], each may be NULL
 *   if not wanted.  Results are bitwise reproducible run to run. */
int im_attention_bwd(const im_shape_t* shape, const void* x, const void* wq, const void* wk, const void* wv,
                     const void* wo, const int32_t* valid_len, const uint8_t* key_pad, const void* saved,
                     const void* dy, void* dx, void* dwq, void* dwk, void* dwv, void* dwo, void* dbq, void* dbk,
                     void* dbv, void* dbo, void* workspace, size_t workspace_bytes, void* hip_stream);

/* im_attention_fwd (inference: nothing saved) for callers that cannot allocate or pass device scratch
 * memory -- code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * projected Q, K, V, the attention output before W_o and the row statistics live in a buffer that is
 * part of the library image: IM_NOALLOC_MAX_BYTES per GPU, held from library load until the process
 * ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating library routine) and
 * returns IM_ERR_WORKSPACE -- before anything is enqueued -- for a shape whose
 * im_attention_sizes workspace exceeds IM_NOALLOC_MAX_BYTES.  Arguments, results and errors are
 * otherwise those of im_attention_fwd with saved = NULL; the output is bitwise the same.
 * All calls on one GPU share that GPU's buffer: calls that may overlap in time on one GPU (different
 * streams or host threads) race and must be serialised by the caller.  Nothing in the buffer needs
 * to start at zero (every part is written before it is read), so the previous call's contents are
 * harmless.  im_noalloc_init looks up the buffer's address on the CURRENT device (hipGetSymbolAddress,
 * once per device); it is optional -- the first call on a device does the same -- but a caller that
 * captures a graph should make it before the capture begins.  Host-side state is mutex-protected. */
#define IM_NOALLOC_MAX_BYTES (64u << 20)
int im_noalloc_init(void);
int im_attention_fwd_noalloc(const im_shape_t* shape, const void* x, const void* wq, const void* wk, const void* wv,
                             const void* wo, const void* bq, const void* bk, const void* bv, const void* bo,
                             const int32_t* valid_len, const uint8_t* key_pad, void* y, void* hip_stream);

/* One GsiT encoder layer, a = MLP o MHSA_2 (Sec. 5 Eq. "allmodalinone fusion";
 * MLP weights W_1 [d, d_ff], W_2 [d_ff, d] as in App. B), in the pre-LayerNorm
 * residual form:  h = x + IMAttention(LN(x; ln1)),  y = h + GELU(LN(h; ln2) W_1 + b_1) W_2 + b_2
 * (exact erf GELU; LayerNorm over the feature axis, biased variance, eps = ln_eps).
 * device in : as im_attention_fwd plus ln1_g, ln1_b, ln2_g, ln2_b [d]; w1 [d,d_ff];
 *             b1 [d_ff] or NULL; w2 [d_ff,d]; b2 [d] or NULL.
 * device out: y [B,T_m,d] (may alias x); workspace of gsit_layer_sizes bytes. */
int gsit_layer_sizes(const im_shape_t* shape, int32_t d_ff, size_t* workspace_bytes);
int gsit_layer_fwd(const im_shape_t* shape, int32_t d_ff, const void* x, const void* ln1_g, const void* ln1_b,
                   const void* wq, const void* wk, const void* wv, const void* wo, const void* bq, const void* bk,
                   const void* bv, const void* bo, const void* ln2_g, const void* ln2_b, const void* w1,
                   const void* b1, const void* w2, const void* b2, float ln_eps, const int32_t* valid_len,
                   const uint8_t* key_pad, void* y, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The GsiT model around the encoder layers (Sec. 5, Eq. "allmodalinone fusion"):
 *   F = Enc_fwd(x) under mask_fwd and B = Enc_bwd(x) under mask_bwd (two stacks of n_layers_inter
 *   layers of width d = shape->d_model with independent weights, shape->n_heads heads, shape->scale),
 *   Vbar = F || B (feature concatenation, width 2d),
 *   A = Enc_intra(Vbar) under mask_intra (n_layers_intra layers of width 2d, n_heads_intra heads,
 *   scale_intra),
 *   out = (|| over segments s of A[b, last step of s, :]) wf + bf          [B, n_out].
 * The paper's masks are IM_IFM_FORWARD, IM_IFM_BACKWARD, IM_IEM; shape->live_mask is ignored.
 * "Last step" of a segment is position max(min(valid_len[b,s], T_s), 1) - 1 when valid_len is
 * given, else T_s - 1.  Layers as in gsit_layer_fwd.
 * host  : shape, model and the three arrays of gsit_layer_params_t it points to.
 * device: every pointer inside gsit_layer_params_t; wf [n_seg*2d, n_out] row-major; bf [n_out] or
 *         NULL; x [B,T_m,d]; valid_len, key_pad as in im_attention_fwd; out [B, n_out] (dtype of
 *         shape->dtype); workspace of gsit_model_sizes bytes.  Nothing is allocated; all work is
 *         enqueued on hip_stream.  Errors as for gsit_layer_fwd. */
typedef struct {
  const void *ln1_g, *ln1_b, *wq, *wk, *wv, *wo, *bq, *bk, *bv, *bo, *ln2_g, *ln2_b, *w1, *b1, *w2, *b2;
} gsit_layer_params_t;

typedef struct {
  int32_t n_layers_inter;  /* layers of each of the two inter-modal (IFM) encoders, >= 1 */
  int32_t n_layers_intra;  /* layers of the intra-modal (IEM) encoder, >= 1 */
  int32_t d_ff_inter;      /* hidden width of the MLPs at width d */
  int32_t d_ff_intra;      /* hidden width of the MLPs at width 2d */
  int32_t n_heads_intra;   /* heads at width 2d; must divide 2d */
  int32_t n_out;           /* outputs of the final linear f */
  float scale_intra;       /* score scale at width 2d, normally 1/sqrt(2d / n_heads_intra) */
  float ln_eps;
  uint64_t mask_fwd, mask_bwd, mask_intra;
  const gsit_layer_params_t* fwd_layers;    /* host array [n_layers_inter] */
  const gsit_layer_params_t* bwd_layers;    /* host array [n_layers_inter] */
  const gsit_layer_params_t* intra_layers;  /* host array [n_layers_intra], width 2d */
  const void* wf;
  const void* bf;
} gsit_model_t;

/* Encoder layer, training.  gsit_layer_fwd_train computes the same y as gsit_layer_fwd and fills
 * `saved` (the attention's saved tensors, h = x + attention, the MLP's pre-activation and
 * activation); gsit_layer_bwd is the gradient of that forward (the calculus of the layer of Sec. 5;
 * the paper analyses no backward pass): given dy [B,T_m,d] it overwrites dx [B,T_m,d] (dtype of
 * shape->dtype) and, for every non-NULL field of `grads`, the fp32 gradient of the parameter of
 * the same name (shapes of the parameters; not accumulated).  A bias gradient may only be
 * requested when that bias was given.  Deterministic (fixed-order reductions).
 * host  : shape, params, grads (structs of device pointers).
 * device: x, dy, saved (gsit_layer_train_sizes' saved_bytes, written by the forward and read by the
 *         backward), y, dx, workspace (workspace_bytes of gsit_layer_train_sizes covers both calls).
 * Errors as for gsit_layer_fwd. */
typedef struct {
  void *ln1_g, *ln1_b, *wq, *wk, *wv, *wo, *bq, *bk, *bv, *bo, *ln2_g, *ln2_b, *w1, *b1, *w2, *b2;
} gsit_layer_grads_t;

int gsit_layer_train_sizes(const im_shape_t* shape, int32_t d_ff, size_t* saved_bytes, size_t* workspace_bytes);
int gsit_layer_fwd_train(const im_shape_t* shape, int32_t d_ff, const void* x, const gsit_layer_params_t* params,
                         float ln_eps, const int32_t* valid_len, const uint8_t* key_pad, void* y, void* saved,
                         void* workspace, size_t workspace_bytes, void* hip_stream);
int gsit_layer_bwd(const im_shape_t* shape, int32_t d_ff, const void* x, const gsit_layer_params_t* params, float ln_eps,
                   const int32_t* valid_len, const uint8_t* key_pad, const void* saved, const void* dy, void* dx,
                   const gsit_layer_grads_t* grads, void* workspace, size_t workspace_bytes, void* hip_stream);

int gsit_model_sizes(const im_shape_t* shape, const gsit_model_t* model, size_t* workspace_bytes);
int gsit_model_fwd(const im_shape_t* shape, const gsit_model_t* model, const void* x, const int32_t* valid_len,
                   const uint8_t* key_pad, void* out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Kernel timing for benchmarks (off by default).  While enabled, the library
 * brackets each kernel family it launches with hipEvents recorded on the call's
 * stream.  im_profile_get synchronises on the recorded events, so call it after
 * the stream has drained; it returns the number of families, and for family
 * `idx` its name (static storage), accumulated milliseconds and launch count
 * since the last non-zero im_profile_enable.  `on`: 0 = off; 1 = every family;
 * any other value = a selection, bit (idx + 1) set <=> family idx is timed (an
 * event pair costs a few microseconds of stream time, so a benchmark that times
 * whole steps brackets only the family it reports).  Not thread-safe; at most 8192
 * launches are recorded between resets (later ones are not timed).  Host memory only. */
int im_profile_enable(int on);
int im_profile_get(int idx, const char** name, double* total_ms, int64_t* launches);

/* Benchmark aids: what this GPU sustains, to set measured rates against.  im_calibrate_mfma enqueues a
 * register-resident loop of `iters` x 16 v_mfma_f32_32x32x16_bf16 per wave on every SIMD (no memory
 * traffic; `sink` is a device pointer to >= 4 bytes that is practically never written) and returns
 * the flops it launched in *flops; im_calibrate_copy enqueues a streaming device copy of `bytes`
 * (16-byte aligned, a multiple of 16).  The caller times them with events on hip_stream. */
int im_calibrate_mfma(int32_t iters, void* sink, double* flops, void* hip_stream);
int im_calibrate_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/* Description of the last error on the calling thread ("" if none).  Static storage. */
const char* im_last_error(void);

/* Library version string, e.g. "imattn 0.1 gfx950". */
const char* im_version(void);

#ifdef __cplusplus
}
#endif
#endif /* IMATTN_H */
