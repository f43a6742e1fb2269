/*
 * vscan.h - C ABI of the MI355X (gfx950) implementation of VScan's two-stage
 * visual token reduction (arXiv 2505.22654).
 *
 * Stage 1 (Sec. 4.1): score the visual encoder's tokens by attention, keep a
 * local top-k per window plus a global top-k, assign every dropped token to its
 * most cosine-similar kept token and average each group (Eq. 1-4).
 * Stage 2 (Sec. 4.2): at a middle LLM layer score the visual tokens by the
 * attention of the last instruction token(s), keep the top-k and compact hidden
 * states and K/V so pruned tokens never reach the cache (Eq. 5, "Remarks on KV
 * Cache").
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  Tensors are
 *     contiguous, row-major, 16-byte aligned.  Descriptors are HOST structs.
 *   - The entry points keep no state between calls and allocate no device
 *     memory: scratch comes in through `workspace` (size from the matching
 *     *_workspace_size call).  The only process-wide state is the optional
 *     measurement aid at the end of this header.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns without synchronising.  Calls that
 *     share a workspace must be ordered on one stream.
 *   - Return value: VSCAN_OK or a negative error.  No exceptions, no abort.
 *     Every argument, shape, budget, alignment and workspace check is made on
 *     the host before the first launch: with any error other than
 *     VSCAN_ERR_HIP nothing has been enqueued and no output is touched.
 *     VSCAN_ERR_HIP reports a launch the runtime refused; kernels enqueued
 *     before it still run, and the outputs are then unspecified.
 *   - Ties are broken towards the lowest index; index outputs are ascending.
 *   - Floating-point inputs must be finite (NaN ordering is unspecified).
 */
#ifndef VSCAN_H
#define VSCAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VSCAN_VERSION 0x00010000u

enum { VSCAN_F32 = 0, VSCAN_BF16 = 1 };

/* Which attention row scores the encoder tokens (Sec. 4.1 "Global Scan"):
 * the [CLS] query row (Eq. 1), or, for encoders without [CLS], the mean
 * attention each token receives from all visual query rows. */
enum { VSCAN_SCORE_CLS_ROW = 0, VSCAN_SCORE_MEAN_RECEIVED = 1 };

/* Softmax key domain.  VISUAL_ONLY follows Eq. 1 / Eq. 5 as written (K_V holds
 * visual keys only).  KEYS_ALL normalises over the whole attention row (encoder:
 * including the [CLS] key; LLM: the causal row of each query) and then takes the
 * visual slice. */
enum { VSCAN_KEYS_VISUAL_ONLY = 0, VSCAN_KEYS_ALL = 1 };

enum {
    VSCAN_OK = 0,
    VSCAN_ERR_NULL = -1,      /* a required pointer is NULL */
    VSCAN_ERR_SHAPE = -2,     /* a dimension is non-positive or inconsistent */
    VSCAN_ERR_BUDGET = -3,    /* a keep budget does not fit */
    VSCAN_ERR_DTYPE = -4,     /* unknown dtype / mode enum */
    VSCAN_ERR_ALIGN = -5,     /* a tensor pointer is not 16-byte aligned */
    VSCAN_ERR_WORKSPACE = -6, /* workspace missing or too small */
    VSCAN_ERR_HIP = -7,       /* a HIP runtime call failed */
    VSCAN_ERR_VERSION = -8,   /* struct_size does not match this library */
    VSCAN_ERR_UNSUPPORTED = -9 /* valid request outside what the kernels cover */
};

/* ---------------------------------------------------------------------------
 * Stage 1: vscan_encoder_reduce  (Sec. 4.1, Eq. 1-4)
 * ------------------------------------------------------------------------- */
typedef struct {
    uint32_t struct_size;   /* sizeof(vscan_encoder_desc) */
    int32_t dtype;          /* of q, k, x, merged: VSCAN_F32 or VSCAN_BF16 */
    int32_t batch;          /* B images */
    int32_t n_segments;     /* C crops per image (1 for single-image encoders) */
    int32_t grid_h, grid_w; /* token grid per segment; N = grid_h * grid_w */
    int32_t has_cls;        /* 1: q/k have S = N + 1 rows and [CLS] is row 0 */
    int32_t score_mode;     /* VSCAN_SCORE_* */
    int32_t softmax_domain; /* VSCAN_KEYS_* */
    int32_t heads;          /* H, 1 .. 1024 */
    int32_t head_dim;       /* dh, multiple of 8, <= 256 */
    int32_t feat_dim;       /* D of x, multiple of 8 */
    int32_t win_rows, win_cols; /* windows per segment along each axis (Eq. 3):
                                   token (r, c) is in window (r*win_rows/grid_h,
                                   c*win_cols/grid_w), integer division */
    int32_t keep_global;    /* |x^g| per segment (Eq. 2) */
    int32_t keep_local;     /* |x^l| per segment (Eq. 3): floor(keep_local / W) per
                               window, the remainder is added to keep_global */
    float scale;            /* logit scale; <= 0 selects 1/sqrt(head_dim) */
} vscan_encoder_desc;

/* Bytes of workspace vscan_encoder_reduce needs for this descriptor.
 * `with_local_pair` != 0 sizes for a call that passes q_local / k_local. */
int vscan_encoder_workspace_size(const vscan_encoder_desc *desc, int with_local_pair,
                                 size_t *bytes);

/*
 * q, k        in  [B, C, H, S, dh]  output-layer queries / keys (only the [CLS]
 *                 query row is read in CLS mode)
 * q_local,    in  same layout, the shallow-layer pair whose scores drive the
 * k_local         local scan (Sec. 4.1 "Local Scan", layer l); both NULL = use q, k
 * x           in  [B, C*N, D]  patch token features (no [CLS] row); cosine
 *                 similarity and Eq. 4 act on these
 * kept_idx    out [B, K] int32, K = C*(keep_global+keep_local): image-level token
 *                 index c*N + r*grid_w + col, ascending
 * merged      out [B, K, D] in `dtype`: Eq. 4 for every kept token
 * assign_out  out optional [B, C*N] int32: slot (0..K-1) each token merged into
 *                 (a kept token reports its own slot)
 * scores_out  out optional [B, C*N] fp32: the global-scan score S^avg (Eq. 2)
 */
int vscan_encoder_reduce(const vscan_encoder_desc *desc, const void *q, const void *k,
                         const void *q_local, const void *k_local, const void *x,
                         int32_t *kept_idx, void *merged, int32_t *assign_out,
                         float *scores_out, void *workspace, size_t workspace_bytes,
                         void *stream);

/* ---------------------------------------------------------------------------
 * Stage 2: vscan_llm_prune  (Sec. 4.2, Eq. 5; "Remarks on KV Cache")
 * ------------------------------------------------------------------------- */
typedef struct {
    uint32_t struct_size;   /* sizeof(vscan_llm_desc) */
    int32_t dtype;          /* of q, k, v, hidden */
    int32_t batch;          /* B sequences, all of the same layout */
    int32_t seq_len;        /* S */
    int32_t vis_start;      /* first visual position */
    int32_t vis_len;        /* V visual tokens, contiguous */
    int32_t n_query;        /* Tq scoring queries = the last Tq positions; the paper
                               uses the last instruction token only (Tq = 1) */
    int32_t q_heads;        /* Hq, 1 .. 1024 */
    int32_t kv_heads;       /* Hkv, divides Hq; query head h reads kv head h/(Hq/Hkv) */
    int32_t head_dim;       /* dh, multiple of 8, <= 256 */
    int32_t hidden;         /* Dh, multiple of 8 */
    int32_t keep;           /* visual tokens kept per sequence (R2 % of V) */
    int32_t softmax_domain; /* VSCAN_KEYS_* */
    int32_t in_place;       /* 1: compact k, v, hidden inside their own buffers */
    float scale;            /* <= 0 selects 1/sqrt(head_dim) */
} vscan_llm_desc;

int vscan_llm_workspace_size(const vscan_llm_desc *desc, size_t *bytes);

/*
 * q           in  [B, Hq, Tq, dh]  layer-k queries of the last Tq positions
 * k, v        in  [B, Hkv, S, dh]  layer-k keys / values (position-encoded as the
 *                 attention layer sees them); mutated iff in_place
 * hidden      in  [B, S, Dh]; mutated iff in_place
 * kept_idx    out [B, keep] int32, ascending, relative to vis_start (may be NULL
 *                 when keep == 0)
 * k_out,v_out out [B, Hkv, S_out, dh], hidden_out [B, S_out, Dh],
 *                 S_out = S - V + keep: rows [0, vis_start) ++ kept visual rows in
 *                 original order ++ rows [vis_start+V, S).  Must be NULL iff
 *                 in_place; in place, slab strides stay those of S and rows
 *                 [S_out, S) of every slab are left unspecified.
 * scores_out  out optional [B, V] fp32: head- and query-averaged attention
 */
int vscan_llm_prune(const vscan_llm_desc *desc, const void *q, void *k, void *v, void *hidden,
                    int32_t *kept_idx, void *k_out, void *v_out, void *hidden_out,
                    float *scores_out, void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * vscan_llm_prune for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Arguments, results and errors are those of vscan_llm_prune
 * without `workspace` / `workspace_bytes`: the scratch is a fixed array of
 * VSCAN_STATIC_SCRATCH_BYTES inside the library's code object, which every GPU
 * the library runs on holds until the process ends.  The call allocates and
 * frees nothing.
 *   - A descriptor whose vscan_llm_workspace_size exceeds
 *     VSCAN_STATIC_SCRATCH_BYTES is refused with VSCAN_ERR_WORKSPACE (nothing is
 *     enqueued).
 *   - The first call on a device looks the array's device address up (one
 *     symbol query, no allocation); make that call outside graph capture.
 *   - All calls on one GPU share the one array, which keeps the last call's
 *     contents: calls must be ordered (one stream, or events between streams);
 *     calls that overlap on one GPU race.
 * ------------------------------------------------------------------------- */
#define VSCAN_STATIC_SCRATCH_BYTES (16u << 20)
int vscan_llm_prune_static(const vscan_llm_desc *desc, const void *q, void *k, void *v,
                           void *hidden, int32_t *kept_idx, void *k_out, void *v_out,
                           void *hidden_out, float *scores_out, void *stream);

/* ---------------------------------------------------------------------------
 * Measurement aid (not part of the method): per-kernel device time.
 *
 * While enabled, every kernel the two entry points launch is bracketed by a pair
 * of HIP events on its stream.  vscan_profile_read waits for the recorded
 * events, adds the elapsed times up per kernel name and clears the record.
 * The switch and the record are process-wide host state; enable it only around
 * measurement passes (events cost a little launch latency) and do not toggle it
 * while another thread is inside an entry point.
 * ------------------------------------------------------------------------- */
typedef struct {
    char name[32];     /* kernel name, NUL-terminated */
    int32_t launches;  /* launches recorded since the last read */
    float total_ms;    /* summed event-to-event device time */
} vscan_kernel_time;

int vscan_profile_enable(int on);
/* out: host array of `capacity` entries; *count receives the entries written.
 * Returns VSCAN_ERR_HIP if an event query fails, VSCAN_ERR_NULL on NULL args. */
int vscan_profile_read(vscan_kernel_time *out, int capacity, int *count);

/* ---------------------------------------------------------------------------
 * Ragged stage-2 batches: every sequence has its own length, visual span and
 * budget (dynamic-resolution encoders emit between 4 and 16384 visual tokens per
 * image, Sec. 5.1 "Models"; re-selection for a later question in a multi-turn
 * dialogue, App. "Remarks on Multi-Turn Conversations", is the out-of-place call
 * again on the same pool).
 *
 * The descriptor gives what the sequences share (dtype, batch, heads, head_dim,
 * hidden, n_query, softmax_domain, scale, in_place) and the CAPACITIES:
 *   desc->seq_len  rows per sequence of k, v, hidden AND of the out-of-place
 *                  outputs (k_out, v_out [B,Hkv,seq_len,dh], hidden_out
 *                  [B,seq_len,hidden]: shaped like the inputs)
 *   desc->vis_len  row length of scores_out [B, vis_len] and of the workspace
 *                  (vscan_llm_workspace_size with this descriptor)
 *   desc->keep     row length of kept_idx [B, keep]
 *   desc->vis_start is ignored.
 * meta_host and meta_device hold the same `batch` entries, on the host (read and
 * validated by the call) and on the device (read by the kernels, so it must stay
 * valid and unchanged until the enqueued work has run).
 * Sequence b: scores_out[b, 0 .. vis_len_b), kept_idx[b, 0 .. keep_b) ascending and
 * -1 in the entries after them; its result occupies rows [0, seq_len_b - vis_len_b
 * + keep_b) of the destinations, later rows are left as they were.
 * Errors as vscan_llm_prune; a sequence that does not fit the capacities or its
 * own length gives VSCAN_ERR_SHAPE / VSCAN_ERR_BUDGET.
 * ------------------------------------------------------------------------- */
typedef struct {
    int32_t seq_len;   /* tokens of this sequence */
    int32_t vis_start; /* first visual position */
    int32_t vis_len;   /* visual tokens, >= 1 */
    int32_t keep;      /* visual tokens to keep, 0 .. vis_len */
} vscan_seq_meta;

int vscan_llm_prune_ragged(const vscan_llm_desc *desc, const vscan_seq_meta *meta_host,
                           const vscan_seq_meta *meta_device, const void *q, void *k, void *v,
                           void *hidden, int32_t *kept_idx, void *k_out, void *v_out,
                           void *hidden_out, float *scores_out, void *workspace,
                           size_t workspace_bytes, void *stream);

/* vscan_llm_prune_fused for a ragged batch: the table, the capacities and the shape of
 * hidden_out ([B, seq_len, hidden], rows past a sequence's result untouched) follow the
 * conventions above; everything else is as for vscan_llm_prune_fused (workspace from
 * vscan_llm_fused_workspace_size with the capacities). */
int vscan_llm_prune_fused_ragged(const vscan_llm_desc *desc, const vscan_seq_meta *meta_host,
                                 const vscan_seq_meta *meta_device, void *hidden, const void *w_q,
                                 const void *w_k_t, int32_t *kept_idx, void *hidden_out,
                                 float *scores_out, void *workspace, size_t workspace_bytes,
                                 void *stream);

/* ---------------------------------------------------------------------------
 * Stage 2 for a caller that does not hold the layer's queries and keys: the
 * scores of Eq. 5 computed as the equation is written, from the hidden states
 * and the layer's projection weights (Sec. 4.2: Q = x_last W_Q^h,
 * K_V = x_V W_K^h per head h, softmax over the key domain, mean over heads),
 * then the same top-`keep` selection, and the compaction applied to the hidden
 * states only (K and V of this layer do not exist yet; the caller computes them
 * for the tokens that are left).  With VSCAN_KEYS_ALL every query position
 * attends causally, to the keys up to and including its own position.  No positional rotation is applied to Q or K,
 * as in the equation.  bf16 or fp32 (hidden states and weights in desc->dtype).
 *
 * desc        HOST; as for vscan_llm_prune.  `hidden` and `head_dim` must be
 *             multiples of 8.
 * hidden      DEVICE [B, S, hidden]; in/out when in_place, else read only
 * w_q         DEVICE [Hq*dh, hidden], read only: row n holds the weights of
 *             output feature n (head n / dh), i.e. q = w_q x
 * w_k_t       DEVICE [hidden, Hkv*dh], read only: row c holds the weights that
 *             input feature c contributes to every output feature, i.e. the
 *             matrix W_K of the paper with the heads side by side (the
 *             transpose of the w_q convention; k = w_k_t^T x)
 * kept_idx    out [B, keep] int32 ascending
 * hidden_out  out [B, S_out, hidden], NULL when in_place
 * scores_out  out optional [B, V] fp32
 * workspace   vscan_llm_fused_workspace_size bytes, caller-owned, 16-byte aligned
 * Errors as vscan_llm_prune; sizes whose byte offsets inside one tensor do not
 * fit 32 bits give VSCAN_ERR_UNSUPPORTED.  Asynchronous on `stream`.
 * ------------------------------------------------------------------------- */
int vscan_llm_fused_workspace_size(const vscan_llm_desc *desc, size_t *bytes);
int vscan_llm_prune_fused(const vscan_llm_desc *desc, void *hidden, const void *w_q,
                          const void *w_k_t, int32_t *kept_idx, void *hidden_out,
                          float *scores_out, void *workspace, size_t workspace_bytes,
                          void *stream);

/* ---------------------------------------------------------------------------
 * Stage 1 for a caller that does not hold the attention layer's queries and
 * keys: the scores of Sec. 4.1 "Global Scan" computed as written, from the rows
 * the layer sees and its projection weights (Q = X W_Q^h, K = X W_K^h), then
 * the same local scan, global scan, assignment and merge as
 * vscan_encoder_reduce.  VSCAN_SCORE_CLS_ROW: the [CLS] row of
 * softmax(Q K^T * scale), mean over heads (Eq. 1-2).  VSCAN_SCORE_MEAN_RECEIVED
 * (encoders without a [CLS] token, last sentence of "Global Scan"): Q and K of
 * every token are projected (fp32) and the mean attention each token receives
 * is computed as in vscan_encoder_reduce; head_dim <= 128 there
 * (VSCAN_ERR_UNSUPPORTED otherwise).  bf16 or fp32 (hidden states and weights in
 * desc->dtype); projection biases are not part of the equations and not applied.
 *
 * desc          HOST; as for vscan_encoder_reduce; the hidden size of the layer
 *               is desc->feat_dim
 * hidden        DEVICE [B*C, S, feat_dim], S = has_cls + grid_h*grid_w, the
 *               [CLS] row first where there is one; read only
 * w_q           DEVICE [H*dh, feat_dim]  (row n: weights of output feature n)
 * w_k_t         DEVICE [feat_dim, H*dh]  (row c: what input feature c
 *               contributes; the paper's W_K with the heads side by side)
 * hidden_local, w_q_local, w_k_t_local
 *               optional (all three or none): the same of the shallow layer
 *               whose scores drive the local scan (Sec. 4.1 "Local Scan")
 * x, kept_idx, merged, assign_out, scores_out, stream: as vscan_encoder_reduce
 * workspace     vscan_encoder_fused_workspace_size bytes
 * ------------------------------------------------------------------------- */
int vscan_encoder_fused_workspace_size(const vscan_encoder_desc *desc, int with_local_triple,
                                       size_t *bytes);
int vscan_encoder_reduce_fused(const vscan_encoder_desc *desc, const void *hidden, const void *w_q,
                               const void *w_k_t, const void *hidden_local,
                               const void *w_q_local, const void *w_k_t_local, const void *x,
                               int32_t *kept_idx, void *merged, int32_t *assign_out,
                               float *scores_out, void *workspace, size_t workspace_bytes,
                               void *stream);

/* ---------------------------------------------------------------------------
 * Host-side budget arithmetic.  Pure functions of their arguments: no GPU, no
 * state; all pointers are HOST pointers.
 * ------------------------------------------------------------------------- */

/* Token counts of the two stages for retention rates r1 (encoder stage) and r2
 * (LLM stage), and the resulting average number of visual tokens over the LLM's
 * layers (Sec. 5.1 "Implementation Details"; App. "Remarks on Ensuring Fair
 * Comparisons": the first `prune_layer` of `n_layers` decoder layers see the
 * stage-1 count, the rest the stage-2 count).
 *   keep_encoder = nearest integer to r1 * n_visual   (halves round up)
 *   keep_llm     = nearest integer to r2 * keep_encoder
 *   avg_tokens   = (prune_layer * keep_encoder + (n_layers - prune_layer) * keep_llm) / n_layers
 * n_visual is the unit the budget applies to (one image, or one crop of a
 * multi-crop image).  Any output pointer may be NULL.
 * Errors: VSCAN_ERR_SHAPE (n_visual < 0, n_layers <= 0, prune_layer outside
 * [0, n_layers]), VSCAN_ERR_BUDGET (a rate outside [0, 1] or not finite). */
int vscan_budget(int32_t n_visual, int32_t n_layers, int32_t prune_layer, double r1, double r2,
                 int32_t *keep_encoder, int32_t *keep_llm, double *avg_tokens);

/* Inverse of the above for a fixed r2 (the paper fixes r2 = 33.3 % and adjusts
 * r1): the r1 whose layer-averaged retention equals avg_rate,
 *   r1 = avg_rate * n_layers / (prune_layer + (n_layers - prune_layer) * r2).
 * Errors as above, plus VSCAN_ERR_BUDGET when the answer would exceed 1 or the
 * denominator is zero. */
int vscan_budget_solve_r1(int32_t n_layers, int32_t prune_layer, double avg_rate, double r2,
                          double *r1);

/* Theoretical prefill FLOPs spent on visual tokens (Eq. 6, App. "Computational
 * Complexity"): sum over layers of 4 n d^2 + 2 n^2 d + 3 n d m, with
 * n = n_per_layer[layer] (host array of n_layers counts), d the hidden size and
 * m the FFN intermediate size.  Errors: VSCAN_ERR_NULL, VSCAN_ERR_SHAPE
 * (n_layers <= 0, d or m <= 0, a negative count). */
int vscan_flops(const int32_t *n_per_layer, int32_t n_layers, int64_t d, int64_t m,
                double *flops);

/* ---------------------------------------------------------------------------
 * Misc
 * ------------------------------------------------------------------------- */
const char *vscan_status_string(int status);
uint32_t vscan_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VSCAN_H */
