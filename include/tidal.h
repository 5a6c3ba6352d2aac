/*
 * tidal.h - C ABI of the MI355X (gfx950) decode-step attention library for
 * TidalDecode (arxiv 2410.05076).
 *
 * One decode step of the paper's Alg. 1 runs, per Transformer layer, one of
 * three attention kinds for the single new query of each sequence:
 *   - full attention over the whole KV cache (Eq. 1; Alg. 1 "FullAttention"),
 *   - full attention with token selection: the same, plus the inner products
 *     <q,K> of every cached token kept on the fly and rho := argTopK(<q,K>, k)
 *     (Sec. 3.1; Alg. 1 "Token Selection Layer"),
 *   - position persistent sparse attention over the rows named by the latest
 *     rho only (Sec. 3.1; Alg. 1 "SparseAttention(q, C[rho])").
 * The entry points below are those three calls, the argTopK step on its own,
 * and a driver that applies a layer schedule (Fig. 2: full attention in the
 * first layers, selection at the next layer and one middle layer, sparse
 * elsewhere).
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers unless a comment says HOST.  The
 *     caller owns q, K, V, out, positions, seq_lens; the library owns only the
 *     workspace inside td_ctx, never frees or reallocates caller memory, and
 *     never synchronises the stream: kernels are enqueued on `hip_stream`
 *     (a hipStream_t passed as void*, NULL = the null stream) and the call
 *     returns.  No call other than td_create / td_destroy allocates or frees.
 *   - q, out : [batch][num_q_heads][head_dim], contiguous, element type `dtype`.
 *   - K, V   : element type `dtype`; element (b, g, j, c) of either lives at
 *              b*kv_stride_batch + g*kv_stride_head + j*kv_stride_tok + c
 *              (strides in elements, multiples of 8; head_dim contiguous).
 *              Token j of sequence b is valid for 0 <= j < seq_lens[b]; the
 *              cache already holds the current token (Alg. 1 appends first),
 *              so 1 <= seq_lens[b] <= max_seq_len.  The lengths live in device
 *              memory and are not checked: values above max_seq_len count as
 *              max_seq_len, and for a sequence of length 0 (or less) the decode
 *              calls leave its rows of `out` untouched and fill its rho with -1.
 *     Pointers must be 16-byte aligned.
 *   - Paged cache (shape.page_size > 0; serving systems hand the cache out in
 *     pages, as the paged full-attention baseline and the page-level method
 *     of the paper's Sec. 4 do): K and V point to page pools shared by all
 *     sequences; element (page p, KV head g, slot s, c) lives at
 *     p*kv_stride_batch + g*kv_stride_head + s*kv_stride_tok + c, and token j
 *     of sequence b is in page block_table[b*block_table_stride + j/page_size]
 *     at slot j % page_size.  Scores, positions and seq_lens stay in logical
 *     token indices, so every call means the same as on the contiguous cache
 *     holding the same tokens.  Only entries of pages that hold a token
 *     j < seq_lens[b] are read; an id outside [0, num_pages) is clamped into
 *     the pool (no access outside it; the result for that sequence is then
 *     unspecified).  The layers of td_decode_step share one block table.
 *   - Query head h reads KV head h / (num_q_heads / num_kv_heads).
 *   - positions : int32 [batch][num_kv_heads][k], ascending token indices; if
 *     k > seq_lens[b] only the first seq_lens[b] entries are tokens and the
 *     rest are -1.  Sparse attention skips entries that are negative or
 *     >= seq_lens[b]; a (sequence, KV head) with no valid entry yields zeros.
 *   - Arithmetic: logits, softmax and accumulation in fp32; out is rounded to
 *     `dtype` (round to nearest even for bf16).
 *   - Grouped-query selection: the query heads that share a KV head share one
 *     rho; the top-k is taken over the per-token sum of the group's scaled
 *     logits (for num_q_heads == num_kv_heads this is the paper's per-head
 *     argTopK).  Ties at the k-th value go to the smaller token index.
 *   - Errors: argument errors are found on the host before anything is
 *     enqueued and returned as TD_ERR_INVALID_ARG / TD_ERR_UNSUPPORTED /
 *     TD_ERR_WORKSPACE; a failed HIP call gives TD_ERR_HIP.  td_last_error
 *     returns a text for the most recent failure on that context.
 *     Supported: head_dim 64 or 128, group size 1, 2, 4 or 8,
 *     batch * num_kv_heads <= 65535, max_seq_len <= 2^30 (2^20 for calls with a
 *     token budget).
 *   - A context serves one stream at a time: calls that use the same context
 *     must be ordered on one stream (they share its workspace).
 */
#ifndef TIDAL_H
#define TIDAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TD_OK = 0,
    TD_ERR_INVALID_ARG = 1,
    TD_ERR_UNSUPPORTED = 2,
    TD_ERR_WORKSPACE = 3,
    TD_ERR_HIP = 4
} td_status;

typedef enum { TD_BF16 = 0, TD_F32 = 1 } td_dtype;

/* How the query heads that share a KV head agree on rho (the paper describes selection per
 * attention head, Sec. 3.1, and is silent on grouped-query attention):
 *   TD_SELECT_GROUP_SUM  top-k over the per-token sum of the group's scaled logits (default);
 *   TD_SELECT_GROUP_MAX  top-k over their per-token maximum;
 *   TD_SELECT_GROUP_MEAN_PROB  top-k over the mean of the heads' attention probabilities
 *                        softmax(s_h)[j] over the whole cache; needs the final softmax
 *                        statistics, so the scores are formed in a second small pass over the
 *                        per-head logits (group_scores then holds probabilities);
 *   TD_SELECT_PER_HEAD   no agreement: every query head selects by its own logits, the
 *                        paper's literal rule.  positions (and group_scores) then have one
 *                        row per QUERY head, [batch][num_q_heads][k], and a sparse layer
 *                        gathers each head's own rows: group-size times the gather traffic.
 * All of them select the same tokens when num_q_heads == num_kv_heads. */
typedef enum {
    TD_SELECT_GROUP_SUM = 0,
    TD_SELECT_GROUP_MAX = 1,
    TD_SELECT_PER_HEAD = 2,
    TD_SELECT_GROUP_MEAN_PROB = 3
} td_selection;

/* Layer kinds of Alg. 1. */
typedef enum { TD_LAYER_DENSE = 0, TD_LAYER_SELECT = 1, TD_LAYER_SPARSE = 2 } td_layer_kind;

typedef struct td_shape {
    int32_t batch;
    int32_t num_q_heads;
    int32_t num_kv_heads;      /* divides num_q_heads */
    int32_t head_dim;          /* 64 or 128 */
    int32_t dtype;             /* td_dtype of q, K, V, out */
    float   sm_scale;          /* 0 => 1/sqrt(head_dim), the scaling of Eq. 1 */
    int64_t kv_stride_batch;   /* elements */
    int64_t kv_stride_head;
    int64_t kv_stride_tok;
    const int32_t *seq_lens;   /* DEVICE int32 [batch]; each in [1, max_seq_len] */
    int32_t max_seq_len;       /* HOST-known upper bound; sizes grids and workspace */
    int64_t total_seq_len;     /* HOST hint: sum of seq_lens, or 0 if unknown.  Only steers the
                                  launch plan (a ragged batch gets smaller chunks); results do
                                  not depend on it */
    /* Paged cache (page_size == 0: the contiguous cache described above, the rest unused). */
    int32_t page_size;         /* tokens per page, a power of two */
    int32_t num_pages;         /* pages in the pools that K and V point to */
    const int32_t *block_table; /* DEVICE int32 [batch][block_table_stride] page ids */
    int64_t block_table_stride; /* entries per sequence, >= ceil(max_seq_len / page_size) */
    int32_t selection;         /* td_selection; 0 = the group sum */
} td_shape;

typedef struct td_ctx td_ctx;  /* opaque; owns the workspace (split partials, group scores) */

/* Host-only check of a shape and budget; the same check every call makes first. */
td_status td_validate(const td_shape *shape, int32_t k);

/* Workspace bytes that any call with this shape and budget k (k <= 0: no
 * selection or sparse call will be made) needs.  Returns 0 for an invalid shape. */
size_t td_workspace_bytes(const td_shape *shape, int32_t k);

/* Workspace bytes that td_topk needs for `rows` rows of at most `max_len` scores. */
size_t td_topk_workspace_bytes(int32_t rows, int32_t max_len);

/* Creates a context on HIP device `device` and allocates `workspace_bytes` of
 * device memory once.  Synchronises the device. */
td_status td_create(td_ctx **out, int device, size_t workspace_bytes);
td_status td_destroy(td_ctx *ctx);

/* FullAttention(q, C[:]) of Alg. 1 (Eq. 1 for one query row per head). */
td_status td_full_attend(td_ctx *ctx, const td_shape *shape, const void *q, const void *K,
                         const void *V, void *out, void *hip_stream);

/* Token selection layer of Alg. 1: out as td_full_attend; positions receives
 * rho.  group_scores (optional, may be NULL) receives the fp32 per-token sums
 * of scaled logits, [batch][num_kv_heads][max_seq_len], entries at or beyond
 * seq_lens[b] untouched; when NULL they are kept in the workspace. */
td_status td_select_tokens(td_ctx *ctx, const td_shape *shape, const void *q, const void *K,
                           const void *V, int32_t k, void *out, int32_t *positions,
                           float *group_scores, void *hip_stream);

/* SparseAttention(q, C[rho]) of Alg. 1. */
td_status td_sparse_attend(td_ctx *ctx, const td_shape *shape, const void *q, const void *K,
                           const void *V, const int32_t *positions, int32_t k, void *out,
                           void *hip_stream);

/* argTopK of Alg. 1 on its own: for each of `rows` rows of fp32 scores (row r
 * at scores + r*row_stride, its length row_lens[r / rows_per_len], row_lens a
 * DEVICE int32 array) writes the ascending indices of the min(k, len) largest
 * scores to positions + r*k, -1 padded.  Scores must not be NaN: a row with a NaN gets
 * an unspecified selection (nothing is written outside its k entries). */
td_status td_topk(td_ctx *ctx, const float *scores, int64_t row_stride, int32_t rows,
                  const int32_t *row_lens, int32_t rows_per_len, int32_t max_len, int32_t k,
                  int32_t *positions, void *hip_stream);

/* The layer loop of Alg. 1, attention part only.  schedule, q_layers,
 * K_layers, V_layers, out_layers are HOST arrays of num_layers entries (the
 * pointers inside are device pointers; every layer shares `shape`).  The i-th
 * selection layer writes rho to positions + i*batch*num_kv_heads*k
 * (positions: int32 [n_select][batch][num_kv_heads][k]); each sparse layer
 * reads the most recent one.  A sparse layer before any selection layer is
 * TD_ERR_INVALID_ARG. */
td_status td_decode_step(td_ctx *ctx, const td_shape *shape, int32_t num_layers,
                         const int32_t *schedule, const void *const *q_layers,
                         const void *const *K_layers, const void *const *V_layers, int32_t k,
                         void *const *out_layers, int32_t *positions, void *hip_stream);

/* Attention of a prefill over the last `num_new` tokens of every sequence - the attention of the
 * cache-correction step (Sec. 3.2), which re-runs full attention for the tokens that were decoded
 * sparsely.  q, out: [batch][num_new][num_q_heads][head_dim]; token j of sequence b sits at
 * position seq_lens[b] - num_new + j (its key and value are already in the cache) and attends,
 * with Eq. 1, to the positions up to and including its own; a token that would sit before the
 * start of the cache (num_new > seq_lens[b]) yields zeros.
 * Two paths.  bf16 with head_dim 128, a contiguous cache or a paged one with pages of 16 tokens
 * or more, kv_stride_tok <= 2^24 elements: a kernel on the matrix cores that reads the cache
 * once per call.  A prefill over few tokens is bound by the stream of the cache, as a decode step
 * is: the tokens are then cut into chunks whose partial states go through the context's workspace.
 * Every other shape the decode calls accept (fp32, head_dim 64, smaller pages, longer token
 * strides): the plain path - the matrix-core kernel is built around the 16x16x32 bf16 tile (128
 * channels are eight of its channel groups, a 16-token half tile comes from one page) and has no
 * vector-ALU twin, so these shapes run the full-attention kernel of the decode step with one grid
 * row block per new token, each attending to the positions up to its own.  That reads the cache
 * once per new token instead of once per call: right for the short corrections the step is meant
 * for, slow for long ones.
 * td_prefill_workspace_bytes is the size that allows every chunk the launch plan would like
 * (matrix-core path; 0 when it wants none) or all new tokens of all sequences in one launch
 * (plain path).  With a smaller workspace the call uses fewer chunks, down to one (correct, slower
 * when num_new * num_q_heads / num_kv_heads rows are too few to fill the GPU), or runs of as many
 * new tokens of one sequence per launch as fit; TD_ERR_WORKSPACE if the plain path has no room
 * for a single token (td_workspace_bytes(shape, 0) is always enough). */
size_t td_prefill_workspace_bytes(const td_shape *shape, int32_t num_new);
td_status td_prefill_attend(td_ctx *ctx, const td_shape *shape, int32_t num_new, const void *q,
                            const void *K, const void *V, void *out, void *hip_stream);

/* The same with C.append(k, v) of Alg. 1 fused into each layer's launch: layer
 * i first appends the current token's key and value, k_new_layers[i] and
 * v_new_layers[i] ([batch][num_kv_heads][head_dim], element type `dtype`,
 * 16-byte aligned; the key already carries its rotary embedding - that is
 * part of the projection that produces q, k, v), as token seq_lens[b] - 1 of
 * K_layers[i] / V_layers[i] (seq_lens counts the current token) and then
 * attends over the cache including it.  The caches are written in place (one
 * row per sequence and KV head, through the block table if paged); rows
 * before seq_lens[b] - 1 must already hold the earlier tokens, that row's old
 * contents are never read. */
td_status td_decode_step_append(td_ctx *ctx, const td_shape *shape, int32_t num_layers,
                                const int32_t *schedule, const void *const *q_layers,
                                const void *const *k_new_layers, const void *const *v_new_layers,
                                void *const *K_layers, void *const *V_layers, int32_t k,
                                void *const *out_layers, int32_t *positions, void *hip_stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): td_decode_step without a context.  The workspace is a device array with
 * static storage inside the library, TD_STATIC_SCRATCH_BYTES per GPU that the library runs on, held
 * until the process ends; the call allocates and frees nothing and uses the default launch plan.
 * Arguments and results are those of td_decode_step.  Shapes with td_workspace_bytes(shape, k) above
 * TD_STATIC_SCRATCH_BYTES return TD_ERR_WORKSPACE before anything is enqueued (the single-sequence
 * benchmark shapes up to 128K tokens and batch 4 x 128K fit; batch 16 x 64K does not).  The kernels
 * run on the device that is current when the call is made; `hip_stream` must belong to it.  Every
 * call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two threads)
 * race and give undefined results; calls ordered on one stream are safe, each one zeroes the ticket
 * counters it uses first.  td_last_error(NULL) returns the text of this thread's last failure. */
#define TD_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
td_status td_decode_step_static(const td_shape *shape, int32_t num_layers, const int32_t *schedule,
                                const void *const *q_layers, const void *const *K_layers,
                                const void *const *V_layers, int32_t k, void *const *out_layers,
                                int32_t *positions, void *hip_stream);

/* Host-only: how a layer of kind `layer_kind` (td_layer_kind) would be launched for this shape
 * and budget - nothing is enqueued.  ctx may be NULL (default tuning).  For sizing, logging
 * and tests of the launch planning. */
typedef struct td_launch_plan {
    int32_t chunk_tokens;        /* tokens (or selected positions) per workgroup */
    int32_t chunks_per_row;      /* workgroups per (sequence, KV head) */
    int32_t waves_per_workgroup; /* 4 or 8 wave64s */
    int32_t matrix_core;         /* 1: the MFMA kernel, 0: the vector-ALU kernel */
    int32_t grid_rows;           /* batch * KV heads (query heads for a per-head sparse layer) */
    int32_t merge_launch;        /* 1: a second small launch folds the chunk partials, 0: the last chunk does */
    int64_t workgroups;          /* grid_rows * chunks_per_row, empty chunks of short sequences included */
} td_launch_plan;
td_status td_plan_launch(const td_ctx *ctx, const td_shape *shape, int32_t layer_kind, int32_t k,
                         td_launch_plan *plan);

/* Tuning knobs for measurement sweeps (0 keeps the default): target number of
 * workgroups per attention launch, the smallest token chunk per workgroup for
 * full and for sparse attention, the largest number of chunks per
 * (sequence, KV head), and the attention kernel (0: chosen per launch - the
 * matrix-core kernel where it applies (bf16, head_dim 128) and is the faster
 * one (groups of four or more query heads; full layers of smaller groups), else
 * the vector-ALU kernel; four or eight waves per workgroup; 1: the matrix-core
 * kernel wherever it applies; 2 / 3:
 * the vector-ALU kernel with four / eight waves per workgroup in every launch;
 * 4 / 5: the same for the matrix-core kernel; plus 8: the chunk partials of
 * every split launch are folded by a second small launch, plus 16: by the
 * chunk that finishes last, instead of the choice per launch (the last chunk,
 * except in the full and selection layers of a ragged batch - see
 * total_seq_len - where a workgroup slot serves several chunks in turn and a
 * second launch is the faster way); plus 32, for
 * timing only: selection calls stop after their attention launch - out and the
 * scores are written, positions are not).  The workspace size does not depend
 * on them. */
td_status td_set_tuning(td_ctx *ctx, int32_t target_workgroups, int32_t min_chunk_dense,
                        int32_t min_chunk_sparse, int32_t max_splits, int32_t kernel_variant);

/* Split launches of the attention calls meet through ticket counters in the context's workspace
 * (one per sequence and KV head), which every launch leaves at zero.  td_reset enqueues a kernel
 * on `hip_stream` that zeroes them: the way back for a context whose launch was cut short (a
 * device error, a process that aborted a stream) or that two streams used at once, both of which
 * would otherwise leave every later result on that context undefined.  A launch that the library
 * itself sees fail triggers the same clearing before the next attention call.  Costs one small
 * launch; not needed in normal operation. */
td_status td_reset(td_ctx *ctx, void *hip_stream);

/* Measurement helper, not part of the attention path: a plain streaming kernel
 * of known size.  Copies `bytes` (rounded down to 16) from src to dst, or only
 * reads src when dst is NULL.  Used to calibrate hardware counters and to
 * report a measured streaming rate next to the published HBM peak.  It touches
 * nothing of the context's workspace (its only write besides dst goes to a word
 * that the context allocates for this call alone). */
td_status td_probe_stream(td_ctx *ctx, void *dst, const void *src, size_t bytes, void *hip_stream);

const char *td_status_string(td_status s);
const char *td_last_error(const td_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* TIDAL_H */
