/*
 * CPU oracle for TidalDecode's decode-step attention (arxiv 2410.05076).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp32
 * implementation of what the HIP path must compute, written from the paper's
 * definitions.  It shares no code with the HIP kernels and must only be used
 * by the tests, the smoke check and the bench's cpu_baseline leg.
 *
 * Notation (paper, Sec. 3.1 and Alg. 1): one new query per head, KV cache of
 * N tokens that already contains the current token (Alg. 1 appends before it
 * attends), token budget k (the paper also writes m and K for it).
 *
 *   full   : Eq. 1 for a single query row, o = softmax(q K^T / sqrt(d)) V
 *   select : full attention, plus the inner products <q,K> kept for every
 *            cached token and the k largest picked (Alg. 1, token selection
 *            layer; Sec. 3.1 "stores the inner product ... on the fly")
 *   sparse : Eq. 1 restricted to the persisted positions rho
 *            (Alg. 1, "SparseAttention(q, C[rho])")
 *   step   : Alg. 1's layer loop, attention part only
 *   prefill: full attention for the last P tokens of a sequence with the causal rule (the
 *            attention of the cache-correction step, Sec. 3.2)
 *   paged  : the same results for a cache stored in pages behind a block
 *            table (tdo_gather_pages states the mapping)
 *
 * Readings where the paper is silent (kept identical in the HIP path):
 *   - grouped-query attention: the G query heads that share a KV head select
 *     one common token set; their scaled logits are summed per token and the
 *     top-k is taken over that sum (for G = 1 this is exactly the paper's
 *     per-head argTopK);
 *   - ties go to the smaller index; rho is emitted in ascending index order;
 *   - k > N: k_eff = min(k, N) positions, the tail of rho is -1, and sparse
 *     attention skips negative entries;
 *   - no causal mask (one query, every cached position is visible).
 *
 * Arithmetic: inputs are fp32 or bf16 (upcast exactly), everything else is
 * sequential fp32 in the index order written here.
 *
 * Parity against paper-printed values: parity unpinned (the paper prints no
 * scores, positions or attention outputs).  The pins are brute force in
 * float64, closed forms and invariants; see tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { TDO_BF16 = 0, TDO_F32 = 1 };
enum { TDO_DENSE = 0, TDO_SELECT = 1, TDO_SPARSE = 2 };
enum { TDO_OK = 0, TDO_BAD_ARG = 1, TDO_NO_MEM = 2, TDO_BAD_POSITION = 3,
       TDO_SPARSE_BEFORE_SELECT = 4 };

typedef struct {
    int32_t batch;        /* B */
    int32_t num_q_heads;  /* Hq */
    int32_t num_kv_heads; /* Hkv, Hq % Hkv == 0 */
    int32_t head_dim;     /* d */
    int32_t dtype;        /* of q, K, V: TDO_BF16 (uint16 storage) or TDO_F32 */
    float   sm_scale;     /* 0 => 1/sqrt(d) (Eq. 1) */
    int64_t kv_stride_batch, kv_stride_head, kv_stride_tok; /* elements */
    const int32_t *seq_lens; /* [B], N_b >= 1, includes the current token */
    int32_t max_seq_len;
} tdo_shape;

static inline float load_elem(const void *base, int dtype, int64_t i) {
    if (dtype == TDO_F32) return ((const float *)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

static float scale_of(const tdo_shape *s) {
    return s->sm_scale != 0.0f ? s->sm_scale : 1.0f / sqrtf((float)s->head_dim);
}

static int shape_ok(const tdo_shape *s) {
    if (!s || !s->seq_lens) return 0;
    if (s->batch < 1 || s->num_q_heads < 1 || s->num_kv_heads < 1 || s->head_dim < 1) return 0;
    if (s->num_q_heads % s->num_kv_heads) return 0;
    if (s->dtype != TDO_BF16 && s->dtype != TDO_F32) return 0;
    for (int b = 0; b < s->batch; ++b)
        if (s->seq_lens[b] < 1 || s->seq_lens[b] > s->max_seq_len) return 0;
    return 1;
}

/*
 * Eq. 1 for one query head against the rows listed in idx[0..n) (idx == NULL
 * means rows 0..n-1).  Negative idx entries are skipped.  logits (optional)
 * receives the scaled inner product of every visited slot t (untouched for
 * skipped slots).  work holds n floats.  Returns the number of rows attended.
 */
static int attend_one(const void *q, int64_t q_off, const void *K, const void *V, int64_t kv_off,
                      int64_t stride_tok, int d, int dtype, float scale, const int32_t *idx,
                      int n, float *out, float *logits, float *work) {
    float m = -INFINITY;
    int used = 0;
    for (int t = 0; t < n; ++t) {
        int64_t j = idx ? idx[t] : t;
        if (j < 0) { work[t] = -INFINITY; continue; }
        float acc = 0.0f;
        for (int c = 0; c < d; ++c)
            acc += load_elem(q, dtype, q_off + c) * load_elem(K, dtype, kv_off + j * stride_tok + c);
        float s = acc * scale;
        work[t] = s;
        if (logits) logits[t] = s;
        if (s > m) m = s;
        ++used;
    }
    for (int c = 0; c < d; ++c) out[c] = 0.0f;
    if (!used) return 0;
    float l = 0.0f;
    for (int t = 0; t < n; ++t) {
        int64_t j = idx ? idx[t] : t;
        if (j < 0) continue;
        float p = expf(work[t] - m);
        l += p;
        for (int c = 0; c < d; ++c)
            out[c] += p * load_elem(V, dtype, kv_off + j * stride_tok + c);
    }
    for (int c = 0; c < d; ++c) out[c] /= l;
    return used;
}

/* Full attention (Alg. 1, full attention layer).  out: fp32 [B][Hq][d].
 * logits (optional): fp32 [B][Hq][max_seq_len], scaled inner products. */
int tdo_full(const tdo_shape *s, const void *q, const void *K, const void *V, float *out,
             float *logits) {
    if (!shape_ok(s) || !q || !K || !V || !out) return TDO_BAD_ARG;
    const int G = s->num_q_heads / s->num_kv_heads, d = s->head_dim;
    const float scale = scale_of(s);
    int err = TDO_OK;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < s->batch; ++b)
        for (int h = 0; h < s->num_q_heads; ++h) {
            int N = s->seq_lens[b], g = h / G;
            float *work = (float *)malloc((size_t)N * sizeof(float));
            if (!work) { err = TDO_NO_MEM; continue; }
            int64_t qo = ((int64_t)b * s->num_q_heads + h) * d;
            int64_t kvo = b * s->kv_stride_batch + g * s->kv_stride_head;
            attend_one(q, qo, K, V, kvo, s->kv_stride_tok, d, s->dtype, scale, NULL, N,
                       out + qo, logits ? logits + ((int64_t)b * s->num_q_heads + h) * s->max_seq_len : NULL,
                       work);
            free(work);
        }
    return err;
}

typedef struct { float score; int32_t index; } scored;

/* larger score first; equal scores: smaller index first */
static int by_score_desc(const void *a, const void *b) {
    const scored *x = (const scored *)a, *y = (const scored *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->index > y->index) - (x->index < y->index);
}

static int by_int_asc(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* argTopK of Alg. 1 over one row of n scores: the min(k, n) largest, ties to
 * the smaller index, written in ascending index order, -1 padded up to k. */
int tdo_topk_row(const float *scores, int n, int k, int32_t *positions) {
    if (!scores || !positions || n < 1 || k < 1) return TDO_BAD_ARG;
    scored *tmp = (scored *)malloc((size_t)n * sizeof(scored));
    if (!tmp) return TDO_NO_MEM;
    for (int j = 0; j < n; ++j) { tmp[j].score = scores[j]; tmp[j].index = j; }
    qsort(tmp, (size_t)n, sizeof(scored), by_score_desc);
    int ke = k < n ? k : n;
    for (int t = 0; t < ke; ++t) positions[t] = tmp[t].index;
    qsort(positions, (size_t)ke, sizeof(int32_t), by_int_asc);
    for (int t = ke; t < k; ++t) positions[t] = -1;
    free(tmp);
    return TDO_OK;
}

/*
 * Token selection layer (Alg. 1): full attention, then for each KV head g the
 * per-token sum over the group's G query heads of the scaled inner products,
 * r_g[j] = sum_{h in g} s_h[j] (h ascending), and rho_g = argTopK(r_g, k).
 * out: fp32 [B][Hq][d]; positions: int32 [B][Hkv][k];
 * group_scores (optional): fp32 [B][Hkv][max_seq_len].
 */
int tdo_select(const tdo_shape *s, const void *q, const void *K, const void *V, int32_t k,
               float *out, int32_t *positions, float *group_scores) {
    if (!shape_ok(s) || !positions || k < 1) return TDO_BAD_ARG;
    const int G = s->num_q_heads / s->num_kv_heads;
    const int64_t maxN = s->max_seq_len;
    float *logits = (float *)malloc((size_t)s->batch * s->num_q_heads * maxN * sizeof(float));
    if (!logits) return TDO_NO_MEM;
    int err = tdo_full(s, q, K, V, out, logits);
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < s->batch; ++b)
        for (int g = 0; g < s->num_kv_heads; ++g) {
            int N = s->seq_lens[b];
            float *r = (float *)malloc((size_t)N * sizeof(float));
            if (!r) { err = TDO_NO_MEM; continue; }
            for (int j = 0; j < N; ++j) {
                float acc = 0.0f;
                for (int i = 0; i < G; ++i)
                    acc += logits[((int64_t)b * s->num_q_heads + g * G + i) * maxN + j];
                r[j] = acc;
            }
            int e = tdo_topk_row(r, N, k, positions + ((int64_t)b * s->num_kv_heads + g) * k);
            if (e) err = e;
            if (group_scores)
                memcpy(group_scores + ((int64_t)b * s->num_kv_heads + g) * maxN, r,
                       (size_t)N * sizeof(float));
            free(r);
        }
    free(logits);
    return err;
}

/*
 * Variants of the selection rule for grouped-query attention.  The paper
 * describes selection per attention head (Sec. 3.1) and does not say how the
 * query heads that share a KV head agree on one token set; tdo_select above
 * takes the sum of the group's scaled logits.  The alternatives:
 *   TDO_REDUCE_MAX  r_g[j] = max_{h in g} s_h[j], one rho per KV head;
 *   TDO_REDUCE_MEAN_PROB  r_g[j] = (1/G) sum_{h in g} softmax(s_h)[j]: the mean of the heads'
 *                   attention probabilities over the whole cache (the selection by "highest
 *                   attention scores" of Sec. 3.1 read on probabilities), one rho per KV head;
 *   TDO_PER_HEAD    no reduction: rho_h = argTopK(s_h, k) for every query head,
 *                   the paper's literal rule; positions are [B][Hq][k] and a
 *                   sparse layer gathers each head's own rows (tdo_sparse_per_head).
 * scores (optional): fp32 [B][Hkv][max_seq_len] for the reductions,
 * [B][Hq][max_seq_len] for TDO_PER_HEAD.
 */
enum { TDO_REDUCE_SUM = 0, TDO_REDUCE_MAX = 1, TDO_PER_HEAD = 2, TDO_REDUCE_MEAN_PROB = 3 };

int tdo_select_variant(const tdo_shape *s, int variant, const void *q, const void *K, const void *V,
                       int32_t k, float *out, int32_t *positions, float *scores) {
    if (variant == TDO_REDUCE_SUM) return tdo_select(s, q, K, V, k, out, positions, scores);
    if (!shape_ok(s) || !positions || k < 1 ||
        (variant != TDO_REDUCE_MAX && variant != TDO_PER_HEAD && variant != TDO_REDUCE_MEAN_PROB))
        return TDO_BAD_ARG;
    const int G = s->num_q_heads / s->num_kv_heads;
    const int64_t maxN = s->max_seq_len;
    float *logits = (float *)malloc((size_t)s->batch * s->num_q_heads * maxN * sizeof(float));
    if (!logits) return TDO_NO_MEM;
    int err = tdo_full(s, q, K, V, out, logits);
    const int rows = variant == TDO_PER_HEAD ? s->num_q_heads : s->num_kv_heads;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < s->batch; ++b)
        for (int x = 0; x < rows; ++x) {
            int N = s->seq_lens[b];
            float *r = (float *)malloc((size_t)N * sizeof(float));
            if (!r) { err = TDO_NO_MEM; continue; }
            if (variant == TDO_REDUCE_MEAN_PROB) {
                for (int j = 0; j < N; ++j) r[j] = 0.0f;
                for (int i = 0; i < G; ++i) {
                    const float *sl = logits + ((int64_t)b * s->num_q_heads + x * G + i) * maxN;
                    float m = sl[0], l = 0.0f;
                    for (int j = 1; j < N; ++j) if (sl[j] > m) m = sl[j];
                    for (int j = 0; j < N; ++j) l += expf(sl[j] - m);
                    for (int j = 0; j < N; ++j) r[j] += expf(sl[j] - m) / l;
                }
                for (int j = 0; j < N; ++j) r[j] /= (float)G;
            }
            for (int j = 0; j < N && variant != TDO_REDUCE_MEAN_PROB; ++j) {
                if (variant == TDO_PER_HEAD) {
                    r[j] = logits[((int64_t)b * s->num_q_heads + x) * maxN + j];
                } else {
                    float best = logits[((int64_t)b * s->num_q_heads + x * G) * maxN + j];
                    for (int i = 1; i < G; ++i) {
                        float v = logits[((int64_t)b * s->num_q_heads + x * G + i) * maxN + j];
                        if (v > best) best = v;
                    }
                    r[j] = best;
                }
            }
            int e = tdo_topk_row(r, N, k, positions + ((int64_t)b * rows + x) * k);
            if (e) err = e;
            if (scores) memcpy(scores + ((int64_t)b * rows + x) * maxN, r, (size_t)N * sizeof(float));
            free(r);
        }
    free(logits);
    return err;
}

/* Sparse attention with one rho per query head: positions [B][Hq][k]; head h
 * attends over its own rows of KV head h / G.  Otherwise as tdo_sparse. */
int tdo_sparse_per_head(const tdo_shape *s, const void *q, const void *K, const void *V,
                        const int32_t *positions, int32_t k, float *out) {
    if (!shape_ok(s) || !q || !K || !V || !out || !positions || k < 1) return TDO_BAD_ARG;
    const int G = s->num_q_heads / s->num_kv_heads, d = s->head_dim;
    const float scale = scale_of(s);
    for (int b = 0; b < s->batch; ++b)
        for (int64_t t = 0; t < (int64_t)s->num_q_heads * k; ++t)
            if (positions[(int64_t)b * s->num_q_heads * k + t] >= s->seq_lens[b])
                return TDO_BAD_POSITION;
    int err = TDO_OK;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < s->batch; ++b)
        for (int h = 0; h < s->num_q_heads; ++h) {
            float *work = (float *)malloc((size_t)k * sizeof(float));
            if (!work) { err = TDO_NO_MEM; continue; }
            int64_t qo = ((int64_t)b * s->num_q_heads + h) * d;
            int64_t kvo = b * s->kv_stride_batch + (h / G) * s->kv_stride_head;
            attend_one(q, qo, K, V, kvo, s->kv_stride_tok, d, s->dtype, scale,
                       positions + ((int64_t)b * s->num_q_heads + h) * k, k, out + qo, NULL, work);
            free(work);
        }
    return err;
}

/* Position persistent sparse attention (Alg. 1, sparse layer): Eq. 1 over the
 * non-negative entries of positions [B][Hkv][k] only.  An entry >= N_b is an
 * error.  A (b, g) with no valid entry yields zeros. */
int tdo_sparse(const tdo_shape *s, const void *q, const void *K, const void *V,
               const int32_t *positions, int32_t k, float *out) {
    if (!shape_ok(s) || !q || !K || !V || !out || !positions || k < 1) return TDO_BAD_ARG;
    const int G = s->num_q_heads / s->num_kv_heads, d = s->head_dim;
    const float scale = scale_of(s);
    for (int b = 0; b < s->batch; ++b)
        for (int64_t t = 0; t < (int64_t)s->num_kv_heads * k; ++t)
            if (positions[(int64_t)b * s->num_kv_heads * k + t] >= s->seq_lens[b])
                return TDO_BAD_POSITION;
    int err = TDO_OK;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < s->batch; ++b)
        for (int h = 0; h < s->num_q_heads; ++h) {
            int g = h / G;
            float *work = (float *)malloc((size_t)k * sizeof(float));
            if (!work) { err = TDO_NO_MEM; continue; }
            int64_t qo = ((int64_t)b * s->num_q_heads + h) * d;
            int64_t kvo = b * s->kv_stride_batch + g * s->kv_stride_head;
            attend_one(q, qo, K, V, kvo, s->kv_stride_tok, d, s->dtype, scale,
                       positions + ((int64_t)b * s->num_kv_heads + g) * k, k, out + qo, NULL, work);
            free(work);
        }
    return err;
}

/*
 * Alg. 1's layer loop, attention part only: rho starts empty; a selection
 * layer overwrites it; every sparse layer reads the latest one.  The queries
 * of all layers are inputs (the projection and FFN between layers need model
 * weights and are not part of this path).
 * positions: int32 [n_select][B][Hkv][k], slot i written by the i-th
 * selection layer (keeping every slot lets a test see each rho).
 */
int tdo_step(const tdo_shape *s, int32_t num_layers, const int32_t *schedule,
             const void *const *q_layers, const void *const *K_layers, const void *const *V_layers,
             int32_t k, float *const *out_layers, int32_t *positions) {
    if (!shape_ok(s) || num_layers < 1 || !schedule || !q_layers || !K_layers || !V_layers ||
        !out_layers || !positions || k < 1)
        return TDO_BAD_ARG;
    const int64_t slot = (int64_t)s->batch * s->num_kv_heads * k;
    const int32_t *rho = NULL;
    int n_sel = 0;
    for (int i = 0; i < num_layers; ++i) {
        int e;
        switch (schedule[i]) {
        case TDO_DENSE:
            e = tdo_full(s, q_layers[i], K_layers[i], V_layers[i], out_layers[i], NULL);
            break;
        case TDO_SELECT: {
            int32_t *dst = positions + slot * n_sel++;
            e = tdo_select(s, q_layers[i], K_layers[i], V_layers[i], k, out_layers[i], dst, NULL);
            rho = dst;
            break;
        }
        case TDO_SPARSE:
            if (!rho) return TDO_SPARSE_BEFORE_SELECT;
            e = tdo_sparse(s, q_layers[i], K_layers[i], V_layers[i], rho, k, out_layers[i]);
            break;
        default:
            return TDO_BAD_ARG;
        }
        if (e) return e;
    }
    return TDO_OK;
}

/*
 * Paged KV cache.  Serving systems keep the cache C of Alg. 1 in fixed-size
 * pages handed out by an allocator (the paper's full-attention baseline and
 * the page-level method it compares with both work on such a cache; Sec. 2
 * and Sec. 4.3).  Paging changes where a token is stored, not what is
 * computed: logical token j of sequence b lives in page
 * block_table[b][j / page_size] at slot j % page_size.  This function writes
 * out the logical cache, [B][Hkv][max_seq_len][d] contiguous, so that the
 * functions above define every paged result.  Element (page, head, slot, c)
 * of the pool is at page*stride_page + head*stride_head + slot*stride_slot + c
 * (elements of elem_bytes bytes).  Rows j >= seq_lens[b] of `logical` are
 * left as they are.  A page id outside [0, num_pages) is an error.
 */
int tdo_gather_pages(int32_t batch, int32_t num_kv_heads, int32_t head_dim, int32_t elem_bytes,
                     const int32_t *seq_lens, int32_t max_seq_len, int32_t page_size,
                     int32_t num_pages, const int32_t *block_table, int64_t block_table_stride,
                     int64_t stride_page, int64_t stride_head, int64_t stride_slot,
                     const void *pool, void *logical) {
    if (batch < 1 || num_kv_heads < 1 || head_dim < 1 || (elem_bytes != 2 && elem_bytes != 4) ||
        !seq_lens || max_seq_len < 1 || page_size < 1 || num_pages < 1 || !block_table || !pool ||
        !logical)
        return TDO_BAD_ARG;
    const size_t row = (size_t)head_dim * (size_t)elem_bytes;
    for (int b = 0; b < batch; ++b) {
        if (seq_lens[b] < 0 || seq_lens[b] > max_seq_len) return TDO_BAD_ARG;
        for (int j = 0; j < seq_lens[b]; ++j) {
            const int32_t page = block_table[b * block_table_stride + j / page_size];
            const int slot = j % page_size;
            if (page < 0 || page >= num_pages) return TDO_BAD_ARG;
            for (int g = 0; g < num_kv_heads; ++g) {
                const int64_t src = page * stride_page + g * stride_head + slot * stride_slot;
                const int64_t dst = (((int64_t)b * num_kv_heads + g) * max_seq_len + j) * head_dim;
                memcpy((char *)logical + dst * elem_bytes, (const char *)pool + src * elem_bytes, row);
            }
        }
    }
    return TDO_OK;
}

/*
 * C.append(k, v) of Alg. 1: every layer appends the current token's key and
 * value to its cache before it attends.  seq_lens already counts the current
 * token, so the new row is row seq_lens[b] - 1 of sequence b.  k_new, v_new:
 * [B][Hkv][d] in the cache dtype (the key arrives with its rotary embedding
 * applied; that belongs to the projection f(W, x) of Alg. 1, not to this
 * path).  K, V are written in place; attention afterwards is the functions above.
 */
int tdo_append(const tdo_shape *s, void *K, void *V, const void *k_new, const void *v_new) {
    if (!shape_ok(s) || !K || !V || !k_new || !v_new) return TDO_BAD_ARG;
    const size_t eb = s->dtype == TDO_F32 ? 4 : 2;
    const size_t row = (size_t)s->head_dim * eb;
    for (int b = 0; b < s->batch; ++b)
        for (int g = 0; g < s->num_kv_heads; ++g) {
            const int64_t dst = b * s->kv_stride_batch + g * s->kv_stride_head +
                                (int64_t)(s->seq_lens[b] - 1) * s->kv_stride_tok;
            const int64_t src = ((int64_t)b * s->num_kv_heads + g) * s->head_dim;
            memcpy((char *)K + dst * eb, (const char *)k_new + src * eb, row);
            memcpy((char *)V + dst * eb, (const char *)v_new + src * eb, row);
        }
    return TDO_OK;
}

/*
 * Attention of the cache-correction step (Sec. 3.2): a prefill over the last P tokens of every
 * sequence, whose keys and values are already in the cache.  Token j (0 <= j < P) of sequence b
 * sits at position N_b - P + j and attends, with full attention (Eq. 1), to the positions up to
 * and including its own - the usual causal rule of a prefill.  q, out: [B][P][Hq][d].
 * Requires P <= N_b for every sequence.
 */
int tdo_prefill(const tdo_shape *s, int32_t num_new, const void *q, const void *K, const void *V, float *out) {
    if (!shape_ok(s) || !q || !K || !V || !out || num_new < 1) return TDO_BAD_ARG;
    for (int b = 0; b < s->batch; ++b)
        if (s->seq_lens[b] < num_new) return TDO_BAD_ARG;
    const int G = s->num_q_heads / s->num_kv_heads, d = s->head_dim;
    const float scale = scale_of(s);
    int err = TDO_OK;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < s->batch; ++b)
        for (int x = 0; x < num_new * s->num_q_heads; ++x) {
            const int j = x / s->num_q_heads, h = x % s->num_q_heads, g = h / G;
            const int visible = s->seq_lens[b] - num_new + j + 1;
            float *work = (float *)malloc((size_t)visible * sizeof(float));
            if (!work) { err = TDO_NO_MEM; continue; }
            const int64_t qo = (((int64_t)b * num_new + j) * s->num_q_heads + h) * d;
            const int64_t kvo = b * s->kv_stride_batch + g * s->kv_stride_head;
            attend_one(q, qo, K, V, kvo, s->kv_stride_tok, d, s->dtype, scale, NULL, visible, out + qo, NULL, work);
            free(work);
        }
    return err;
}

int tdo_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
