// Host side of the C ABI declared in tidal.h: argument checks, workspace layout, launch
// planning and the layer loop of Alg. 1.
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "common.h"

using namespace tidal;

struct td_ctx {
    int device = 0;
    char *workspace = nullptr;
    size_t workspace_bytes = 0;
    uint32_t *probe_sink = nullptr;  // one word of its own for td_probe_stream; never product state
    bool counters_dirty = false;     // a launch failed: the ticket counters are cleared before the next one
    int32_t target_workgroups = 0, min_chunk_dense = 0, min_chunk_sparse = 0, max_splits = 0, kernel_variant = 0;
    int32_t merge_mode = 0;          // 0: chosen per launch, 1: a second launch merges the partials, 2: the last chunk does
    bool attention_only = false;     // measurement: selection calls stop after their attention launch
    char error[256] = {0};
};

namespace {

constexpr int32_t kDefaultTargetWorkgroups = 1024;
constexpr int32_t kRaggedTargetWorkgroups = 8192;
constexpr int32_t kDefaultMinChunkDense = 128;
constexpr int32_t kDefaultMinChunkSparse = 128;
constexpr int32_t kChunkGranule = 128;
// chunks per (sequence, KV head): every chunk takes a ticket on one counter and the last one
// merges all partials alone, so the tail grows with the count
constexpr int32_t kDefaultMaxSplits = 64;
// a selection layer's attention launch bins its scores itself when a row has at most this many chunks
constexpr int32_t kFusedHistMaxSplits = 32;

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
int32_t ceil_div(int64_t a, int64_t b) { return (int32_t)((a + b - 1) / b); }

td_status fail(td_ctx *ctx, td_status s, const char *fmt, const char *detail = "") {
    if (ctx) snprintf(ctx->error, sizeof ctx->error, fmt, detail);
    return s;
}

// Rows of positions and scores per sequence: one per KV head, or per query head when every
// head selects for itself.
int32_t selection_rows(const td_shape *s) {
    return s->selection == TD_SELECT_PER_HEAD ? s->num_q_heads : s->num_kv_heads;
}

// Longest chunk of a paged full / selection launch: its pages' table entries fit the LDS stage
// (a chunk may start inside a page), rounded down to the chunk granule.
int64_t paged_chunk_limit(int32_t page_size) {
    const int64_t tokens = (int64_t)(kPageStageMax - 1) * page_size;
    return std::max<int64_t>(kChunkGranule, tokens / kChunkGranule * kChunkGranule);
}

// Why a shape or budget is unusable, or nullptr.  Host only.
const char *shape_problem(const td_shape *s, int32_t k, td_status *code) {
    *code = TD_ERR_INVALID_ARG;
    if (!s) return "shape is NULL";
    if (s->batch < 1) return "batch < 1";
    if (s->num_q_heads < 1 || s->num_kv_heads < 1) return "head count < 1";
    if (s->num_q_heads % s->num_kv_heads) return "num_q_heads is not a multiple of num_kv_heads";
    if (s->max_seq_len < 1) return "max_seq_len < 1";
    if (!s->seq_lens) return "seq_lens is NULL";
    if (s->dtype != TD_BF16 && s->dtype != TD_F32) return "dtype is neither TD_BF16 nor TD_F32";
    if (!(s->sm_scale >= 0.f)) return "sm_scale is negative or NaN";
    if (s->kv_stride_tok < s->head_dim || s->kv_stride_head < 1 || s->kv_stride_batch < 0)
        return "KV strides are too small for head_dim";
    if (s->kv_stride_tok % 8 || s->kv_stride_head % 8 || s->kv_stride_batch % 8)
        return "KV strides must be multiples of 8 elements";
    if (k > kSparseChunkMax * kSplitsMax) return "k is larger than 524288";
    if (s->total_seq_len < 0) return "total_seq_len is negative";
    if (s->selection < TD_SELECT_GROUP_SUM || s->selection > TD_SELECT_GROUP_MEAN_PROB) return "selection is not a td_selection";
    if (s->page_size < 0 || (s->page_size & (s->page_size - 1))) return "page_size is not a power of two";
    if (s->page_size > 0) {
        if (!s->block_table) return "block_table is NULL";
        if (s->num_pages < 1) return "num_pages < 1";
        if (s->block_table_stride < ((int64_t)s->max_seq_len + s->page_size - 1) / s->page_size)
            return "block_table_stride is smaller than the pages of max_seq_len tokens";
        if (s->kv_stride_batch < 1) return "page stride < 1";
    }
    *code = TD_ERR_UNSUPPORTED;
    if (s->head_dim != 64 && s->head_dim != 128) return "head_dim must be 64 or 128";
    if (s->max_seq_len > (1 << 30)) return "max_seq_len above 2^30";  // chunk arithmetic is done in 32 bits
    const int g = s->num_q_heads / s->num_kv_heads;
    if (g != 1 && g != 2 && g != 4 && g != 8) return "group size must be 1, 2, 4 or 8";
    if (s->batch > 65535 || s->num_kv_heads > 65535 || (int64_t)s->batch * selection_rows(s) > 65535)
        return "batch * num_kv_heads (num_q_heads with per-head selection) above 65535";
    // a selection chunk stages its scores in LDS; kSplitsMax chunks must cover the context
    if (k > 0 && (int64_t)s->max_seq_len > (int64_t)kSplitsMax * 4 * kScoreStagePerWave)
        return "max_seq_len is too long for a selection layer (above 1048576)";
    // a paged chunk stages its block-table entries in LDS; kSplitsMax chunks must cover the context
    if (s->page_size > 0 && (int64_t)s->max_seq_len > (int64_t)kSplitsMax * paged_chunk_limit(s->page_size))
        return "max_seq_len is too long for this page size";
    *code = TD_OK;
    return nullptr;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Workspace: [ticket counters | top-k state of up to kTopkFusedRows rows: fixed size, the same place for every
// shape][top-k state of larger launches][top-k scratch][chunk partials][group scores].
// Only the fixed part carries state from one call to the next: it is zero between launches, and because no
// launch of any shape writes anything else there, it stays so when calls with different shapes share a context.
struct Workspace {
    size_t counters, fused, topk_state, topk, part_acc, part_ml, scores, head_logits, ml_final, total;
    int64_t score_stride;
};

constexpr size_t kCountersBytes = (size_t)kCountersMax * sizeof(int32_t);
constexpr size_t kFusedBytes = (size_t)kTopkFusedRows * sizeof(TopkRow);
constexpr size_t kFixedBytes = kCountersBytes + kFusedBytes;
static_assert(kFixedBytes % 256 == 0, "what follows the fixed part stays aligned");

// Where the top-k state of a launch with `rows` rows lives and what follows it.
struct TopkPlace {
    size_t state, scratch;  // byte offsets in the workspace
    bool fixed;             // state inside the fixed part (zero between launches); else it is reset before use
};
TopkPlace topk_place(int32_t rows) {
    TopkPlace t;
    t.fixed = rows <= kTopkFusedRows;
    t.state = t.fixed ? kCountersBytes : kFixedBytes;
    t.scratch = t.fixed ? kFixedBytes : kFixedBytes + (size_t)rows * sizeof(TopkRow);
    t.scratch = (t.scratch + 255) / 256 * 256;
    return t;
}

// Zeroes the first n0 32-bit words of a and the first n1 of b.  A kernel rather than hipMemsetAsync so that
// the callers stay capturable into a HIP graph.
__global__ __launch_bounds__(256) void clear_words_kernel(uint32_t *a, size_t n0, uint32_t *b, size_t n1) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n0 + n1; i += (size_t)gridDim.x * 256) {
        if (i < n0) a[i] = 0u; else b[i - n0] = 0u;
    }
}

// Zeroes the state that launches expect to find at zero: the first `counters` ticket counters and the top-k
// state of the first `topk_rows` rows of the fixed part.
hipError_t clear_counters(char *workspace, size_t counters, size_t topk_rows, hipStream_t stream) {
    const size_t n1 = topk_rows * (sizeof(TopkRow) / 4);
    const int blocks = (int)std::min<size_t>(512, (counters + n1 + 255) / 256);
    hipLaunchKernelGGL(clear_words_kernel, dim3(blocks), dim3(256), 0, stream, reinterpret_cast<uint32_t *>(workspace),
                       counters, reinterpret_cast<uint32_t *>(workspace + kCountersBytes), n1);
    return hipGetLastError();
}

// splits: chunks per (sequence, KV head) that the partials have to hold; every decode call reserves kSplitsMax,
// so that the layout does not depend on the launch plan.
Workspace workspace_layout(const td_shape *s, int32_t k, int32_t splits = kSplitsMax) {
    Workspace w;
    const size_t heads = (size_t)s->batch * s->num_q_heads;
    const int32_t rows = s->batch * selection_rows(s);
    w.score_stride = (int64_t)align_up((size_t)s->max_seq_len, 4);
    w.counters = 0;
    w.fused = kCountersBytes;
    const TopkPlace tp = topk_place(rows);
    w.topk_state = tp.state;
    w.topk = k > 0 ? tp.scratch : kFixedBytes;
    w.part_acc = align_up(w.topk + (k > 0 ? topk_scratch_bytes(rows, s->max_seq_len, k) : 0), 256);
    w.part_ml = align_up(w.part_acc + heads * splits * s->head_dim * sizeof(float), 256);
    w.scores = align_up(w.part_ml + heads * splits * 2 * sizeof(float), 256);
    const size_t score_bytes = k > 0 ? (size_t)rows * w.score_stride * sizeof(float) : 0;
    // the mean-of-probabilities rule also keeps every head's logits and final softmax statistics
    const bool two_pass = k > 0 && s->selection == TD_SELECT_GROUP_MEAN_PROB;
    w.head_logits = align_up(w.scores + score_bytes, 256);
    w.ml_final = align_up(w.head_logits + (two_pass ? heads * w.score_stride * sizeof(float) : 0), 256);
    w.total = align_up(w.ml_final + (two_pass ? heads * 2 * sizeof(float) : 0), 256);
    return w;
}

// Known from the host's hint only: the sequences fill less than 90 % of batch * max_seq_len.
bool ragged_batch(const td_shape *s) {
    const int64_t dense_tokens = (int64_t)s->batch * s->max_seq_len;
    return s->total_seq_len > 0 && s->total_seq_len * 10 < dense_tokens * 9;
}

void plan_chunks(const td_ctx *ctx, const td_shape *s, int mode, int32_t waves, int32_t tokens,
                 int32_t *chunk, int32_t *splits) {
    const bool sparse = mode == kSparse;
    // sparse launches are latency-bound: fewer, fatter workgroups shorten the ticket and merge tail
    const td_ctx defaults;
    if (!ctx) ctx = &defaults;
    int32_t target = (ctx->target_workgroups > 0 ? ctx->target_workgroups : kDefaultTargetWorkgroups) / (sparse ? 2 : 1);
    // a ragged batch leaves many chunks of the grid empty and the rest unevenly spread over
    // the CUs: smaller chunks balance it
    if (!sparse && ctx->target_workgroups == 0 && ragged_batch(s)) target = kRaggedTargetWorkgroups;
    int32_t floor_chunk = sparse ? (ctx->min_chunk_sparse > 0 ? ctx->min_chunk_sparse : kDefaultMinChunkSparse)
                                 : (ctx->min_chunk_dense > 0 ? ctx->min_chunk_dense : kDefaultMinChunkDense);
    const int64_t groups = (int64_t)s->batch * (sparse ? selection_rows(s) : s->num_kv_heads);
    int32_t cap = std::min(kSplitsMax, ctx->max_splits > 0 ? ctx->max_splits : kDefaultMaxSplits);
    if (waves == 8) {  // the same number of waves in half as many workgroups, with chunks twice as long
        target = std::max(1, target / 2);
        cap = std::max(1, cap / 2);
        if (!sparse) floor_chunk *= 2;
    }
    const int32_t want = (int32_t)std::min<int64_t>(cap, std::max<int64_t>(1, target / groups));
    int32_t c = std::max(ceil_div(tokens, want), floor_chunk);
    c = std::max(c, ceil_div(tokens, cap));
    c = (int32_t)align_up((size_t)c, kChunkGranule);
    // Many chunks per workgroup slot (a ragged batch): chunks whose length is a power of two start
    // at addresses that are the same modulo a few hundred KiB, and the workgroups that run side by
    // side then press on the same memory channels (measured on a 16-sequence batch of 8K-64K tokens:
    // full layer 490 us with chunks of 1024 tokens, 469 with 512, 420-430 with 896, 1152, 1280, 1536 or 1792).
    // An odd number of 128-token granules keeps the starts apart.
    if (!sparse && ragged_batch(s) && (c / kChunkGranule) % 2 == 0) c += kChunkGranule;
    if (sparse) c = std::min(c, kSparseChunkMax);
    if (!sparse && s->page_size > 0) c = (int32_t)std::min<int64_t>(c, paged_chunk_limit(s->page_size));
    if (mode == kSelect) c = std::min(c, waves * kScoreStagePerWave);  // the chunk's scores are staged in LDS
    *chunk = c;
    *splits = ceil_div(tokens, c);
}

// What one attention launch will look like: decided on the host from the shape alone.
struct LaunchPlan {
    int32_t chunk, splits;       // tokens per workgroup, workgroups per grid row
    int32_t waves;               // wave64s per workgroup
    int32_t group;               // query heads served by a grid row
    int32_t grid_rows_per_seq;   // KV heads, or query heads when a sparse layer follows the per-head rule
    bool matrix_core;
    bool separate_merge;         // the chunk partials are folded by a second launch instead of the last chunk
};

LaunchPlan plan_launch(const td_ctx *ctx, const td_shape *s, int mode, int32_t k) {
    LaunchPlan plan;
    plan.group = s->num_q_heads / s->num_kv_heads;
    plan.grid_rows_per_seq = s->num_kv_heads;
    if (mode == kSparse && s->selection == TD_SELECT_PER_HEAD) {
        plan.grid_rows_per_seq = s->num_q_heads;
        plan.group = 1;
    }
    // The matrix-core kernel (bf16, head_dim 128) serves up to 16 query heads from one K/V tile
    // for the same instruction count.  Measured per launch against the vector-ALU kernel: groups
    // of eight 28.6 vs 43.3 us (full) and 11.2 vs 15.1 us (sparse); groups of four 26.6 vs 28.0 us
    // and 9.5 vs 10.0 us at 32K tokens, 328 vs 351 us at 4 x 128K; a single head per KV head
    // 319-327 vs 334 us for a full layer, but 20.0 vs 18.6 us for a sparse one, where most of the
    // 16-row tile is empty.  Hence: every layer kind for groups of four and more, full layers
    // only for smaller groups.
    const bool mfma_ok = s->dtype == TD_BF16 && s->head_dim == 128;
    const int32_t kv = ctx ? ctx->kernel_variant : 0;  // the low three bits of td_set_tuning's kernel_variant
    plan.matrix_core = mfma_ok && (kv == 1 || kv == 4 || kv == 5 || (kv == 0 && (plan.group >= 4 || mode == kDense)));
    // Workgroup size.  Full and selection layers use eight waves (half as many partials to merge
    // across workgroups; measured 3 to 9 % faster per launch on the uniform workloads) unless the
    // batch is ragged, where many small chunks balance better; sparse layers are one short burst
    // per wave and finish sooner with four.
    // (On the matrix-core kernel a sparse layer of eight-head groups does better with eight waves of
    // one tile each: its merge moves twice the partials, and 512 threads fetch them faster: 10.9 vs
    // 11.5 us; groups of four lose, 9.9 vs 9.6 us.)
    plan.waves = mode != kSparse && !ragged_batch(s) ? 8 : 4;
    if (mode == kSparse && plan.matrix_core && plan.group == 8) plan.waves = 8;
    // Larger gathers also do better with eight waves (half as many partials, one tile per wave and iteration):
    // measured four / eight waves, us per sparse layer - 32 rows: k 1024 10.5 / 11.0, k 2048 14.9 / 13.5,
    // k 4096 20.5 / 19.1, k 16384 54.2 / 51.8; 8 rows: k 2048 9.8 / 10.1, k 4096 12.9 / 12.2, k 8192 20.0 / 14.5;
    // 128 ragged rows, k 2048: 30.4 / 29.7; 32 rows of one head each (vector-ALU kernel), k 4096: 18.1 / 17.75.
    if (mode == kSparse && (k >= 4096 || (int64_t)s->batch * plan.grid_rows_per_seq * k >= 65536)) plan.waves = 8;
    if (kv == 2 || kv == 4) plan.waves = 4;
    if (kv == 3 || kv == 5) plan.waves = 8;
    if (!attend_supports_waves(plan.group, plan.waves)) plan.waves = 4;
    plan_chunks(ctx, s, mode, plan.waves, mode == kSparse ? k : s->max_seq_len, &plan.chunk, &plan.splits);
    const int32_t merge_mode = ctx ? ctx->merge_mode : 0;
    // The last chunk of a (sequence, KV head) folds the partials inside the launch - except on a ragged
    // batch: there a workgroup slot serves several chunks one after the other, and the publish-and-ticket
    // trips at the end of each of them, slow while the memory system is saturated, keep the slot from
    // streaming (same batch as above: full layer 519 us, 490 with the fold in a launch of its own).
    plan.separate_merge = plan.splits > 1 && (merge_mode == 1 || (merge_mode == 0 && mode != kSparse && ragged_batch(s)));
    return plan;
}

// Rows of a prefill served by the decode kernel (AttendParams): s->batch is then the number of row blocks.
struct PrefillRows {
    int32_t new_per_seq, new_first, num_new, cache_first;
};

td_status attend(td_ctx *ctx, const td_shape *s, int mode, const void *q, const void *K, const void *V,
                 const int32_t *positions, int32_t k, float *scores, int64_t score_stride, void *out,
                 hipStream_t stream, const void *k_new = nullptr, const void *v_new = nullptr,
                 int32_t score_rule = -1, float *ml_out = nullptr, TopkRow *fused_rows = nullptr,
                 const PrefillRows *prefill = nullptr) {
    const LaunchPlan plan = plan_launch(ctx, s, mode, k);
    // a prefill through this kernel may have many more rows than a decode step: its partials take what the plan needs
    const Workspace w = workspace_layout(s, mode == kDense ? 0 : k, prefill ? plan.splits : kSplitsMax);
    AttendParams p;
    memset(&p, 0, sizeof p);
    if (prefill) {
        p.new_per_seq = prefill->new_per_seq;
        p.new_first = prefill->new_first;
        p.num_new = prefill->num_new;
        p.cache_first = prefill->cache_first;
    }
    p.q = q; p.K = K; p.V = V; p.out = out;
    p.k_new = k_new; p.v_new = v_new;
    p.seq_lens = s->seq_lens;
    p.positions = positions;
    p.scores = scores;
    p.score_stride = score_stride;
    p.part_acc = reinterpret_cast<float *>(ctx->workspace + w.part_acc);
    p.part_ml = reinterpret_cast<float *>(ctx->workspace + w.part_ml);
    p.counters = reinterpret_cast<int32_t *>(ctx->workspace + w.counters);
    p.topk_rows = fused_rows;
    p.stride_batch = s->kv_stride_batch;
    if (s->page_size > 0) {
        p.block_table = s->block_table;
        p.bt_stride = s->block_table_stride;
        p.num_pages = s->num_pages;
        while ((1 << p.page_shift) < s->page_size) ++p.page_shift;
    }
    p.stride_head = s->kv_stride_head;
    p.stride_tok = s->kv_stride_tok;
    p.batch = s->batch;
    p.num_q_heads = s->num_q_heads;
    p.num_kv_heads = s->num_kv_heads;
    p.select_rule = score_rule >= 0 ? score_rule : s->selection;  // what the selection mode writes to `scores`
    p.ml_out = ml_out;
    p.kv_div = 1;
    p.max_seq_len = s->max_seq_len;
    p.k = k;
    p.scale = s->sm_scale > 0.f ? s->sm_scale : 1.0f / sqrtf((float)s->head_dim);
    if (plan.grid_rows_per_seq != s->num_kv_heads) {
        // one grid row per query head, each gathering its own rho from KV head (row / group)
        p.kv_div = s->num_q_heads / s->num_kv_heads;
        p.num_kv_heads = s->num_q_heads;
    }
    p.chunk = plan.chunk;
    p.num_splits = plan.splits;
    p.separate_merge = plan.separate_merge ? 1 : 0;
    const int group = plan.group, waves = plan.waves;
    const bool mfma = plan.matrix_core && !prefill;  // only the vector-ALU kernel knows prefill rows
    if (ctx->counters_dirty) {  // an earlier launch on this context failed: start from zeroed tickets
        const hipError_t ce = clear_counters(ctx->workspace, kCountersMax, kTopkFusedRows, stream);
        if (ce != hipSuccess) return fail(ctx, TD_ERR_HIP, "clearing the ticket counters failed: %s", hipGetErrorString(ce));
        ctx->counters_dirty = false;
    }
    const hipError_t e = mfma ? launch_attend_mfma(group, waves, mode, p, stream)
                              : launch_attend(s->dtype, s->head_dim, group, waves, mode, p, stream);
    if (e != hipSuccess) {
        ctx->counters_dirty = true;
        return fail(ctx, TD_ERR_HIP, "attention launch failed: %s", hipGetErrorString(e));
    }
    if (plan.separate_merge) {
        const hipError_t me = launch_merge(s->dtype, s->head_dim, mode, p, stream);
        if (me != hipSuccess) return fail(ctx, TD_ERR_HIP, "merge launch failed: %s", hipGetErrorString(me));
    }
    return TD_OK;
}

// Checks common to every attention call; `k` <= 0 when the call has no budget.
td_status check_call(td_ctx *ctx, const td_shape *s, int32_t k, bool needs_k, const void *q, const void *K,
                     const void *V, const void *out, bool needs_workspace = true) {
    if (!ctx) return TD_ERR_INVALID_ARG;
    td_status code;
    if (const char *why = shape_problem(s, k, &code)) return fail(ctx, code, "%s", why);
    if (needs_k && k < 1) return fail(ctx, TD_ERR_INVALID_ARG, "%s", "k < 1");
    if (!q || !K || !V || !out) return fail(ctx, TD_ERR_INVALID_ARG, "%s", "q, K, V or out is NULL");
    if (misaligned(q) || misaligned(K) || misaligned(V) || misaligned(out))
        return fail(ctx, TD_ERR_INVALID_ARG, "%s", "q, K, V and out must be 16-byte aligned");
    if (needs_workspace && workspace_layout(s, needs_k ? k : 0).total > ctx->workspace_bytes)
        return fail(ctx, TD_ERR_WORKSPACE, "%s", "workspace is smaller than td_workspace_bytes(shape, k)");
    return TD_OK;
}

td_status select_tokens(td_ctx *ctx, const td_shape *s, const void *q, const void *K, const void *V,
                        int32_t k, void *out, int32_t *positions, float *group_scores, hipStream_t stream,
                        const void *k_new = nullptr, const void *v_new = nullptr) {
    const Workspace w = workspace_layout(s, k);
    float *scores = group_scores ? group_scores : reinterpret_cast<float *>(ctx->workspace + w.scores);
    const int64_t stride = group_scores ? (int64_t)s->max_seq_len : w.score_stride;
    int64_t stride_for_topk = stride;
    td_status st;
    if (s->selection == TD_SELECT_GROUP_MEAN_PROB) {
        // pass 1 writes every head's logits and final (max, sum); pass 2 forms the group's mean probability
        float *logits = reinterpret_cast<float *>(ctx->workspace + w.head_logits);
        float *ml = reinterpret_cast<float *>(ctx->workspace + w.ml_final);
        st = attend(ctx, s, kSelect, q, K, V, nullptr, k, logits, w.score_stride, out, stream, k_new, v_new,
                    TD_SELECT_PER_HEAD, ml);
        if (st != TD_OK) return st;
        // top-k ranks log2 of the probabilities, kept in the workspace; the caller's buffer gets the probabilities
        float *rank = reinterpret_cast<float *>(ctx->workspace + w.scores);
        const hipError_t pe = launch_mean_prob(logits, w.score_stride, ml, s->seq_lens, s->batch, s->num_kv_heads,
                                               s->num_q_heads / s->num_kv_heads, s->max_seq_len, rank, w.score_stride,
                                               group_scores, s->max_seq_len, stream);
        if (pe != hipSuccess) return fail(ctx, TD_ERR_HIP, "mean-probability launch failed: %s", hipGetErrorString(pe));
        scores = rank;
        stride_for_topk = w.score_stride;
    }
    // The group rules leave one score row per KV head, staged in LDS by the attention launch, which then also
    // bins them for the top-k launch; that needs top-k state at a place that is zero between launches, the
    // fixed part of the workspace.
    const int32_t rows = selection_rows(s), all_rows = s->batch * rows;
    const TopkPlace tp = topk_place(all_rows);
    TopkRow *state = reinterpret_cast<TopkRow *>(ctx->workspace + tp.state);
    // (With many short chunks per row - a ragged batch - the chunks' histogram updates trickle into memory
    // between the streaming reads all through the launch and cost more than the histogram launch they
    // replace: 553 vs 483 us for the attention launch of 16 ragged sequences with 63 chunks each.)
    const bool fused = tp.fixed && (s->selection == TD_SELECT_GROUP_SUM || s->selection == TD_SELECT_GROUP_MAX) &&
                       plan_launch(ctx, s, kSelect, k).splits <= kFusedHistMaxSplits;
    if (s->selection != TD_SELECT_GROUP_MEAN_PROB) {
        st = attend(ctx, s, kSelect, q, K, V, nullptr, k, scores, stride, out, stream, k_new, v_new, -1, nullptr,
                    fused ? state : nullptr);
        if (st != TD_OK) return st;
    }
    if (ctx->attention_only) return TD_OK;  // timing of the attention launch alone; the row histograms stay as they are
    hipError_t e = hipSuccess;
    if (!tp.fixed) e = launch_topk_reset(state, all_rows, stream);
    if (e == hipSuccess)
        e = launch_topk(scores, stride_for_topk, all_rows, s->seq_lens, rows, s->max_seq_len, k, positions, state,
                        ctx->workspace + w.topk, fused, ragged_batch(s), stream);
    if (e != hipSuccess) {
        ctx->counters_dirty = true;
        return fail(ctx, TD_ERR_HIP, "top-k launch failed: %s", hipGetErrorString(e));
    }
    return TD_OK;
}

td_status decode_step(td_ctx *ctx, const td_shape *shape, int32_t num_layers, const int32_t *schedule,
                      const void *const *q_layers, const void *const *k_new_layers, const void *const *v_new_layers,
                      const void *const *K_layers, const void *const *V_layers, int32_t k, void *const *out_layers,
                      int32_t *positions, void *hip_stream) {
    if (!ctx) return TD_ERR_INVALID_ARG;
    if (num_layers < 1 || !schedule || !q_layers || !K_layers || !V_layers || !out_layers)
        return fail(ctx, TD_ERR_INVALID_ARG, "%s", "num_layers < 1 or a layer array is NULL");
    bool any_budget = false, selected = false;
    for (int i = 0; i < num_layers; ++i) {
        if (schedule[i] < TD_LAYER_DENSE || schedule[i] > TD_LAYER_SPARSE)
            return fail(ctx, TD_ERR_INVALID_ARG, "%s", "schedule entry is not a td_layer_kind");
        if (schedule[i] == TD_LAYER_SELECT) selected = true;
        if (schedule[i] == TD_LAYER_SPARSE && !selected)
            return fail(ctx, TD_ERR_INVALID_ARG, "%s", "sparse layer before any selection layer");
        if (schedule[i] != TD_LAYER_DENSE) any_budget = true;
    }
    if (any_budget && !positions) return fail(ctx, TD_ERR_INVALID_ARG, "%s", "positions is NULL");
    for (int i = 0; i < num_layers; ++i) {
        td_status st = check_call(ctx, shape, k, any_budget, q_layers[i], K_layers[i], V_layers[i], out_layers[i]);
        if (st != TD_OK) return st;
        if (k_new_layers && (!k_new_layers[i] || !v_new_layers[i] || misaligned(k_new_layers[i]) || misaligned(v_new_layers[i])))
            return fail(ctx, TD_ERR_INVALID_ARG, "%s", "k_new / v_new of a layer is NULL or not 16-byte aligned");
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t slot = (int64_t)shape->batch * selection_rows(shape) * k;
    const int32_t *rho = nullptr;
    int n_sel = 0;
    for (int i = 0; i < num_layers; ++i) {
        td_status st;
        const void *kn = k_new_layers ? k_new_layers[i] : nullptr, *vn = k_new_layers ? v_new_layers[i] : nullptr;
        if (schedule[i] == TD_LAYER_DENSE) {
            st = attend(ctx, shape, kDense, q_layers[i], K_layers[i], V_layers[i], nullptr, 0, nullptr, 0,
                        out_layers[i], stream, kn, vn);
        } else if (schedule[i] == TD_LAYER_SELECT) {
            int32_t *dst = positions + slot * n_sel++;
            st = select_tokens(ctx, shape, q_layers[i], K_layers[i], V_layers[i], k, out_layers[i], dst, nullptr, stream,
                               kn, vn);
            rho = dst;
        } else {
            st = attend(ctx, shape, kSparse, q_layers[i], K_layers[i], V_layers[i], rho, k, nullptr, 0,
                        out_layers[i], stream, kn, vn);
        }
        if (st != TD_OK) return st;
    }
    return TD_OK;
}

}  // namespace

extern "C" {

td_status td_validate(const td_shape *shape, int32_t k) {
    td_status code;
    shape_problem(shape, k, &code);
    return code;
}

size_t td_workspace_bytes(const td_shape *shape, int32_t k) {
    td_status code;
    if (shape_problem(shape, k, &code)) return 0;
    return workspace_layout(shape, k).total;
}

size_t td_topk_workspace_bytes(int32_t rows, int32_t max_len) {
    if (rows < 1 || max_len < 1) return 0;
    return align_up(topk_place(rows).scratch + topk_scratch_bytes(rows, max_len, max_len), 256);
}

td_status td_create(td_ctx **out, int device, size_t workspace_bytes) {
    if (!out) return TD_ERR_INVALID_ARG;
    *out = nullptr;
    td_ctx *ctx = new (std::nothrow) td_ctx;
    if (!ctx) return TD_ERR_HIP;
    ctx->device = device;
    hipError_t e = hipSetDevice(device);
    if (e == hipSuccess && workspace_bytes) e = hipMalloc(reinterpret_cast<void **>(&ctx->workspace), workspace_bytes);
    if (e == hipSuccess && workspace_bytes) e = hipMemset(ctx->workspace, 0, workspace_bytes);  // chunk counters start at zero
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&ctx->probe_sink), 256);
    if (e == hipSuccess) e = hipMemset(ctx->probe_sink, 0, 256);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        if (ctx->workspace) (void)hipFree(ctx->workspace);
        if (ctx->probe_sink) (void)hipFree(ctx->probe_sink);
        delete ctx;
        return TD_ERR_HIP;
    }
    ctx->workspace_bytes = workspace_bytes;
    *out = ctx;
    (void)static_scratch_setup();  // set-up for td_decode_step_static on this device; that call repeats it on failure
    return TD_OK;
}

td_status td_destroy(td_ctx *ctx) {
    if (!ctx) return TD_ERR_INVALID_ARG;
    hipError_t e = hipSuccess;
    if (ctx->workspace) e = hipFree(ctx->workspace);
    if (ctx->probe_sink) {
        const hipError_t e2 = hipFree(ctx->probe_sink);
        if (e == hipSuccess) e = e2;
    }
    delete ctx;
    return e == hipSuccess ? TD_OK : TD_ERR_HIP;
}

td_status td_plan_launch(const td_ctx *ctx, const td_shape *shape, int32_t layer_kind, int32_t k, td_launch_plan *plan) {
    if (!plan || layer_kind < TD_LAYER_DENSE || layer_kind > TD_LAYER_SPARSE) return TD_ERR_INVALID_ARG;
    td_status code;
    if (shape_problem(shape, k, &code)) return code;
    if (layer_kind != TD_LAYER_DENSE && k < 1) return TD_ERR_INVALID_ARG;
    const LaunchPlan lp = plan_launch(ctx, shape, layer_kind, k);
    plan->chunk_tokens = lp.chunk;
    plan->chunks_per_row = lp.splits;
    plan->waves_per_workgroup = lp.waves;
    plan->matrix_core = lp.matrix_core ? 1 : 0;
    plan->merge_launch = lp.separate_merge ? 1 : 0;
    plan->grid_rows = shape->batch * lp.grid_rows_per_seq;
    plan->workgroups = (int64_t)plan->grid_rows * lp.splits;
    return TD_OK;
}

td_status td_set_tuning(td_ctx *ctx, int32_t target_workgroups, int32_t min_chunk_dense,
                        int32_t min_chunk_sparse, int32_t max_splits, int32_t kernel_variant) {
    if (!ctx) return TD_ERR_INVALID_ARG;
    if (target_workgroups < 0 || min_chunk_dense < 0 || min_chunk_sparse < 0 || max_splits < 0 ||
        kernel_variant < 0 || kernel_variant >= 64 || (kernel_variant & 7) > 5 || ((kernel_variant >> 3) & 3) > 2)
        return fail(ctx, TD_ERR_INVALID_ARG, "%s", "tuning values must be >= 0, kernel_variant one of those the header lists");
    ctx->target_workgroups = target_workgroups;
    ctx->min_chunk_dense = min_chunk_dense;
    ctx->min_chunk_sparse = min_chunk_sparse;
    ctx->max_splits = max_splits;
    ctx->kernel_variant = kernel_variant & 7;
    ctx->merge_mode = (kernel_variant >> 3) & 3;
    const bool attention_only = (kernel_variant & 32) != 0;
    // selection calls that stopped after their attention launch have left their score histograms in the
    // rows' state: it is cleared before the next launch, whichever way the switch goes
    if (attention_only || ctx->attention_only) ctx->counters_dirty = true;
    ctx->attention_only = attention_only;
    return TD_OK;
}

td_status td_full_attend(td_ctx *ctx, const td_shape *shape, const void *q, const void *K, const void *V,
                         void *out, void *hip_stream) {
    td_status st = check_call(ctx, shape, 0, false, q, K, V, out);
    if (st != TD_OK) return st;
    return attend(ctx, shape, kDense, q, K, V, nullptr, 0, nullptr, 0, out, static_cast<hipStream_t>(hip_stream));
}

td_status td_select_tokens(td_ctx *ctx, const td_shape *shape, const void *q, const void *K, const void *V,
                           int32_t k, void *out, int32_t *positions, float *group_scores, void *hip_stream) {
    td_status st = check_call(ctx, shape, k, true, q, K, V, out);
    if (st != TD_OK) return st;
    if (!positions) return fail(ctx, TD_ERR_INVALID_ARG, "%s", "positions is NULL");
    if (group_scores && misaligned(group_scores))
        return fail(ctx, TD_ERR_INVALID_ARG, "%s", "group_scores must be 16-byte aligned");
    return select_tokens(ctx, shape, q, K, V, k, out, positions, group_scores, static_cast<hipStream_t>(hip_stream));
}

namespace {
PrefillPlan prefill_plan_for(const td_shape *s, int32_t num_new, size_t avail) {
    const int64_t pairs = (int64_t)s->batch * s->num_kv_heads;
    // the maxima and denominators come first, rounded up to 256 bytes; the rest holds the numerators
    const size_t slack = 256;
    return plan_prefill((int64_t)num_new * (s->num_q_heads / s->num_kv_heads), pairs, s->max_seq_len,
                        avail > slack ? avail - slack : 0);
}
size_t prefill_ml_bytes(const PrefillPlan &pl, const td_shape *s) {
    const size_t slots = (size_t)pl.row_blocks * s->batch * s->num_kv_heads * pl.chunks * pl.rows_per_wg;
    return align_up(slots * 2 * sizeof(float), 256);
}

// The matrix-core prefill kernel takes bf16 with head_dim 128, contiguous or in pages of 16 tokens and more,
// with token strides its 32-bit lane offsets can express.
bool prefill_kernel_takes(const td_shape *s) {
    return s->dtype == TD_BF16 && s->head_dim == 128 && (s->page_size == 0 || s->page_size >= 16) &&
           s->kv_stride_tok <= (int64_t)1 << 24;
}

// Every other shape goes through the vector-ALU decode kernel in full mode: one row block of the grid per new
// token, each attending to the positions up to its own (AttendParams::new_per_seq).  The cache is then read
// once per new token - it is the plain path, for shapes outside the matrix-core kernel's reach.
// A launch takes as many row blocks as the grid, the ticket counters and the workspace allow: all
// batch * num_new at once if they fit, else runs of new tokens of one sequence at a time.
struct PlainPrefill {
    int32_t rows;        // row blocks per launch
    bool whole;          // one launch covers every sequence
    size_t workspace;    // bytes such a launch needs
};
size_t plain_prefill_bytes(const td_ctx *ctx, const td_shape *s, int32_t rows) {
    td_shape rs = *s;
    rs.batch = rows;
    rs.total_seq_len = 0;
    return workspace_layout(&rs, 0, plan_launch(ctx, &rs, kDense, 0).splits).total;
}
PlainPrefill plan_plain_prefill(const td_ctx *ctx, const td_shape *s, int32_t num_new, size_t avail) {
    const int64_t most = std::min<int64_t>(65535, kCountersMax / s->num_kv_heads);  // grid.z, one ticket counter per (row block, KV head)
    PlainPrefill pp;
    const int64_t all = (int64_t)s->batch * num_new;
    if (all <= most && plain_prefill_bytes(ctx, s, (int32_t)all) <= avail) {
        pp.rows = (int32_t)all;
        pp.whole = true;
        pp.workspace = plain_prefill_bytes(ctx, s, pp.rows);
        return pp;
    }
    pp.whole = false;
    pp.rows = (int32_t)std::min<int64_t>(num_new, most);
    while (pp.rows > 1 && plain_prefill_bytes(ctx, s, pp.rows) > avail) pp.rows = (pp.rows + 1) / 2;
    pp.workspace = plain_prefill_bytes(ctx, s, pp.rows);
    return pp;
}

td_status plain_prefill(td_ctx *ctx, const td_shape *s, int32_t num_new, const void *q, const void *K, const void *V,
                        void *out, hipStream_t stream) {
    const PlainPrefill pp = plan_plain_prefill(ctx, s, num_new, ctx->workspace_bytes);
    if (pp.workspace > ctx->workspace_bytes)
        return fail(ctx, TD_ERR_WORKSPACE, "%s", "workspace is smaller than td_workspace_bytes(shape, 0): not even one new token fits");
    td_shape rs = *s;
    rs.batch = pp.rows;
    rs.total_seq_len = 0;
    PrefillRows pr;
    pr.num_new = num_new;
    if (pp.whole) {
        pr.new_per_seq = num_new;
        pr.new_first = 0;
        pr.cache_first = 0;
        return attend(ctx, &rs, kDense, q, K, V, nullptr, 0, nullptr, 0, out, stream, nullptr, nullptr, -1, nullptr, nullptr, &pr);
    }
    const size_t row_bytes = (size_t)s->num_q_heads * s->head_dim * (s->dtype == TD_BF16 ? 2 : 4);
    for (int32_t b = 0; b < s->batch; ++b) {
        for (int32_t first = 0; first < num_new; first += pp.rows) {
            rs.batch = std::min(pp.rows, num_new - first);
            pr.new_per_seq = rs.batch;
            pr.new_first = first;
            pr.cache_first = b;
            const size_t at = ((size_t)b * num_new + first) * row_bytes;
            const td_status st = attend(ctx, &rs, kDense, static_cast<const char *>(q) + at, K, V, nullptr, 0, nullptr, 0,
                                        static_cast<char *>(out) + at, stream, nullptr, nullptr, -1, nullptr, nullptr, &pr);
            if (st != TD_OK) return st;
        }
    }
    return TD_OK;
}
}  // namespace

size_t td_prefill_workspace_bytes(const td_shape *shape, int32_t num_new) {
    td_status code;
    if (shape_problem(shape, 0, &code) || num_new < 1 || num_new > shape->max_seq_len) return 0;
    if (!prefill_kernel_takes(shape)) return plan_plain_prefill(nullptr, shape, num_new, ~(size_t)0).workspace;
    const PrefillPlan pl = prefill_plan_for(shape, num_new, ~(size_t)0);
    return pl.chunks > 1 ? align_up(kFixedBytes + 256 + pl.part_bytes, 256) : 0;
}

td_status td_prefill_attend(td_ctx *ctx, const td_shape *shape, int32_t num_new, const void *q, const void *K,
                            const void *V, void *out, void *hip_stream) {
    td_status st = check_call(ctx, shape, 0, false, q, K, V, out, false);
    if (st != TD_OK) return st;
    if (num_new < 1 || num_new > shape->max_seq_len)
        return fail(ctx, TD_ERR_INVALID_ARG, "%s", "num_new outside [1, max_seq_len]");
    if (!prefill_kernel_takes(shape)) return plain_prefill(ctx, shape, num_new, q, K, V, out, static_cast<hipStream_t>(hip_stream));
    PrefillParams p;
    memset(&p, 0, sizeof p);
    p.q = q; p.K = K; p.V = V; p.out = out;
    p.seq_lens = shape->seq_lens;
    p.stride_batch = shape->kv_stride_batch;
    p.stride_head = shape->kv_stride_head;
    p.stride_tok = shape->kv_stride_tok;
    p.batch = shape->batch;
    p.num_q_heads = shape->num_q_heads;
    p.num_kv_heads = shape->num_kv_heads;
    p.max_seq_len = shape->max_seq_len;
    p.num_new = num_new;
    p.scale = shape->sm_scale > 0.f ? shape->sm_scale : 1.0f / sqrtf((float)shape->head_dim);
    if (shape->page_size > 0) {
        p.block_table = shape->block_table;
        p.bt_stride = shape->block_table_stride;
        p.num_pages = shape->num_pages;
        while ((1 << p.page_shift) < shape->page_size) ++p.page_shift;
    }
    // token chunks as far as the workspace holds their partial states
    const size_t avail = ctx->workspace_bytes > kFixedBytes ? ctx->workspace_bytes - kFixedBytes : 0;
    const PrefillPlan pl = prefill_plan_for(shape, num_new, avail);
    p.rows_per_wg = pl.rows_per_wg;
    p.row_blocks = pl.row_blocks;
    p.chunk = pl.chunk;
    p.chunks = pl.chunks;
    if (pl.chunks > 1) {
        p.part_ml = reinterpret_cast<float *>(ctx->workspace + kFixedBytes);
        p.part_acc = reinterpret_cast<float *>(ctx->workspace + kFixedBytes + prefill_ml_bytes(pl, shape));
    }
    const hipError_t e = launch_prefill(shape->num_q_heads / shape->num_kv_heads, p, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(ctx, TD_ERR_HIP, "prefill launch failed: %s", hipGetErrorString(e));
    return TD_OK;
}

td_status td_sparse_attend(td_ctx *ctx, const td_shape *shape, const void *q, const void *K, const void *V,
                           const int32_t *positions, int32_t k, void *out, void *hip_stream) {
    td_status st = check_call(ctx, shape, k, true, q, K, V, out);
    if (st != TD_OK) return st;
    if (!positions) return fail(ctx, TD_ERR_INVALID_ARG, "%s", "positions is NULL");
    return attend(ctx, shape, kSparse, q, K, V, positions, k, nullptr, 0, out, static_cast<hipStream_t>(hip_stream));
}

td_status td_topk(td_ctx *ctx, const float *scores, int64_t row_stride, int32_t rows, const int32_t *row_lens,
                  int32_t rows_per_len, int32_t max_len, int32_t k, int32_t *positions, void *hip_stream) {
    if (!ctx) return TD_ERR_INVALID_ARG;
    if (!scores || !row_lens || !positions) return fail(ctx, TD_ERR_INVALID_ARG, "%s", "scores, row_lens or positions is NULL");
    if (rows < 1 || rows_per_len < 1 || max_len < 1 || k < 1 || row_stride < max_len)
        return fail(ctx, TD_ERR_INVALID_ARG, "%s", "rows, rows_per_len, max_len, k must be >= 1 and row_stride >= max_len");
    if (misaligned(scores)) return fail(ctx, TD_ERR_INVALID_ARG, "%s", "scores must be 16-byte aligned");
    if (rows > 65535) return fail(ctx, TD_ERR_UNSUPPORTED, "%s", "more than 65535 rows");
    const TopkPlace tp = topk_place(rows);
    if (tp.scratch + topk_scratch_bytes(rows, max_len, k) > ctx->workspace_bytes)
        return fail(ctx, TD_ERR_WORKSPACE, "%s", "workspace is smaller than td_topk_workspace_bytes(rows, max_len)");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    TopkRow *state = reinterpret_cast<TopkRow *>(ctx->workspace + tp.state);
    hipError_t e = hipSuccess;
    if (ctx->counters_dirty) {
        e = clear_counters(ctx->workspace, kCountersMax, kTopkFusedRows, stream);
        if (e == hipSuccess) ctx->counters_dirty = false;
    }
    if (e == hipSuccess && !tp.fixed) e = launch_topk_reset(state, rows, stream);
    if (e == hipSuccess)
        e = launch_topk(scores, row_stride, rows, row_lens, rows_per_len, max_len, k, positions, state,
                        ctx->workspace + tp.scratch, false, false, stream);
    if (e != hipSuccess) {
        ctx->counters_dirty = true;
        return fail(ctx, TD_ERR_HIP, "top-k launch failed: %s", hipGetErrorString(e));
    }
    return TD_OK;
}

td_status td_decode_step(td_ctx *ctx, const td_shape *shape, int32_t num_layers, const int32_t *schedule,
                         const void *const *q_layers, const void *const *K_layers, const void *const *V_layers,
                         int32_t k, void *const *out_layers, int32_t *positions, void *hip_stream) {
    return decode_step(ctx, shape, num_layers, schedule, q_layers, nullptr, nullptr, K_layers, V_layers, k, out_layers,
                       positions, hip_stream);
}

td_status td_decode_step_append(td_ctx *ctx, const td_shape *shape, int32_t num_layers, const int32_t *schedule,
                                const void *const *q_layers, const void *const *k_new_layers,
                                const void *const *v_new_layers, void *const *K_layers, void *const *V_layers,
                                int32_t k, void *const *out_layers, int32_t *positions, void *hip_stream) {
    if (!ctx) return TD_ERR_INVALID_ARG;
    if (!k_new_layers || !v_new_layers) return fail(ctx, TD_ERR_INVALID_ARG, "%s", "k_new_layers or v_new_layers is NULL");
    return decode_step(ctx, shape, num_layers, schedule, q_layers, k_new_layers, v_new_layers,
                       const_cast<const void *const *>(K_layers), const_cast<const void *const *>(V_layers), k,
                       out_layers, positions, hip_stream);
}

td_status td_probe_stream(td_ctx *ctx, void *dst, const void *src, size_t bytes, void *hip_stream) {
    if (!ctx) return TD_ERR_INVALID_ARG;
    if (!src || bytes < 16 || misaligned(src) || (dst && misaligned(dst)))
        return fail(ctx, TD_ERR_INVALID_ARG, "%s", "src (and dst) must be 16-byte aligned and bytes >= 16");
    const hipError_t e = launch_probe(dst, src, bytes, ctx->probe_sink, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(ctx, TD_ERR_HIP, "probe launch failed: %s", hipGetErrorString(e));
    return TD_OK;
}

const char *td_status_string(td_status s) {
    switch (s) {
    case TD_OK: return "ok";
    case TD_ERR_INVALID_ARG: return "invalid argument";
    case TD_ERR_UNSUPPORTED: return "unsupported shape";
    case TD_ERR_WORKSPACE: return "workspace too small";
    case TD_ERR_HIP: return "HIP error";
    }
    return "unknown status";
}

const char *td_last_error(const td_ctx *ctx) { return ctx ? ctx->error : static_last_error(); }

}  // extern "C"

// The layer loop on a workspace that the caller names, with the default launch plan.  The ticket
// counters that this shape uses are zeroed first (the workspace may hold anything); `error`
// receives the text of a failure.
td_status tidal::decode_step_on_workspace(char *workspace, size_t workspace_bytes, const td_shape *shape,
                                          int32_t num_layers, const int32_t *schedule, const void *const *q_layers,
                                          const void *const *K_layers, const void *const *V_layers, int32_t k,
                                          void *const *out_layers, int32_t *positions, void *hip_stream,
                                          char (&error)[256]) {
    td_ctx local;
    local.workspace = workspace;
    local.workspace_bytes = workspace_bytes;
    td_status code;
    td_status st;
    if (const char *why = shape_problem(shape, k, &code)) {
        st = fail(&local, code, "%s", why);
    } else {
        const size_t rows = (size_t)shape->batch * std::max(shape->num_kv_heads, selection_rows(shape));
        const hipError_t e = workspace_layout(shape, k).total <= workspace_bytes
                                 ? clear_counters(workspace, rows, std::min<size_t>(rows, kTopkFusedRows),
                                                  static_cast<hipStream_t>(hip_stream))
                                 : hipSuccess;  // too small: decode_step says so before anything is enqueued
        st = e != hipSuccess ? fail(&local, TD_ERR_HIP, "clearing the ticket counters failed: %s", hipGetErrorString(e))
                             : decode_step(&local, shape, num_layers, schedule, q_layers, nullptr, nullptr, K_layers,
                                           V_layers, k, out_layers, positions, hip_stream);
    }
    memcpy(error, local.error, sizeof local.error);
    return st;
}

extern "C" {

td_status td_reset(td_ctx *ctx, void *hip_stream) {
    if (!ctx) return TD_ERR_INVALID_ARG;
    if (!ctx->workspace || ctx->workspace_bytes < kFixedBytes) {
        ctx->counters_dirty = false;  // no attention call fits this workspace, nothing to clear
        return TD_OK;
    }
    const hipError_t e = clear_counters(ctx->workspace, kCountersMax, kTopkFusedRows, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(ctx, TD_ERR_HIP, "clearing the ticket counters failed: %s", hipGetErrorString(e));
    ctx->counters_dirty = false;
    return TD_OK;
}

}  // extern "C"
