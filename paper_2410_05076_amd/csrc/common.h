// Internal declarations shared by the host API and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tidal.h"
#include "topk_math.h"

namespace tidal {

constexpr int kWave = 64;
constexpr int kSplitsMax = 256;        // upper bound on token chunks per (sequence, KV head)
// group scores of one chunk are staged in LDS (selection layers): tokens per wave of the workgroup
constexpr int kScoreStagePerWave = 1024;
constexpr int kPageStageMax = 1024;    // block-table entries of one chunk are staged in LDS
constexpr int kSparseChunkMax = 2048;  // positions of one chunk are staged in LDS
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kCountersMax = 65536;    // ticket counters, one per (sequence, KV head)
// Per-row state of the top-k kernels.  `hist` must be zero when a selection launch sequence starts
// and the last top-k launch leaves it at zero again (like the ticket counters).  A selection
// layer's attention launch adds its chunks' score histograms to it (fused mode); this is only
// possible for state at a place that no other shape's launch ever writes, so the fused rows live
// in a fixed region right after the ticket counters, kTopkFusedRows of them; launches with more
// rows reset their state and run the histogram as a kernel.
struct TopkRow {
    uint32_t hist[kTopkBins];
    uint32_t ncand;      // scores of the k-th bin appended to the candidate list (zeroed by whoever builds the histogram)
    uint32_t remaining;  // rank of the k-th largest inside its bin
    int32_t kth_bin;
    float center, inv;   // bin(x) = topk_bin(x, center, inv)
    uint32_t pad[3];
};
static_assert(sizeof(TopkRow) % 16 == 0, "rows of state stay 16-byte aligned");
constexpr int kTopkFusedRows = 256;

// Global scratch of the top-k launch for `rows` rows of at most max_len scores and budget k.
size_t topk_scratch_bytes(int32_t rows, int32_t max_len, int32_t k);

enum AttendMode { kDense = 0, kSelect = 1, kSparse = 2 };

struct AttendParams {
    const void *q, *K, *V;
    const void *k_new, *v_new;  // fused C.append: [B][Hkv][D] rows for token seq_lens[b] - 1, or nullptr
    const int32_t *seq_lens;
    const int32_t *positions;  // sparse: [B][Hkv][k]
    float *scores;             // select: [B][Hkv][score_stride]
    float *part_acc;           // [B][Hq][num_splits][D]
    float *part_ml;            // [B][Hq][num_splits][2]  (running max in log2 units, sum)
    int32_t *counters;         // [B][Hkv] chunks finished so far; zero between launches
    TopkRow *topk_rows;        // select, fused histogram: TopkRow [B][Hkv] that receives the chunks' histograms, else nullptr
    void *out;                 // [B][Hq][D]
    float *ml_out;             // optional [B][Hq][2]: final softmax maximum (log2 units) and sum per head
    int64_t stride_batch, stride_head, stride_tok;  // elements; paged: stride_batch is the page stride
    const int32_t *block_table;  // paged cache: [B][bt_stride] page ids, else nullptr
    int64_t bt_stride;
    int32_t page_shift;  // log2(page size)
    int32_t num_pages;   // pages in the pool
    int32_t select_rule; // select mode: td_selection (per-head: scores has one row per query head)
    int32_t kv_div;      // KV head of grid row g is g / kv_div (1, or the group size when a sparse
                         // layer runs one grid row per query head)
    int64_t score_stride;
    int32_t batch, num_q_heads, num_kv_heads;
    int32_t max_seq_len;
    int32_t k;
    int32_t chunk;       // tokens per workgroup
    int32_t num_splits;  // grid.x
    int32_t separate_merge;  // 1: the chunks only leave their partials and launch_merge folds them
    // Prefill through the decode kernel (vector-ALU kernel, full mode only): grid row block b is not a
    // sequence but new token new_first + b % new_per_seq of sequence cache_first + b / new_per_seq, which
    // attends to the positions up to its own, seq_lens[sequence] - num_new + token.  0: a decode step.
    int32_t new_per_seq, new_first, num_new, cache_first;
    float scale;
};

// Enqueues the split attention kernel (the last chunk to finish merges the partials).
// launch_attend: vector-ALU kernel for every supported dtype / head_dim, with `waves` wave64s
// per workgroup (4, or 8 where attend_supports_waves says so);
// launch_attend_mfma: matrix-core kernel, bf16 with head_dim 128 only, 4 or 8 waves.
bool attend_supports_waves(int group, int waves);
hipError_t launch_attend(int dtype, int head_dim, int group, int waves, int mode, const AttendParams &p,
                         hipStream_t stream);
hipError_t launch_attend_mfma(int group, int waves, int mode, const AttendParams &p, hipStream_t stream);

// Second launch of a split layer (p.separate_merge): one workgroup per (sequence, query head)
// folds the chunk partials that the attention launch left and writes the output row.  p and mode
// are those of the attention launch.
hipError_t launch_merge(int dtype, int head_dim, int mode, const AttendParams &p, hipStream_t stream);

// Prefill attention over the last num_new tokens of every sequence (bf16, head_dim 128; contiguous cache, or
// paged with pages of at least 16 tokens).
// The query rows of a KV head are the (token, head) pairs; a workgroup takes rows_per_wg of them and one
// chunk of the tokens.  With more than one chunk the workgroups leave partial states
//   part_ml [wg][chunk][rows_per_wg][2], part_acc [wg][chunk][rows_per_wg][128]   (wg = pair * row_blocks + row block)
// and a second kernel merges them.
struct PrefillParams {
    const void *q, *K, *V;  // q: [B][num_new][Hq][128]
    void *out;              // like q
    const int32_t *seq_lens;
    float *part_acc, *part_ml;
    int64_t stride_batch, stride_head, stride_tok;  // elements; paged: stride_batch is the page stride
    const int32_t *block_table;                     // paged cache: [B][bt_stride] page ids, else nullptr
    int64_t bt_stride;
    int32_t page_shift, num_pages;                  // log2(page size) >= 4; pages in the pool
    int32_t batch, num_q_heads, num_kv_heads, max_seq_len, num_new;
    int32_t rows_per_wg;  // 32 or 64
    int32_t row_blocks;   // workgroups per (sequence, KV head) and chunk
    int32_t chunk;        // tokens per chunk, a multiple of 64
    int32_t chunks;       // grid.y
    float scale;
};
struct PrefillPlan {
    int32_t rows_per_wg, row_blocks, chunk, chunks;
    size_t part_bytes;  // workspace for the partial states (0 with one chunk)
};
// Launch shape for `rows` = num_new * group query rows per (sequence, KV head), `pairs` such pairs and
// up to `part_avail` bytes for partial states.
PrefillPlan plan_prefill(int64_t rows, int64_t pairs, int32_t max_seq_len, size_t part_avail);
hipError_t launch_prefill(int group, const PrefillParams &p, hipStream_t stream);

// Mean-of-probabilities rule: prob[b][g][j] = mean over the group's heads of
// exp2(logit[b][h][j] * log2(e) - m_h) / l_h, from the per-head scaled logits and the final
// (m_h, l_h) that a selection launch leaves in ml.  rank receives log2(prob), which top-k ranks;
// prob (optional) receives the probabilities.
hipError_t launch_mean_prob(const float *head_logits, int64_t logit_stride, const float *ml, const int32_t *seq_lens,
                            int32_t batch, int32_t num_kv_heads, int32_t group, int32_t max_seq_len, float *rank,
                            int64_t rank_stride, float *prob, int64_t prob_stride, hipStream_t stream);

// argTopK over rows of fp32 scores.  state: TopkRow[rows], zero on entry and on exit; scratch:
// topk_scratch_bytes(rows, max_len, k) bytes.  have_histogram: a selection attention launch has
// already added every score to state[row].hist and set its bin map (one launch follows);
// otherwise the histogram is built here (two launches).  lengths_first: the rows' lengths differ
// a lot (a ragged batch), so a workgroup reads its row's length before it requests any score, and
// the many slices beyond a row's end cost no memory traffic; otherwise the scores are requested
// first, which saves one wait for memory in every workgroup.
hipError_t launch_topk(const float *scores, int64_t row_stride, int32_t rows, const int32_t *row_lens,
                       int32_t rows_per_len, int32_t max_len, int32_t k, int32_t *positions, TopkRow *state,
                       void *scratch, bool have_histogram, bool lengths_first, hipStream_t stream);
// Zeroes TopkRow[rows] (state outside the fixed region, before a launch_topk without histogram).
hipError_t launch_topk_reset(TopkRow *state, int32_t rows, hipStream_t stream);

// The layer loop of td_decode_step on a workspace that the caller names (default launch plan).  The
// ticket counters the shape uses are zeroed first; `error` receives the text of a failure.
td_status decode_step_on_workspace(char *workspace, size_t workspace_bytes, const td_shape *shape, int32_t num_layers,
                                   const int32_t *schedule, const void *const *q_layers, const void *const *K_layers,
                                   const void *const *V_layers, int32_t k, void *const *out_layers, int32_t *positions,
                                   void *hip_stream, char (&error)[256]);

// static_entry.hip: resolves the current device's copy of the static scratch array (idempotent);
// the text of the last failure of td_decode_step_static on this thread.
hipError_t static_scratch_setup();
const char *static_last_error();

// Streaming probe: copies `bytes` from src to dst, or (dst == nullptr) only reads src.
hipError_t launch_probe(void *dst, const void *src, size_t bytes, uint32_t *sink, hipStream_t stream);

}  // namespace tidal
