// Second pass of the mean-of-probabilities selection rule (a grouped-query reading of the
// paper's "tokens with the highest attention scores", Sec. 3.1): the selection launch has
// written every head's scaled logits and left the heads' final softmax maximum and sum; this
// kernel turns them into one row of group scores per KV head,
//   prob[b][g][j] = (1/G) sum_{h in g} exp(s_h[j] - max_h) / sum_h,
// four tokens per thread.  It reads G floats and writes one per token, all L2-resident.  Top-k
// ranks log2(prob) - the same order, but spread evenly enough for its histogram, which
// attention probabilities (a few large, most tiny) are not; the probabilities themselves go to
// the caller's buffer when there is one.
#include "common.h"

namespace tidal {
namespace {

constexpr int kProbThreads = 256;

template <int G>
__global__ __launch_bounds__(kProbThreads) void mean_prob_kernel(const float *head_logits, int64_t logit_stride,
                                                                 const float *ml, const int32_t *seq_lens,
                                                                 int32_t num_kv_heads, int32_t max_seq_len,
                                                                 float *rank, int64_t rank_stride, float *prob,
                                                                 int64_t prob_stride) {
    const int g = blockIdx.y, b = blockIdx.z;
    const int n = min(max(seq_lens[b], 0), max_seq_len);
    const int j0 = (blockIdx.x * kProbThreads + threadIdx.x) * 4;
    if (j0 >= n) return;
    const int64_t head0 = ((int64_t)b * num_kv_heads + g) * G;
    float m[G], inv[G];
#pragma unroll
    for (int i = 0; i < G; ++i) {
        m[i] = ml[(head0 + i) * 2];
        const float l = ml[(head0 + i) * 2 + 1];
        inv[i] = l > 0.f ? 1.f / (l * G) : 0.f;
    }
    const bool wide = j0 + 4 <= n && (logit_stride & 3) == 0 && (reinterpret_cast<uintptr_t>(head_logits) & 15u) == 0;
    float r[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < G; ++i) {
        const float *src = head_logits + (head0 + i) * logit_stride + j0;
        float x[4];
        if (wide) {
            const float4 v = *reinterpret_cast<const float4 *>(src);
            x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = j0 + e < n ? src[e] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = fmaf(__builtin_amdgcn_exp2f(x[e] * kLog2e - m[i]), inv[i], r[e]);
    }
    auto write4 = [&](float *row, int64_t stride, const float (&v)[4]) {
        float *dst = row + ((int64_t)b * num_kv_heads + g) * stride + j0;
        if (j0 + 4 <= n && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
            *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (j0 + e < n) dst[e] = v[e];
        }
    };
    if (prob) write4(prob, prob_stride, r);
    float lg[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) lg[e] = fmaxf(__builtin_amdgcn_logf(r[e]), -200.f);  // log2; zero probability ranks last
    write4(rank, rank_stride, lg);
}

}  // namespace

hipError_t launch_mean_prob(const float *head_logits, int64_t logit_stride, const float *ml, const int32_t *seq_lens,
                            int32_t batch, int32_t num_kv_heads, int32_t group, int32_t max_seq_len, float *rank,
                            int64_t rank_stride, float *prob, int64_t prob_stride, hipStream_t stream) {
    const dim3 grid((max_seq_len + kProbThreads * 4 - 1) / (kProbThreads * 4), num_kv_heads, batch), block(kProbThreads);
#define TIDAL_MEAN_PROB(G)                                                                                           \
    hipLaunchKernelGGL(mean_prob_kernel<G>, grid, block, 0, stream, head_logits, logit_stride, ml, seq_lens,          \
                       num_kv_heads, max_seq_len, rank, rank_stride, prob, prob_stride)
    switch (group) {
    case 1: TIDAL_MEAN_PROB(1); break;
    case 2: TIDAL_MEAN_PROB(2); break;
    case 4: TIDAL_MEAN_PROB(4); break;
    case 8: TIDAL_MEAN_PROB(8); break;
    default: return hipErrorInvalidValue;
    }
#undef TIDAL_MEAN_PROB
    return hipGetLastError();
}

}  // namespace tidal
