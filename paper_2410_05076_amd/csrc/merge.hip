// Second launch of a split attention layer: folds the chunk partials (running maximum, sum and
// weighted V accumulator of Eq. 1's softmax) that the attention launch left in the workspace and
// writes the output rows.  Used instead of the in-kernel ticket and last-chunk merge where a
// kernel boundary is cheaper than that chain: one compute unit reads partials back at about
// 30 GB/s, so the lone last chunk of a (sequence, KV head) needs 1.5 to 4 us for its G heads, while
// here every query head has a workgroup of its own and the boundary costs about 1.4 us.
#include "attend_tail.h"

namespace tidal {
namespace {

constexpr int kMergeThreads = 256;

template <int DT, int D>
__global__ __launch_bounds__(kMergeThreads) void merge_partials_kernel(const AttendParams p, int mode) {
    const int head = blockIdx.x, b = blockIdx.y;
    const int N = min(max(p.seq_lens[b], 0), p.max_seq_len);
    const int n_tok = mode == kSparse ? (N > 0 ? p.k : 0) : N;
    const int ns = (n_tok + p.chunk - 1) / p.chunk;  // chunks that had work
    if (ns <= 1) return;                             // nothing to do, or the only chunk wrote the row itself
    __shared__ MergeShared<kMergeThreads> red;
    merge_partials<DT, D, 1, kMergeThreads, false>(p, red, (int64_t)b * p.num_q_heads + head, ns);
}

template <int DT, int D>
hipError_t launch(int mode, const AttendParams &p, hipStream_t stream) {
    // one workgroup per query head: in a sparse layer that runs one grid row per query head,
    // p.num_kv_heads already counts query heads
    hipLaunchKernelGGL((merge_partials_kernel<DT, D>), dim3(p.num_q_heads, p.batch), dim3(kMergeThreads), 0, stream, p,
                       mode);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_merge(int dtype, int head_dim, int mode, const AttendParams &p, hipStream_t stream) {
    if (dtype == TD_BF16 && head_dim == 128) return launch<TD_BF16, 128>(mode, p, stream);
    if (dtype == TD_BF16 && head_dim == 64) return launch<TD_BF16, 64>(mode, p, stream);
    if (dtype == TD_F32 && head_dim == 128) return launch<TD_F32, 128>(mode, p, stream);
    if (dtype == TD_F32 && head_dim == 64) return launch<TD_F32, 64>(mode, p, stream);
    return hipErrorInvalidValue;
}

}  // namespace tidal
