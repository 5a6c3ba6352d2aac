// argTopK of Alg. 1 over rows of fp32 scores: an exact selection of the k-th largest score,
// then an order-preserving compaction, so positions come out in ascending token order and
// ties at the k-th value go to the smaller index.
//
// A row (up to 128K scores and more per KV head, few rows) is cut into slices of 4096 scores,
// one workgroup of 256 threads each, so that a handful of rows still fills the chip.  Slices of
// a row meet through global memory at kernel boundaries:
//   hist  every score is binned by the monotone map topk_bin (64 bins per octave around a
//         centre; bins of constant relative width resolve the upper tail, where the k-th largest
//         lives).  A selection layer's attention launch does this itself while the chunk's scores
//         sit in LDS (map centred on zero), so that two launches follow it; rows that come from
//         elsewhere are binned by topk_hist_kernel, which centres and scales the map on 256
//         samples of the row.  Each slice builds its histogram in LDS and adds the non-empty bins
//         to the row's histogram.
//   pick  every slice scans the row histogram from the top for the bin b* holding the k-th
//         largest score, counts its own scores above b* and appends its scores inside b*
//         (a few dozen per row for smooth distributions) to the row's candidate list.
//   emit  every slice selects the k-th key exactly among the candidates (order-preserving
//         uint32 image of the float), derives its output offset from the counts of the
//         slices before it, and compacts its scores in index order (each thread owns 16
//         consecutive scores, one prefix sum over the workgroup orders the slice).
// pick and emit never bin a score: "in bin b or above" is "scaled score >= topk_bin_floor(b)", so a
// score is classified by two compares with constants, and inside b* by a compare with the k-th
// score itself (the same order as the keys').  A row's bounds are checked per score only in its
// first and last slice.
// If a row has more candidates than the list holds (many equal scores), emit falls back to
// an exact radix select over the row's scores inside b*: slow, but never wrong.
// The row histogram is zero when a launch sequence starts and emit leaves it zero again (state
// of up to kTopkFusedRows rows lives where no other launch writes, so this holds across calls of
// different shapes; larger launches reset their state first).
#include "common.h"

namespace tidal {
namespace {

constexpr int kTopkWaves = kTopkThreads / kWave;
constexpr int kPerThread = kTopkPerThread / 4;             // 16-byte granules per thread
constexpr int kSliceGranules = kTopkThreads * kPerThread;  // 1024 granules = 4096 scores
constexpr int kBins = kTopkBins;
constexpr int kCandMax = kTopkCandMax;
static_assert(kSliceGranules * 4 == kTopkSliceScores, "slice size");

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, int lane) {
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t t = __shfl_up(v, o);
        if (lane >= o) v += t;
    }
    return v;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) v += __shfl_xor(v, o);
    return v;
}

// Inclusive prefix sum over the workgroup; *total receives the block sum.  s_tot: [kTopkWaves].
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, int lane, int wave, uint32_t *s_tot,
                                                        uint32_t *total) {
    const uint32_t incl = wave_inclusive_scan(v, lane);
    if (lane == kWave - 1) s_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) {
        const uint32_t t = s_tot[w];
        if (w < wave) before += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return incl + before;
}

// One row as 16-byte granules (it may start up to 3 floats into one; the buffer itself is
// 16-byte aligned, so the granule of a valid score never leaves the allocation), and the
// slice of it this workgroup owns.
struct Slice {
    const float *src;
    const float4 *src4;
    int mis, n, n4, first;  // first: index of the slice's first granule
    TopkRow *state;
    bool active;
};

__device__ __forceinline__ Slice open_slice(const float *scores, int64_t row_stride, const int32_t *row_lens,
                                            int rows_per_len, int max_len, int k, TopkRow *states) {
    Slice s;
    const int row = blockIdx.y;
    s.n = min(max(row_lens[row / rows_per_len], 0), max_len);
    s.src = scores + (int64_t)row * row_stride;
    s.mis = (int)((reinterpret_cast<uintptr_t>(s.src) >> 2) & 3);
    s.src4 = reinterpret_cast<const float4 *>(s.src - s.mis);
    s.n4 = topk_row_granules(s.mis, s.n);
    s.first = blockIdx.x * kSliceGranules;
    s.state = states + row;
    s.active = k < s.n && s.first < s.n4;  // k >= n needs no selection at all
    return s;
}

// The slice's scores: granule u of thread t is first + u*256 + t.  They are requested before the
// row's length is known (one wait for memory instead of two in a row): indices are clamped to
// the granule of score max_len - 1, which lies inside the row's buffer, and for_each_score masks
// what lies beyond the row's length.
__device__ __forceinline__ void load_slice_early(const float *scores, int64_t row_stride, int max_len, int tid,
                                                 float4 (&v)[kPerThread]) {
    const float *src = scores + (int64_t)blockIdx.y * row_stride;
    const int mis = (int)((reinterpret_cast<uintptr_t>(src) >> 2) & 3);
    const float4 *src4 = reinterpret_cast<const float4 *>(src - mis);
    const int last4 = ((mis + max_len + 3) >> 2) - 1;
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) v[u] = src4[min((int)blockIdx.x * kSliceGranules + u * kTopkThreads + tid, last4)];
}

// fn(score, token index, slot) for the slice's scores that lie inside the row; slot = 4 * u + e counts the
// thread's 16 scores.  A slice that lies wholly inside its row (all but the first and last of a row)
// skips the per-score bounds.
template <class Fn>
__device__ __forceinline__ void for_each_score(const Slice &s, int tid, const float4 (&v)[kPerThread], Fn fn) {
    const bool interior = 4 * s.first - s.mis >= 0 && 4 * (s.first + kSliceGranules) - s.mis <= s.n;
    if (interior) {
#pragma unroll
        for (int u = 0; u < kPerThread; ++u) {
            const int j = 4 * (s.first + u * kTopkThreads + tid) - s.mis;
            fn(v[u].x, j, 4 * u);
            fn(v[u].y, j + 1, 4 * u + 1);
            fn(v[u].z, j + 2, 4 * u + 2);
            fn(v[u].w, j + 3, 4 * u + 3);
        }
        return;
    }
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
        const int i = s.first + u * kTopkThreads + tid;
        const float f[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = 4 * i - s.mis + e;
            if (i < s.n4 && j >= 0 && j < s.n) fn(f[e], j, 4 * u + e);
        }
    }
}

__global__ __launch_bounds__(kTopkThreads) void topk_reset_kernel(TopkRow *states) {
    uint32_t *words = reinterpret_cast<uint32_t *>(states + blockIdx.x);
    for (int i = threadIdx.x; i < (int)(sizeof(TopkRow) / 4); i += kTopkThreads) words[i] = 0;
}

__global__ __launch_bounds__(kTopkThreads) void topk_hist_kernel(const float *scores, int64_t row_stride,
                                                                const int32_t *row_lens, int rows_per_len,
                                                                int max_len, int k, TopkRow *states,
                                                                bool lengths_first) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    float4 v[kPerThread];
    if (!lengths_first) load_slice_early(scores, row_stride, max_len, tid, v);
    asm volatile("" ::: "memory");  // requested before the row's length is read
    const Slice s = open_slice(scores, row_stride, row_lens, rows_per_len, max_len, k, states);
    if (!s.active) return;
    if (lengths_first) load_slice_early(scores, row_stride, max_len, tid, v);
    __shared__ __align__(8) uint32_t s_hist[kBins];
    __shared__ float s_lo[kTopkWaves], s_hi[kTopkWaves];
    // value range from 256 samples of the whole row: the same in every slice of the row
    const float x = s.src[(int64_t)tid * s.n / kTopkThreads];
    float lo = x, hi = x;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, o));
        hi = fmaxf(hi, __shfl_xor(hi, o));
    }
    if (lane == 0) {
        s_lo[wave] = lo;
        s_hi[wave] = hi;
    }
    for (int i = tid; i < kBins; i += kTopkThreads) s_hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) {
        lo = fminf(lo, s_lo[w]);
        hi = fmaxf(hi, s_hi[w]);
    }
    // The map is centred on the middle of the sampled range and scaled so that one sampled width is
    // 64 units: its 2^-8 .. 2^8 span then covers four sampled widths either side of the centre, at a
    // resolution far below the width.  A degenerate range (all samples equal or closer than the scale
    // can express, an infinity or a NaN among them) takes the plain map around zero, which stays monotone
    // for every input; such a row mostly lands in one bin and the exact paths decide.
    const float width = hi - lo;
    const bool usable = width > 1.0e-30f && width < 3.0e38f;
    const float center = usable ? 0.5f * lo + 0.5f * hi : 0.f;
    const float inv = usable ? 64.f / width : 1.f;
    if (blockIdx.x == 0 && tid == 0) {
        s.state->center = center;
        s.state->inv = inv;
        s.state->ncand = 0;
    }
    for_each_score(s, tid, v, [&](float f, int, int) { atomicAdd(&s_hist[topk_bin(f, center, inv)], 1u); });
    __syncthreads();
    // two neighbouring bins per 64-bit atomic (a count never carries out of its 32 bits)
    const uint64_t *pairs = reinterpret_cast<const uint64_t *>(s_hist);
    uint64_t *row_pairs = reinterpret_cast<uint64_t *>(s.state->hist);
    for (int i = tid; i < kBins / 2; i += kTopkThreads) {
        const uint64_t c = pairs[i];
        if (c) __hip_atomic_fetch_add(&row_pairs[i], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__global__ __launch_bounds__(kTopkThreads) void topk_pick_kernel(const float *scores, int64_t row_stride,
                                                                const int32_t *row_lens, int rows_per_len,
                                                                int max_len, int k, TopkRow *states, uint32_t *cand_key,
                                                                int32_t *cand_idx, uint32_t *slice_above,
                                                                int slices_per_row, bool lengths_first) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    if (lengths_first) {  // a slice beyond its row's end leaves before it requests anything else
        const int n = min(max(row_lens[blockIdx.y / rows_per_len], 0), max_len);
        const int mis = (int)((reinterpret_cast<uintptr_t>(scores + (int64_t)blockIdx.y * row_stride) >> 2) & 3);
        if (k >= n || (int)blockIdx.x * kSliceGranules >= topk_row_granules(mis, n)) return;
    }
    // the slice's scores, the row histogram and the bin map are requested before the row's length is read
    float4 v[kPerThread];
    load_slice_early(scores, row_stride, max_len, tid, v);
    // bin of the k-th largest: thread t owns bins 2047-8t .. 2040-8t, the scan walks downwards
    constexpr int PER = kBins / kTopkThreads;
    const TopkRow *early = states + blockIdx.y;
    uint32_t cnt[PER], mine = 0;
#pragma unroll
    for (int e = 0; e < PER; ++e) cnt[e] = early->hist[kBins - 1 - PER * tid - e];
    const float lo = early->center, inv = early->inv;  // the bin map's centre and scale
    asm volatile("" ::: "memory");
    const Slice s = open_slice(scores, row_stride, row_lens, rows_per_len, max_len, k, states);
    if (!s.active) return;
    __shared__ uint32_t s_tot[kTopkWaves];
    __shared__ uint32_t s_bin, s_remaining;
#pragma unroll
    for (int e = 0; e < PER; ++e) mine += cnt[e];
    uint32_t total;
    const uint32_t incl = block_inclusive_scan(mine, lane, wave, s_tot, &total);
    const uint32_t want = (uint32_t)k;
    uint32_t run = incl - mine;
    if (run < want && want <= incl) {
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            if (run < want && want <= run + cnt[e]) {
                s_bin = kBins - 1 - PER * tid - e;
                s_remaining = want - run;
            }
            run += cnt[e];
        }
    }
    __syncthreads();
    const int kth_bin = (int)s_bin;
    if (blockIdx.x == 0 && tid == 0) {
        s.state->kth_bin = kth_bin;
        s.state->remaining = s_remaining;
    }
    const int row = blockIdx.y;
    // its scores above the bin are counted, those inside it go to the row's candidate list: the
    // workgroup reserves room for all of its candidates with one atomic (one per candidate would
    // queue up on the row's counter)
    // (a scaled score lies in bin b or above exactly when it is at least topk_bin_floor(b): two compares
    // per score instead of the bin arithmetic)
    const float y_cand = topk_bin_floor(kth_bin), y_above = topk_bin_floor(kth_bin + 1);
    uint32_t above_mask = 0, cand_mask = 0;  // bit `slot` of a mask: the thread's slot-th score
    for_each_score(s, tid, v, [&](float f, int, int slot) {
        const float y = topk_scaled(f, lo, inv);
        const bool a = y >= y_above, c = y >= y_cand;
        above_mask |= (a ? 1u : 0u) << slot;
        cand_mask |= (c && !a ? 1u : 0u) << slot;
    });
    const uint32_t above = (uint32_t)__popc(above_mask);
    const uint32_t mine_c = (uint32_t)__popc(cand_mask);
    uint32_t both;
    const uint32_t excl = block_inclusive_scan(above | (mine_c << 16), lane, wave, s_tot, &both) - (above | (mine_c << 16));
    __shared__ uint32_t s_base;
    if (tid == 0) {
        slice_above[(int64_t)row * slices_per_row + blockIdx.x] = both & 0xffffu;
        s_base = (both >> 16) ? atomicAdd(&s.state->ncand, both >> 16) : 0u;
    }
    __syncthreads();
    if (cand_mask == 0) return;
    uint32_t at = s_base + (excl >> 16);
    for_each_score(s, tid, v, [&](float f, int j, int slot) {
        if ((cand_mask >> slot) & 1u) {
            if (at < (uint32_t)kCandMax) {
                cand_key[(int64_t)row * kCandMax + at] = order_key(f);
                cand_idx[(int64_t)row * kCandMax + at] = j;
            }
            ++at;
        }
    });
}

struct EmitShared {
    uint32_t key[kCandMax];
    int32_t idx[kCandMax];
    uint32_t hist[256];
    uint32_t member[kTopkThreads];  // keys of the candidates in the bucket of the k-th key
    uint32_t tot[kTopkWaves], lo[kTopkWaves], hi[kTopkWaves];
    uint32_t bin, remaining, kth, need, members;
};
static_assert(sizeof(EmitShared) <= 32 * 1024, "five workgroups per compute unit");

// Exact radix select (4 passes of 8 bits, most significant first) of the `remaining`-th
// largest key among either the candidate list in LDS or, with FROM_ROW, all scores of the
// row whose bin is kth_bin.  Leaves the key in sm.kth and the tie count in sm.need.
template <bool FROM_ROW>
__device__ __forceinline__ void radix_select(const Slice &s, EmitShared &sm, uint32_t count, uint32_t remaining,
                                             int kth_bin, float lo, float inv, int tid, int lane, int wave) {
    uint32_t prefix = 0, mask = 0;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        sm.hist[tid] = 0;
        __syncthreads();
        auto add = [&](uint32_t key) {
            if ((key & mask) == prefix) atomicAdd(&sm.hist[(key >> shift) & 255u], 1u);
        };
        if constexpr (FROM_ROW) {
            for (int i = tid; i < s.n4; i += kTopkThreads) {
                const float4 v = s.src4[i];
                const float f[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int j = 4 * i - s.mis + e;
                    if (j >= 0 && j < s.n && topk_bin(f[e], lo, inv) == kth_bin) add(order_key(f[e]));
                }
            }
        } else {
            for (uint32_t i = tid; i < count; i += kTopkThreads) add(sm.key[i]);
        }
        __syncthreads();
        const uint32_t cnt = sm.hist[255 - tid];  // thread t owns bin 255 - t: the scan walks downwards
        uint32_t total;
        const uint32_t incl = block_inclusive_scan(cnt, lane, wave, sm.tot, &total);
        const uint32_t excl = incl - cnt;
        if (excl < remaining && remaining <= incl) {
            sm.bin = 255 - tid;
            sm.remaining = remaining - excl;
        }
        __syncthreads();
        prefix |= sm.bin << shift;
        mask |= 0xffu << shift;
        remaining = sm.remaining;
        __syncthreads();
    }
    if (tid == 0) {
        sm.kth = prefix;
        sm.need = remaining;
    }
    __syncthreads();
}

// The `remaining`-th largest of the `count` keys in sm.key, and how many of its equals belong to the
// selection: leaves the key in sm.kth and that number in sm.need.  Every slice of a row does this, so it
// has to be cheap: the candidates of a row share a histogram bin, i.e. their keys lie in a narrow range, and
// 256 buckets spread linearly over exactly that range leave one or two keys in the bucket of the k-th -
// one pass of LDS atomics and one scan instead of a loop over all candidates in every thread (4.5 us for
// 230 candidates with four workgroups per compute unit) or four passes of a radix select over key bits
// that are mostly equal.  The bucket's few members are then ranked by counting.  A crowded bucket (many
// equal keys) takes the radix select.
__device__ __forceinline__ void select_among_candidates(const Slice &s, EmitShared &sm, uint32_t count, uint32_t remaining,
                                                        int kth_bin, float center, float inv, int tid, int lane, int wave) {
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    for (uint32_t i = tid; i < count; i += kTopkThreads) {
        kmin = min(kmin, sm.key[i]);
        kmax = max(kmax, sm.key[i]);
    }
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o));
    }
    if (lane == 0) {
        sm.lo[wave] = kmin;
        sm.hi[wave] = kmax;
    }
    sm.hist[tid] = 0;
    if (tid == 0) sm.members = 0;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) {
        kmin = min(kmin, sm.lo[w]);
        kmax = max(kmax, sm.hi[w]);
    }
    const uint32_t range = kmax - kmin;
    const int shift = range < 256u ? 0 : 24 - __clz(range);  // (range >> shift) < 256
    for (uint32_t i = tid; i < count; i += kTopkThreads) atomicAdd(&sm.hist[(sm.key[i] - kmin) >> shift], 1u);
    __syncthreads();
    const uint32_t cnt = sm.hist[255 - tid];  // thread t owns bucket 255 - t: the scan walks downwards
    uint32_t total;
    const uint32_t incl = block_inclusive_scan(cnt, lane, wave, sm.tot, &total);
    if (incl - cnt < remaining && remaining <= incl) {
        sm.bin = 255 - tid;
        sm.remaining = remaining - (incl - cnt);  // rank of the k-th key inside its bucket
    }
    __syncthreads();
    const uint32_t bucket = sm.bin, rank = sm.remaining, population = sm.hist[bucket];
    if (population > (uint32_t)kTopkThreads) {
        __syncthreads();  // everybody has read the bucket before the radix select reuses the histogram
        radix_select<false>(s, sm, count, remaining, kth_bin, center, inv, tid, lane, wave);
        return;
    }
    for (uint32_t i = tid; i < count; i += kTopkThreads) {
        const uint32_t key = sm.key[i];
        if (((key - kmin) >> shift) == bucket) sm.member[atomicAdd(&sm.members, 1u)] = key;
    }
    __syncthreads();
    // one member per thread: its rank by counting; equal keys agree on the answer
    const uint32_t mine = tid < (int)population ? sm.member[tid] : 0u;
    uint32_t above = 0, same = 0;
    for (uint32_t i = 0; i < population; ++i) {
        const uint32_t other = sm.member[i];
        above += other > mine ? 1u : 0u;
        same += other == mine ? 1u : 0u;
    }
    if (tid < (int)population && above < rank && rank <= above + same) {
        sm.kth = mine;
        sm.need = rank - above;
    }
    __syncthreads();
}

__global__ __launch_bounds__(kTopkThreads) void topk_emit_kernel(const float *scores, int64_t row_stride,
                                                                const int32_t *row_lens, int rows_per_len,
                                                                int max_len, int k, TopkRow *states,
                                                                const uint32_t *cand_key, const int32_t *cand_idx,
                                                                const uint32_t *slice_above, int slices_per_row,
                                                                int32_t *positions, bool lengths_first) {
    static_assert(kTopkThreads == 256, "one radix bin per thread");
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int row = blockIdx.y;
    if (lengths_first) {  // a slice beyond its row's end only zeroes its share of the histogram
        const int n = min(max(row_lens[row / rows_per_len], 0), max_len);
        const int mis = (int)((reinterpret_cast<uintptr_t>(scores + (int64_t)row * row_stride) >> 2) & 3);
        if (k < n && (int)blockIdx.x * kSliceGranules >= topk_row_granules(mis, n)) {
            for (int i = blockIdx.x * kTopkThreads + tid; i < kBins; i += gridDim.x * kTopkThreads) states[row].hist[i] = 0;
            return;
        }
    }
    // Everything whose address follows from the launch arguments alone is requested before the
    // row's length is read, so that the kernel waits for memory once, not three times in a row:
    // the row's state, the first candidates (rarely more than a workgroup's worth), the counts
    // of the earlier slices, and the slice's own scores (granules clamped into the row's buffer
    // of max_len scores; what lies beyond the row's length is masked further down).
    TopkRow *state = states + row;
    const uint32_t ncand = state->ncand, remaining = state->remaining;
    const int kth_bin = state->kth_bin;
    const float lo = state->center, inv = state->inv;  // the bin map's centre and scale
    const uint32_t early_key = cand_key[(int64_t)row * kCandMax + tid];
    const int32_t early_idx = cand_idx[(int64_t)row * kCandMax + tid];
    uint32_t gt_before = 0, eq_before = 0;
    for (int i = tid; i < (int)blockIdx.x; i += kTopkThreads) gt_before += slice_above[(int64_t)row * slices_per_row + i];
    float4 own[kPerThread];
    {
        const float *src = scores + (int64_t)row * row_stride;
        const int mis = (int)((reinterpret_cast<uintptr_t>(src) >> 2) & 3);
        const float4 *src4 = reinterpret_cast<const float4 *>(src - mis);
        const int last4 = ((mis + max_len + 3) >> 2) - 1;
#pragma unroll
        for (int u = 0; u < kPerThread; ++u)
            own[u] = src4[min((int)blockIdx.x * kSliceGranules + kPerThread * tid + u, last4)];
    }
    asm volatile("" ::: "memory");  // the loads above stay above the branches on the row's length
    // the row's histogram has served (pick read it in the launch before): back to zero for the next
    // launch sequence, every slice of the grid a share of the bins
    for (int i = blockIdx.x * kTopkThreads + tid; i < kBins; i += gridDim.x * kTopkThreads) state->hist[i] = 0;

    const Slice s = open_slice(scores, row_stride, row_lens, rows_per_len, max_len, k, states);
    int32_t *dst = positions + (int64_t)row * k;
    if (k >= s.n) {  // every token is selected: slice x writes entries x*4096 .. and the last one the -1 tail
        const int lo_i = blockIdx.x * kTopkSliceScores;
        const int hi_i = blockIdx.x == gridDim.x - 1 ? k : min(k, lo_i + kTopkSliceScores);
        for (int i = lo_i + tid; i < hi_i; i += kTopkThreads) dst[i] = i < s.n ? i : -1;
        return;
    }
    if (!s.active) return;

    __shared__ EmitShared sm;
    const int slice_start = 4 * s.first - s.mis;  // first token index of this slice

    if (ncand <= (uint32_t)kCandMax) {
        if (tid < (int)ncand) {
            sm.key[tid] = early_key;
            sm.idx[tid] = early_idx;
        }
        for (uint32_t i = tid + kTopkThreads; i < ncand; i += kTopkThreads) {
            sm.key[i] = cand_key[(int64_t)row * kCandMax + i];
            sm.idx[i] = cand_idx[(int64_t)row * kCandMax + i];
        }
        __syncthreads();
        select_among_candidates(s, sm, ncand, remaining, kth_bin, lo, inv, tid, lane, wave);
        const uint32_t kth = sm.kth;
        for (uint32_t i = tid; i < ncand; i += kTopkThreads) {
            if (sm.idx[i] < slice_start) {
                gt_before += sm.key[i] > kth ? 1u : 0u;
                eq_before += sm.key[i] == kth ? 1u : 0u;
            }
        }
    } else {
        radix_select<true>(s, sm, 0, remaining, kth_bin, lo, inv, tid, lane, wave);
        const uint32_t kth = sm.kth;
        for (int i = tid; i < min(s.first, s.n4); i += kTopkThreads) {
            const float4 q = s.src4[i];
            const float f[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = 4 * i - s.mis + e;
                if (j >= 0 && j < s.n && topk_bin(f[e], lo, inv) == kth_bin) {
                    const uint32_t key = order_key(f[e]);
                    gt_before += key > kth ? 1u : 0u;
                    eq_before += key == kth ? 1u : 0u;
                }
            }
        }
    }
    const uint32_t kth = sm.kth, need = sm.need;
    gt_before = wave_sum(gt_before);
    eq_before = wave_sum(eq_before);
    __syncthreads();
    if (lane == 0) {
        sm.tot[wave] = gt_before;
        sm.hist[wave] = eq_before;
    }
    __syncthreads();
    uint32_t gt_base = 0, eq_base = 0;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) {
        gt_base += sm.tot[w];
        eq_base += sm.hist[w];
    }
    __syncthreads();

    // compaction in index order: each thread owns 16 consecutive scores, so one prefix sum
    // over the threads orders the slice.  A score is selected for certain if it lies above the k-th
    // bin or inside it above the k-th key; the map is monotone, so inside the bin the float compare
    // with the k-th score says the same as the compare of the keys.
    const float y_cand = topk_bin_floor(kth_bin), y_above = topk_bin_floor(kth_bin + 1);
    const float kth_score = key_to_float(kth);
    uint32_t gt_mask = 0, eq_mask = 0;  // bit 4*u + e
    const int g0 = s.first + kPerThread * tid;  // the thread's first granule
    const int j0 = 4 * g0 - s.mis;              // and first token
    auto classify = [&](float f, int slot) {
        const float y = topk_scaled(f, lo, inv);
        const bool inbin = y >= y_cand;
        const bool gt = y >= y_above || (inbin && f > kth_score);
        const bool eq = inbin && f == kth_score;  // never true above the bin: the k-th score lies inside it
        gt_mask |= (gt ? 1u : 0u) << slot;
        eq_mask |= (eq && !gt ? 1u : 0u) << slot;
    };
    if (j0 >= 0 && j0 + 4 * kPerThread <= s.n) {
#pragma unroll
        for (int u = 0; u < kPerThread; ++u) {
            classify(own[u].x, 4 * u);
            classify(own[u].y, 4 * u + 1);
            classify(own[u].z, 4 * u + 2);
            classify(own[u].w, 4 * u + 3);
        }
    } else {
#pragma unroll
        for (int u = 0; u < kPerThread; ++u) {
            const float f[4] = {own[u].x, own[u].y, own[u].z, own[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = j0 + 4 * u + e;
                if (g0 + u < s.n4 && j >= 0 && j < s.n) classify(f[e], 4 * u + e);
            }
        }
    }
    const uint32_t packed = (uint32_t)__popc(gt_mask) | ((uint32_t)__popc(eq_mask) << 16);
    uint32_t total;
    const uint32_t excl = block_inclusive_scan(packed, lane, wave, sm.tot, &total) - packed;
    uint32_t gtb = gt_base + (excl & 0xffffu), eqb = eq_base + (excl >> 16);
    // the thread's selected scores in index order; an output index never leaves the row's k entries,
    // whatever the scores were (rows with NaNs are binned by their bits and compared as floats, so
    // their counts need not add up)
    uint32_t todo = gt_mask | eq_mask;
    while (todo) {
        const int t = __builtin_ctz(todo);
        todo &= todo - 1;
        if ((gt_mask >> t) & 1u) {
            const uint32_t at = gtb + min(eqb, need);
            if (at < (uint32_t)k) dst[at] = j0 + t;
            ++gtb;
        } else {
            if (eqb < need && gtb + eqb < (uint32_t)k) dst[gtb + eqb] = j0 + t;
            ++eqb;
        }
    }
}

}  // namespace

size_t topk_scratch_bytes(int32_t rows, int32_t max_len, int32_t) {
    const size_t slices = (size_t)topk_slices(max_len);
    return (size_t)rows * ((size_t)kCandMax * 8 + slices * 4);
}

hipError_t launch_topk_reset(TopkRow *state, int32_t rows, hipStream_t stream) {
    hipLaunchKernelGGL(topk_reset_kernel, dim3(rows), dim3(kTopkThreads), 0, stream, state);
    return hipGetLastError();
}

hipError_t launch_topk(const float *scores, int64_t row_stride, int32_t rows, const int32_t *row_lens,
                       int32_t rows_per_len, int32_t max_len, int32_t k, int32_t *positions, TopkRow *state,
                       void *scratch, bool have_histogram, bool lengths_first, hipStream_t stream) {
    const int slices = topk_slices(max_len);
    uint32_t *cand_key = static_cast<uint32_t *>(scratch);
    int32_t *cand_idx = reinterpret_cast<int32_t *>(cand_key + (size_t)rows * kCandMax);
    uint32_t *slice_above = reinterpret_cast<uint32_t *>(cand_idx + (size_t)rows * kCandMax);
    const dim3 grid(slices, rows), block(kTopkThreads);
    if (!have_histogram)
        hipLaunchKernelGGL(topk_hist_kernel, grid, block, 0, stream, scores, row_stride, row_lens, rows_per_len, max_len,
                           k, state, lengths_first);
    hipLaunchKernelGGL(topk_pick_kernel, grid, block, 0, stream, scores, row_stride, row_lens, rows_per_len, max_len,
                       k, state, cand_key, cand_idx, slice_above, slices, lengths_first);
    hipLaunchKernelGGL(topk_emit_kernel, grid, block, 0, stream, scores, row_stride, row_lens, rows_per_len, max_len,
                       k, state, cand_key, cand_idx, slice_above, slices, positions, lengths_first);
    return hipGetLastError();
}

}  // namespace tidal
