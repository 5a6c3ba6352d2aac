// Shared by the attention kernels: constants, small device helpers, and the tail of a chunk -
// folding the workgroup's online-softmax states through LDS, publishing the chunk's partial,
// taking a ticket, and (in the chunk that finishes last) merging all partials of the
// (sequence, KV head) and writing the output row.
#pragma once
#include "coherent.h"
#include "common.h"

namespace tidal {
namespace {

constexpr int kWavesPerGroup = 4;  // default workgroup: four wave64s
constexpr int kThreads = kWavesPerGroup * kWave;
constexpr float kEmptyMax = -3.0e38f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// 16-byte load of cache data that is read exactly once: the non-temporal hint keeps the
// stream from displacing other lines (a plain 2 GiB streaming read measures ~6.3 TB/s with
// ordinary loads and ~7.2 TB/s with this hint on MI355X).
__device__ __forceinline__ uint4 stream_load16(const void *p) {
    const u32x4_t v = __builtin_nontemporal_load(static_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ uint32_t bf16_bits_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <int DT>
__device__ __forceinline__ void store_out(void *out, int64_t i, float v) {
    if constexpr (DT == TD_BF16)
        static_cast<uint16_t *>(out)[i] = (uint16_t)bf16_bits_rne(v);
    else
        static_cast<float *>(out)[i] = v;
}

// Writes the n scores that the workgroup's waves have put into LDS to dst, 16 bytes per lane
// where dst allows it.  Every thread of the workgroup calls it.  The stores are write-through
// (device scope), so the scores do not wait in the L2 for the write-back at the end of the launch:
// 16 MiB of scores at 4 x 128K tokens cost the launch 21 us that way and 11 us written through, in
// launches timed back to back on their own (non-temporal stores: the same for the matrix-core kernel,
// 4 us worse than either for the vector-ALU kernel); inside a whole decode step the difference is
// within the run-to-run spread.
template <int T>
__device__ __forceinline__ void write_staged_scores(const float *staged, int n, float *dst) {
    __syncthreads();
    if ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
        const int n4 = n & ~3;
        const __amdgpu_buffer_rsrc_t window = coherent_window(dst, (uint32_t)n4 * 4);
        for (int i = threadIdx.x * 4; i < n4; i += T * 4) {
            const float4 v = *reinterpret_cast<const float4 *>(staged + i);
            const u32x4_t x = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
            __builtin_amdgcn_raw_buffer_store_b128(x, window, (uint32_t)i * 4, 0, kCachePolicySc1);
        }
        for (int i = n4 + threadIdx.x; i < n; i += T) dst[i] = staged[i];
    } else {
        for (int i = threadIdx.x; i < n; i += T) dst[i] = staged[i];
    }
}

// Fused histogram of a selection layer: while a chunk's group scores pass through the kernel they
// are also binned, with the top-k launch's bin map centred on zero, into a histogram in LDS
// (kTopkBins words, 8-byte aligned, zeroed before the loop and a barrier), one LDS atomic per score
// inside the streaming loop, where it hides behind the loads; after the loop (and a barrier) the
// non-empty bins are added to the row's histogram in memory.  That one is zero when the launch
// starts (the top-k launch leaves it so).
// (Leaving out the bins below the one where the chunk's own count from the top reaches k, which the
// top-k launch can never need, was measured and gained nothing.)
__device__ __forceinline__ void bin_score(uint32_t *hist, float score) {
    atomicAdd(&hist[topk_bin(score, 0.f, 1.f)], 1u);
}
template <int T>
__device__ __forceinline__ void flush_score_histogram(TopkRow *row, const uint32_t *hist, bool first_chunk) {
    // two neighbouring bins per 64-bit atomic (a count never carries out of its 32 bits: a row has
    // fewer than 2^32 scores): half as many updates of the row's histogram in memory
    const uint64_t *pairs = reinterpret_cast<const uint64_t *>(hist);
    uint64_t *row_pairs = reinterpret_cast<uint64_t *>(row->hist);
    for (int i = threadIdx.x; i < kTopkBins / 2; i += T) {
        const uint64_t c = pairs[i];
        if (c) __hip_atomic_fetch_add(&row_pairs[i], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (first_chunk && threadIdx.x == 0) {
        row->center = 0.f;
        row->inv = 1.f;
        row->ncand = 0;  // the candidate list of the launches that follow starts empty
    }
}

// LDS needed by fold_states / finish_chunks for RG states of GC heads each, in a workgroup
// of T threads.
template <int D, int GC, int RG, int T>
struct TailShared {
    float m[RG][GC], l[RG][GC];
    // state accumulators [RG][GC][D]; reused by the final merge as [T] float4 + float2
    static constexpr int kAccFloats = RG * GC * D > T * 6 ? RG * GC * D : T * 6;
    __align__(16) float acc[kAccFloats];
    int last;
};

// Folds the RG online-softmax states of heads h0 .. h0+GC-1 (already in sm.m, sm.l, sm.acc;
// the caller has synchronised after writing them) with the rescaling rule.  With a single
// chunk the output row is written at once, otherwise the chunk's partial is published.
template <int DT, int D, int G, int GC, int RG, int T>
__device__ __forceinline__ void fold_states(const AttendParams &p, TailShared<D, GC, RG, T> &sm, int b, int g,
                                            int split, int ns, int h0) {
    for (int idx = threadIdx.x; idx < GC * D; idx += T) {
        const int i = idx / D, ch = idx % D;
        float mx = sm.m[0][i];
#pragma unroll
        for (int y = 1; y < RG; ++y) mx = fmaxf(mx, sm.m[y][i]);
        float ls = 0.f, as = 0.f;
#pragma unroll
        for (int y = 0; y < RG; ++y) {
            const float w = fast_exp2(sm.m[y][i] - mx);
            ls = fmaf(sm.l[y][i], w, ls);
            as = fmaf(sm.acc[(y * GC + i) * D + ch], w, as);
        }
        const int64_t head = (int64_t)b * p.num_q_heads + g * G + h0 + i;
        if (ns == 1) {  // the only chunk: finish here, no partials
            store_out<DT>(p.out, head * D + ch, ls > 0.f ? as / ls : 0.f);
            if (p.ml_out && ch == 0) {
                p.ml_out[head * 2] = mx;
                p.ml_out[head * 2 + 1] = ls;
            }
        } else if (p.separate_merge) {  // a second launch merges: the kernel boundary makes plain stores visible
            const int64_t slot = head * p.num_splits + split;
            p.part_acc[slot * D + ch] = as;
            if (ch == 0) {
                p.part_ml[slot * 2] = mx;
                p.part_ml[slot * 2 + 1] = ls;
            }
        } else {
            const int64_t slot = head * p.num_splits + split;
            publish(&p.part_acc[slot * D + ch], as);
            if (ch == 0) {
                publish(&p.part_ml[slot * 2], mx);
                publish(&p.part_ml[slot * 2 + 1], ls);
            }
        }
    }
}

// LDS of merge_partials for a workgroup of T threads: one float4 and one (max, sum) pair per thread.
template <int T>
struct MergeShared {
    __align__(16) float4 a[T];
    float2 ml[T];
};

// Folds the ns chunk partials of GH query heads (head0 .. head0 + GH - 1 of the flattened
// [sequence][query head] index) and writes their output rows.  Every thread of a workgroup of T
// threads calls it.  One pass over the partials: thread (sg, col) folds chunks sg, sg + NG, ... of
// one float4 column of one head with the online rescaling rule, eight chunks in flight at a time,
// then the NG threads of a column are folded through LDS.
// COHERENT: the partials come from workgroups of the same launch (device-scope write-through
// stores), so they are read with device-scope loads, which need no cache invalidate; otherwise an
// earlier launch wrote them and ordinary loads do.  (A single CU sustains only about 30 GB/s on
// these loads however many are in flight, so this phase costs about 1 us per 32 KiB of partials.)
template <int DT, int D, int GH, int T, bool COHERENT>
__device__ __forceinline__ void merge_partials(const AttendParams &p, MergeShared<T> &red, int64_t head0, int ns) {
    constexpr int COLS = GH * D / 4;  // float4 columns over all heads merged here
    constexpr int NG = T / COLS;      // chunk groups working in parallel
    static_assert(NG >= 1 && NG * COLS == T, "GH * D / 4 must divide the workgroup size");
    const int col = threadIdx.x % COLS, sg = threadIdx.x / COLS;
    const int hi = col / (D / 4), c4 = col % (D / 4);
    const int64_t head = head0 + hi;
    const __amdgpu_buffer_rsrc_t pa =  // the heads' partials, [GH][num_splits][D]
        coherent_window(p.part_acc + head0 * p.num_splits * D, (uint32_t)(GH * p.num_splits * D) * 4);
    const __amdgpu_buffer_rsrc_t pml =  // and their (max, sum) pairs, [GH][num_splits][2]
        coherent_window(p.part_ml + head0 * p.num_splits * 2, (uint32_t)(GH * p.num_splits) * 8);
    const uint32_t pa_off = ((uint32_t)(hi * p.num_splits) * D + c4 * 4) * 4;
    const uint32_t pml_off = (uint32_t)(hi * p.num_splits) * 8;
    constexpr int kPolicy = COHERENT ? kCachePolicySc1 : 0;
    float mm = kEmptyMax, ll = 0.f;
    float4 aa = make_float4(0.f, 0.f, 0.f, 0.f);
    constexpr int kBatch = 8;  // partials in flight per thread
    for (int s0 = sg; s0 < ns; s0 += NG * kBatch) {
        u32x4_t x[kBatch];
        u32x2_t v[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t s = min(s0 + j * NG, ns - 1);  // clamped repeats are ignored below
            x[j] = __builtin_amdgcn_raw_buffer_load_b128(pa, pa_off + s * (D * 4), 0, kPolicy);
            v[j] = __builtin_amdgcn_raw_buffer_load_b64(pml, pml_off + s * 8, 0, kPolicy);
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            if (s0 + j * NG < ns) {
                const float mj = __uint_as_float(v[j].x);
                const float mn = fmaxf(mm, mj);
                const float wa = fast_exp2(mm - mn), wb = fast_exp2(mj - mn);
                ll = ll * wa + __uint_as_float(v[j].y) * wb;
                aa.x = aa.x * wa + __uint_as_float(x[j].x) * wb;
                aa.y = aa.y * wa + __uint_as_float(x[j].y) * wb;
                aa.z = aa.z * wa + __uint_as_float(x[j].z) * wb;
                aa.w = aa.w * wa + __uint_as_float(x[j].w) * wb;
                mm = mn;
            }
        }
    }
    if constexpr (NG > 1) {
        red.a[threadIdx.x] = aa;
        red.ml[threadIdx.x] = make_float2(mm, ll);
        __syncthreads();
        if (sg == 0) {
#pragma unroll
            for (int o = 1; o < NG; ++o) {
                const float2 v = red.ml[o * COLS + col];
                const float4 x = red.a[o * COLS + col];
                const float mn = fmaxf(mm, v.x);
                const float wa = fast_exp2(mm - mn), wb = fast_exp2(v.x - mn);
                ll = ll * wa + v.y * wb;
                aa.x = aa.x * wa + x.x * wb;
                aa.y = aa.y * wa + x.y * wb;
                aa.z = aa.z * wa + x.z * wb;
                aa.w = aa.w * wa + x.w * wb;
                mm = mn;
            }
        }
    }
    if (sg == 0) {
        if (p.ml_out && c4 == 0) {
            p.ml_out[head * 2] = mm;
            p.ml_out[head * 2 + 1] = ll;
        }
        const float inv = ll > 0.f ? 1.f / ll : 0.f;
        const int64_t oi = head * D + c4 * 4;
        store_out<DT>(p.out, oi, aa.x * inv);
        store_out<DT>(p.out, oi + 1, aa.y * inv);
        store_out<DT>(p.out, oi + 2, aa.z * inv);
        store_out<DT>(p.out, oi + 3, aa.w * inv);
    }
}

// After every head's partial of this chunk has been published: the chunk that finishes last
// merges all partials of its (sequence, KV head).  Partials are published with device-scope
// write-through stores and every wave waits for its stores to complete before the barrier,
// so they are in memory before this workgroup's ticket is taken.  (A release fence in every
// workgroup would write back the whole L2 each time.)  The counter returns to zero for the
// next launch.
template <int DT, int D, int G, int GC, int RG, int T>
__device__ __forceinline__ void finish_chunks(const AttendParams &p, TailShared<D, GC, RG, T> &sm, int b, int g,
                                              int ns) {
    wait_for_stores();
    __syncthreads();
    if (threadIdx.x == 0) {
        int *counter = p.counters + b * p.num_kv_heads + g;
        const int done = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sm.last = done == ns - 1;
        if (sm.last) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!sm.last) return;
    static_assert(sizeof(MergeShared<T>) <= sizeof(sm.acc), "the merge reuses the state buffer");
    merge_partials<DT, D, G, T, true>(p, *reinterpret_cast<MergeShared<T> *>(sm.acc),  // sm.acc is free now
                                      (int64_t)b * p.num_q_heads + g * G, ns);
}

}  // namespace
}  // namespace tidal
