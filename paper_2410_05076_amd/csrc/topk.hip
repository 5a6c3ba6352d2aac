// argTopK of Alg. 1 over rows of fp32 scores: an exact selection of the k-th largest score,
// then an order-preserving compaction, so positions come out in ascending token order and
// ties at the k-th value go to the smaller index.
//
// One workgroup of 1024 threads per row; the row is streamed three times (it was just
// written by the selection layer and sits in L2 / Infinity Cache).
//   1. 1024 samples give a value range [lo, hi]; every score is binned by the monotone map
//      bin(x) = clamp(floor((x - lo) * 2048 / (hi - lo))) into a 2048-bin LDS histogram.
//      Linear bins spread the atomics (the top bits of a float key would pile most scores
//      into a handful of bins).  A block-wide scan from the top finds the bin holding the
//      k-th largest score and how many scores above that bin are already taken.
//   2. The keys of that one bin (a few dozen for smooth distributions) are gathered into
//      LDS and an exact radix select (4 passes of 8 bits on the order-preserving uint32
//      image of the float) finds the k-th key and the number of ties to take.  If the bin
//      holds more keys than the LDS list (all-equal rows, say) the radix select runs over
//      the whole row instead.
//   3. Compaction in index order, 4096 scores per tile, eight tiles per round, with a
//      block-wide prefix sum of (greater, equal) counts.
// Every streaming loop issues eight independent 16-byte loads per thread before it uses
// any of them, and rows of up to 32768 scores are read once and kept in registers.
#include "common.h"

namespace tidal {
namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / kWave;
constexpr int kBins = 2048;
constexpr int kCandMax = 8192;

__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0;  // -0 and +0 compare equal
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int linear_bin(float x, float lo, float inv) {
    return (int)fminf(fmaxf((x - lo) * inv, 0.f), (float)(kBins - 1));
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, int lane) {
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t t = __shfl_up(v, o);
        if (lane >= o) v += t;
    }
    return v;
}

// Inclusive prefix sum over the 1024 threads; *total receives the block sum.
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, int lane, int wave, uint32_t *s_wave_tot,
                                                        uint32_t *total) {
    const uint32_t incl = wave_inclusive_scan(v, lane);
    if (lane == kWave - 1) s_wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) {
        const uint32_t t = s_wave_tot[w];
        if (w < wave) before += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return incl + before;
}

// The scores of one row as 16-byte granules; the row may start up to 3 floats into one.
struct RowView {
    const float4 *src4;
    int mis, n, n4;
};

constexpr int kBatch = 8;  // 16-byte loads in flight per thread

// The scores of a row, streamed in rounds of kBatch granules per thread.  With RESIDENT the
// row fits one round: it is loaded once and later walks reuse the registers.
template <bool RESIDENT>
struct RowReader {
    const RowView &row;
    int tid;
    float4 regs[kBatch];

    __device__ __forceinline__ RowReader(const RowView &r, int t) : row(r), tid(t) {
        if constexpr (RESIDENT) load(0, regs);
    }
    __device__ __forceinline__ void load(int base, float4 (&v)[kBatch]) const {
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = base + u * kTopkThreads + tid;
            v[u] = i < row.n4 ? row.src4[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    // Calls fn(score, j) for every score of the row.
    template <class Fn>
    __device__ __forceinline__ void for_each(Fn fn) const {
        for (int base = 0; base < row.n4; base += kBatch * kTopkThreads) {
            float4 tmp[kBatch];
            if constexpr (!RESIDENT) load(base, tmp);
            const float4(&v)[kBatch] = RESIDENT ? regs : tmp;
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int i = base + u * kTopkThreads + tid;
                const float f[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int j = 4 * i - row.mis + e;
                    if (i < row.n4 && j >= 0 && j < row.n) fn(f[e], j);
                }
            }
        }
    }
};

struct Shared {
    uint32_t hist[kBins];
    uint32_t cand[kCandMax];
    uint32_t wave_tot[kTopkWaves];
    uint32_t tile_tot[kBatch][kTopkWaves];  // compaction: per (tile, wave) counts, then exclusive offsets
    float wave_lo[kTopkWaves], wave_hi[kTopkWaves];
    uint32_t bin, remaining, ncand;
};

// Exact radix select over keys: either the gathered list in LDS or every score of the row.
// On return *kth is the `remaining`-th largest key and *need how many keys equal to it
// still have to be taken.
template <bool FROM_ROW, class Reader>
__device__ __forceinline__ void radix_select(const Reader &reader, Shared &sm, uint32_t count, uint32_t remaining,
                                             int tid, int lane, int wave, uint32_t *kth, uint32_t *need) {
    uint32_t prefix = 0, mask = 0;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) sm.hist[tid] = 0;
        __syncthreads();
        auto add = [&](uint32_t key) {
            if ((key & mask) == prefix) atomicAdd(&sm.hist[(key >> shift) & 255u], 1u);
        };
        if constexpr (FROM_ROW) {
            reader.for_each([&](float f, int) { add(order_key(f)); });
        } else {
            for (uint32_t i = tid; i < count; i += kTopkThreads) add(sm.cand[i]);
        }
        __syncthreads();
        // thread t < 256 owns bin 255 - t, so the scan walks the bins downwards
        const uint32_t cnt = tid < 256 ? sm.hist[255 - tid] : 0u;
        uint32_t total;
        const uint32_t incl = block_inclusive_scan(cnt, lane, wave, sm.wave_tot, &total);
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
    *kth = prefix;
    *need = remaining;
}

template <bool RESIDENT>
__device__ __forceinline__ void topk_row(const RowView &row, const float *src, int k, int32_t *dst, Shared &sm,
                                         int tid, int lane, int wave) {
    const int n = row.n;
    // 1. value range from 1024 samples, linear histogram, bin of the k-th largest
    {
        const float x = src[(int64_t)tid * n / kTopkThreads];
        float lo = x, hi = x;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            lo = fminf(lo, __shfl_xor(lo, o));
            hi = fmaxf(hi, __shfl_xor(hi, o));
        }
        if (lane == 0) {
            sm.wave_lo[wave] = lo;
            sm.wave_hi[wave] = hi;
        }
        for (int i = tid; i < kBins; i += kTopkThreads) sm.hist[i] = 0;
        if (tid == 0) sm.ncand = 0;
    }
    const RowReader<RESIDENT> reader(row, tid);
    __syncthreads();
    float lo = sm.wave_lo[0], hi = sm.wave_hi[0];
#pragma unroll
    for (int w = 1; w < kTopkWaves; ++w) {
        lo = fminf(lo, sm.wave_lo[w]);
        hi = fmaxf(hi, sm.wave_hi[w]);
    }
    const float inv = hi > lo ? (float)kBins / (hi - lo) : 0.f;
    reader.for_each([&](float f, int) { atomicAdd(&sm.hist[linear_bin(f, lo, inv)], 1u); });
    __syncthreads();
    uint32_t remaining = (uint32_t)k;
    {
        // thread t owns bins 2047 - 2t and 2046 - 2t: the scan walks the bins downwards
        const uint32_t c1 = sm.hist[kBins - 1 - 2 * tid], c2 = sm.hist[kBins - 2 - 2 * tid];
        uint32_t total;
        const uint32_t incl = block_inclusive_scan(c1 + c2, lane, wave, sm.wave_tot, &total);
        const uint32_t excl = incl - (c1 + c2);
        if (excl < remaining && remaining <= incl) {
            const bool first = remaining <= excl + c1;
            sm.bin = kBins - 1 - 2 * tid - (first ? 0 : 1);
            sm.remaining = remaining - excl - (first ? 0u : c1);
        }
    }
    __syncthreads();
    const int kth_bin = (int)sm.bin;
    remaining = sm.remaining;

    // 2. gather that bin's keys and select exactly among them
    reader.for_each([&](float f, int) {
        if (linear_bin(f, lo, inv) == kth_bin) {
            const uint32_t at = atomicAdd(&sm.ncand, 1u);
            if (at < kCandMax) sm.cand[at] = order_key(f);
        }
    });
    __syncthreads();
    const uint32_t ncand = sm.ncand;
    uint32_t kth, need;
    if (ncand <= kCandMax)
        radix_select<false>(reader, sm, ncand, remaining, tid, lane, wave, &kth, &need);
    else
        radix_select<true>(reader, sm, 0, (uint32_t)k, tid, lane, wave, &kth, &need);

    // 3. compaction in index order: tile u of a round holds granules base + u*1024 + tid
    uint32_t gt_base = 0, eq_base = 0;
    for (int base = 0; base < row.n4; base += kBatch * kTopkThreads) {
        float4 tmp[kBatch];
        if constexpr (!RESIDENT) reader.load(base, tmp);
        const float4(&v)[kBatch] = RESIDENT ? reader.regs : tmp;
        uint32_t flags[kBatch], packed[kBatch];  // flags: bit e = greater, bit 4+e = equal
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = base + u * kTopkThreads + tid;
            const float f[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            flags[u] = 0;
            packed[u] = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = 4 * i - row.mis + e;
                if (i < row.n4 && j >= 0 && j < n) {
                    const uint32_t key = order_key(f[e]);
                    if (key > kth) {
                        flags[u] |= 1u << e;
                        packed[u] += 1u;
                    } else if (key == kth) {
                        flags[u] |= 16u << e;
                        packed[u] += 0x10000u;
                    }
                }
            }
        }
        uint32_t incl[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            incl[u] = wave_inclusive_scan(packed[u], lane);
            if (lane == kWave - 1) sm.tile_tot[u][wave] = incl[u];
        }
        __syncthreads();
        // exclusive offsets over the (tile, wave) pairs in tile-major order: 128 values, one wave
        static_assert(kBatch * kTopkWaves == 2 * kWave, "two values per lane");
        if (wave == 0) {
            uint32_t *flat = &sm.tile_tot[0][0];
            const uint32_t c0 = flat[2 * lane], c1 = flat[2 * lane + 1];
            const uint32_t inc = wave_inclusive_scan(c0 + c1, lane);
            flat[2 * lane] = inc - c0 - c1;
            flat[2 * lane + 1] = inc - c1;
            if (lane == kWave - 1) sm.wave_tot[0] = inc;  // round total
        }
        __syncthreads();
        const uint32_t round_total = sm.wave_tot[0];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = base + u * kTopkThreads + tid;
            const uint32_t excl = sm.tile_tot[u][wave] + incl[u] - packed[u];
            uint32_t gtb = gt_base + (excl & 0xffffu), eqb = eq_base + (excl >> 16);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = 4 * i - row.mis + e;
                if (flags[u] & (1u << e)) {
                    dst[gtb + min(eqb, need)] = j;
                    ++gtb;
                } else if (flags[u] & (16u << e)) {
                    if (eqb < need) dst[gtb + eqb] = j;
                    ++eqb;
                }
            }
        }
        gt_base += round_total & 0xffffu;
        eq_base += round_total >> 16;
        __syncthreads();
    }
}

__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float *scores, int64_t row_stride,
                                                           const int32_t *row_lens, int rows_per_len,
                                                           int max_len, int k, int32_t *positions) {
    const int r = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int n = min(max(row_lens[r / rows_per_len], 0), max_len);
    const float *src = scores + (int64_t)r * row_stride;
    int32_t *dst = positions + (int64_t)r * k;
    if (k >= n) {
        for (int i = tid; i < k; i += kTopkThreads) dst[i] = i < n ? i : -1;
        return;
    }
    // the buffer is 16-byte aligned, so the granule of a valid score never leaves the allocation
    RowView row;
    row.mis = (int)((reinterpret_cast<uintptr_t>(src) >> 2) & 3);
    row.src4 = reinterpret_cast<const float4 *>(src - row.mis);
    row.n = n;
    row.n4 = (row.mis + n + 3) >> 2;
    __shared__ Shared sm;
    if (row.n4 <= kBatch * kTopkThreads)
        topk_row<true>(row, src, k, dst, sm, tid, lane, wave);
    else
        topk_row<false>(row, src, k, dst, sm, tid, lane, wave);
}

}  // namespace

hipError_t launch_topk(const float *scores, int64_t row_stride, int32_t rows, const int32_t *row_lens,
                       int32_t rows_per_len, int32_t max_len, int32_t k, int32_t *positions,
                       hipStream_t stream) {
    hipLaunchKernelGGL(topk_kernel, dim3(rows), dim3(kTopkThreads), 0, stream, scores, row_stride,
                       row_lens, rows_per_len, max_len, k, positions);
    return hipGetLastError();
}

}  // namespace tidal
