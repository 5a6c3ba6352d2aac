// argTopK of Alg. 1 over rows of fp32 scores: exact radix select of the k-th largest key,
// then an order-preserving compaction, so positions come out in ascending token order and
// ties at the k-th value go to the smaller index.
//
// One workgroup of 1024 threads per row.  fp32 scores are compared through the usual
// order-preserving map to uint32.  Four passes of 8 bits (most significant first) build a
// 256-bin histogram in LDS of the keys that still match the prefix found so far and pick
// the bin holding the k-th largest; after the last pass the prefix is that key exactly and
// `remaining` is how many keys equal to it are still to be taken.  The compaction pass
// walks the row in index order, 4096 scores per tile, with a block-wide prefix sum of
// (greater, equal) counts.
#include "common.h"

namespace tidal {
namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / kWave;

__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0;  // -0 and +0 compare equal
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, int lane) {
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t t = __shfl_up(v, o);
        if (lane >= o) v += t;
    }
    return v;
}

__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float *scores, int64_t row_stride,
                                                           const int32_t *row_lens, int rows_per_len,
                                                           int max_len, int k, int32_t *positions) {
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int n = min(max(row_lens[row / rows_per_len], 0), max_len);
    const float *src = scores + (int64_t)row * row_stride;
    int32_t *dst = positions + (int64_t)row * k;
    if (k >= n) {
        for (int i = tid; i < k; i += kTopkThreads) dst[i] = i < n ? i : -1;
        return;
    }

    // 16-byte granules: the row may start up to 3 floats into one (the buffer itself is
    // 16-byte aligned, so the granule of a valid score never leaves the allocation)
    const int mis = (int)((reinterpret_cast<uintptr_t>(src) >> 2) & 3);
    const float4 *src4 = reinterpret_cast<const float4 *>(src - mis);
    const int n4 = (mis + n + 3) >> 2;

    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_bin, s_remaining;
    __shared__ uint32_t s_wave_tot[kTopkWaves];

    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)k;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) s_hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < n4; i += kTopkThreads) {
            const float4 v = src4[i];
            const float f[4] = {v.x, v.y, v.z, v.w};
            const int j0 = 4 * i - mis;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = j0 + e;
                if (j >= 0 && j < n) {
                    const uint32_t key = order_key(f[e]);
                    if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255u], 1u);
                }
            }
        }
        __syncthreads();
        if (wave == 0) {
            // lane L owns bins 255-4L .. 252-4L, so ascending lanes walk the bins downwards
            uint32_t cnt[4], tot = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                cnt[e] = s_hist[255 - 4 * lane - e];
                tot += cnt[e];
            }
            const uint32_t incl = wave_inclusive_scan(tot, lane);
            uint32_t run = incl - tot;
            if (run < remaining && remaining <= incl) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (run < remaining && remaining <= run + cnt[e]) {
                        s_bin = 255 - 4 * lane - e;
                        s_remaining = remaining - run;
                    }
                    run += cnt[e];
                }
            }
        }
        __syncthreads();
        prefix |= s_bin << shift;
        mask |= 0xffu << shift;
        remaining = s_remaining;
    }

    const uint32_t kth = prefix, need = remaining;
    uint32_t gt_base = 0, eq_base = 0;
    for (int tile = 0; tile < n4; tile += kTopkThreads) {
        const int i = tile + tid;
        bool gt[4] = {false, false, false, false}, eq[4] = {false, false, false, false};
        uint32_t packed = 0;
        if (i < n4) {
            const float4 v = src4[i];
            const float f[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = 4 * i - mis + e;
                if (j >= 0 && j < n) {
                    const uint32_t key = order_key(f[e]);
                    gt[e] = key > kth;
                    eq[e] = key == kth;
                    packed += (gt[e] ? 1u : 0u) + (eq[e] ? 0x10000u : 0u);
                }
            }
        }
        const uint32_t incl = wave_inclusive_scan(packed, lane);
        if (lane == kWave - 1) s_wave_tot[wave] = incl;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kTopkWaves; ++w) {
            const uint32_t t = s_wave_tot[w];
            if (w < wave) before += t;
            total += t;
        }
        const uint32_t excl = incl - packed + before;
        uint32_t gtb = gt_base + (excl & 0xffffu), eqb = eq_base + (excl >> 16);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = 4 * i - mis + e;
            if (gt[e]) {
                dst[gtb + min(eqb, need)] = j;
                ++gtb;
            } else if (eq[e]) {
                if (eqb < need) dst[gtb + eqb] = j;
                ++eqb;
            }
        }
        gt_base += total & 0xffffu;
        eq_base += total >> 16;
        __syncthreads();
    }
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
