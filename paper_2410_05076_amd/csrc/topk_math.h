// Pure integer / bit arithmetic of the argTopK kernels (Alg. 1's rho := argTopK(<q,K>, k)): the
// order-preserving key of a score, its histogram bin, and the geometry of the slices a row is cut
// into.  No memory access and nothing GPU-specific, so the same functions compile for the device
// and, with a host compiler, into the CPU model that the tests run against the oracle.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define TD_HD __host__ __device__ __forceinline__
#else
#define TD_HD inline
#endif

namespace tidal {

constexpr int kTopkBins = 2048;         // histogram bins per row
constexpr int kTopkCandMax = 3584;      // scores of the k-th bin kept per row (with this the emit kernel needs under 32 KB of LDS: five workgroups per CU)
constexpr int kTopkSliceScores = 4096;  // scores per top-k workgroup
constexpr int kTopkThreads = 256;       // threads per top-k workgroup
constexpr int kTopkPerThread = kTopkSliceScores / kTopkThreads;  // 16 consecutive scores per thread

TD_HD uint32_t f32_bits(float f) {
    uint32_t u;
    __builtin_memcpy(&u, &f, 4);
    return u;
}

TD_HD float bits_f32(uint32_t u) {
    float f;
    __builtin_memcpy(&f, &u, 4);
    return f;
}

// Unsigned image of a float that orders like the float; -0 and +0 map to the same key.
TD_HD uint32_t order_key(float f) {
    uint32_t u = f32_bits(f);
    if (u == 0x80000000u) u = 0;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Histogram bin of a score: a monotone (non-decreasing) map of x onto [0, kTopkBins).
// y = (x - center) * inv, then 64 bins per octave of |y| over 2^-8 <= |y| < 2^8 on either side of
// zero: bins of constant relative width resolve the upper tail, where the k-th largest lives,
// whatever the scale of the scores.  |y| below 2^-8 (zero of either sign included) shares the two
// innermost bins, |y| of 2^8 and more the two outermost.  Scores whose keys are equal get the same
// bin; a row whose k-th bin holds more scores than the candidate list is selected exactly by a
// slower path, so the map only has to be monotone, never well balanced.
constexpr uint32_t kTopkBinLo = (uint32_t)(127 - 8) << 23;        // bits of 2^-8
constexpr uint32_t kTopkBinHi = ((uint32_t)(127 + 8) << 23) - 1;  // largest float below 2^8

TD_HD float topk_scaled(float x, float center, float inv) { return (x - center) * inv; }

TD_HD int topk_bin_of_scaled(float y) {
    const uint32_t u = f32_bits(y);
    uint32_t a = u & 0x7fffffffu;
    a = a < kTopkBinLo ? kTopkBinLo : (a > kTopkBinHi ? kTopkBinHi : a);
    const int t = (int)((a - kTopkBinLo) >> 17);  // 16 octaves x 64 = 0 .. 1023
    const bool negative = (u >> 31) != 0 && (u & 0x7fffffffu) != 0;
    return negative ? 1023 - t : 1024 + t;
}

TD_HD int topk_bin(float x, float center, float inv) { return topk_bin_of_scaled(topk_scaled(x, center, inv)); }

// The smallest scaled score whose bin is b or more: for every y that is not a NaN,
// topk_bin_of_scaled(y) >= b exactly when y >= topk_bin_floor(b).  With it a kernel that knows the
// bin of the k-th largest compares scaled scores with two constants instead of binning each one.
// b <= 0: every score (-inf); b >= kTopkBins: none (a NaN, which compares false).
TD_HD float topk_bin_floor(int b) {
    if (b >= kTopkBins) return bits_f32(0x7fc00000u);
    if (b > 1024) return bits_f32(kTopkBinLo + ((uint32_t)(b - 1024) << 17));
    if (b == 1024) return 0.f;  // -0 compares equal and lands in bin 1024 as well
    if (b <= 0) return bits_f32(0xff800000u);
    // negative side: bin 1023 - t for magnitudes a with (a - lo) >> 17 == t, so bin >= b means
    // a < lo + ((1024 - b) << 17): every y above minus that magnitude
    return bits_f32(0x80000000u | (kTopkBinLo + ((uint32_t)(1024 - b) << 17) - 1));
}

// The float whose order_key is `key` (the positive zero for the key of the zeros).
TD_HD float key_to_float(uint32_t key) { return bits_f32((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key); }

// A row of n scores starting `mis` floats (0..3) into a 16-byte granule is cut into slices of
// kTopkSliceScores / 4 granules; slice x covers granules [x * 1024, x * 1024 + 1024) of the row's
// granule sequence, i.e. tokens 4096 x - mis .. 4096 x - mis + 4095 clipped to [0, n).
TD_HD int topk_row_granules(int mis, int n) { return (mis + n + 3) >> 2; }
TD_HD int topk_active_slices(int mis, int n) {  // slices that hold at least one score; 1 for an empty row
    const int g = topk_row_granules(mis, n);
    const int s = (g + kTopkSliceScores / 4 - 1) / (kTopkSliceScores / 4);
    return s < 1 ? 1 : s;
}
TD_HD int topk_slice_first_token(int slice, int mis) { return slice * kTopkSliceScores - mis; }

inline int topk_slices(int32_t max_len) { return (int)(((int64_t)max_len + 3 + kTopkSliceScores - 1) / kTopkSliceScores); }

}  // namespace tidal
