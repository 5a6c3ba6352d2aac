// CPU model of the index arithmetic of the argTopK kernels (paper_2410_05076_amd/csrc/topk.hip),
// for tests only: the same three phases - histogram, pick (k-th bin, per-slice counts of the scores
// above it, candidate list in arbitrary order), emit (exact k-th key among the candidates, output
// offset of a slice from the counts and candidates before it, order-preserving compaction, and the
// exact fallback when the list overflows) - written as plain sequential loops over rows and
// slices.  It shares with the kernels only the pure functions of topk_math.h (key, bin map, slice
// geometry).  Tests compare it with the oracle's argTopK on rows built around the slice and
// candidate-list boundaries, so that the offset logic is checked without a GPU.  Nothing in the
// library calls it.
#include <stdint.h>
#include <stdlib.h>

#include <algorithm>
#include <vector>

#include "topk_math.h"

using namespace tidal;

namespace {

struct Cand {
    uint32_t key;
    int32_t idx;
    uint32_t defb;
};

// scores of the row by token index, or a value that never matters outside [0, n)
struct Row {
    const float *src;
    int mis, n;
    float at(int j) const { return src[j]; }
};

void bin_map_from_samples(const Row &r, float *center, float *inv) {
    float lo = 0.f, hi = 0.f;
    for (int t = 0; t < kTopkThreads; ++t) {
        const float x = r.src[(int64_t)t * r.n / kTopkThreads];
        lo = t ? std::min(lo, x) : x;
        hi = t ? std::max(hi, x) : x;
    }
    const float width = hi - lo;
    const bool usable = width > 1.0e-30f && width < 3.0e38f;
    *center = usable ? 0.5f * lo + 0.5f * hi : 0.f;
    *inv = usable ? 64.f / width : 1.f;
}

void select_row(const Row &r, int k, bool fused_bins, int cand_max, uint32_t order_seed, int32_t *dst, int *path) {
    const int n = r.n;
    const int nslices = topk_active_slices(r.mis, n);
    if (k >= n) {
        for (int i = 0; i < k; ++i) dst[i] = i < n ? i : -1;
        *path = 0;
        return;
    }
    // hist
    float center = 0.f, inv = 1.f;
    if (!fused_bins) bin_map_from_samples(r, &center, &inv);
    std::vector<uint32_t> hist(kTopkBins, 0);
    for (int j = 0; j < n; ++j) ++hist[topk_bin(r.at(j), center, inv)];
    // pick: bin of the k-th largest, scanning from the top
    int kth_bin = 0;
    uint32_t remaining = 0, run = 0;
    for (int b = kTopkBins - 1; b >= 0; --b) {
        if (run < (uint32_t)k && (uint32_t)k <= run + hist[b]) {
            kth_bin = b;
            remaining = (uint32_t)k - run;
        }
        run += hist[b];
    }
    // ... every slice counts its scores above the bin and appends those inside it (as the kernels do:
    // by comparing the scaled score with the lower ends of the bin and of the next one); slices run
    // in an arbitrary order, which decides the order of the list
    const float y_cand = topk_bin_floor(kth_bin), y_above = topk_bin_floor(kth_bin + 1);
    std::vector<int> order(nslices);
    for (int i = 0; i < nslices; ++i) order[i] = i;
    uint32_t rng = order_seed * 2654435761u + 12345u;
    for (int i = nslices - 1; i > 0; --i) {
        rng = rng * 1664525u + 1013904223u;
        std::swap(order[i], order[(rng >> 8) % (uint32_t)(i + 1)]);
    }
    std::vector<uint32_t> slice_above(nslices, 0);
    std::vector<Cand> list;
    uint32_t ncand = 0;
    for (int oi = 0; oi < nslices; ++oi) {
        const int sl = order[oi];
        const int first = topk_slice_first_token(sl, r.mis);
        for (int t = 0; t < kTopkSliceScores; ++t) {
            const int j = first + t;
            if (j < 0 || j >= n) continue;
            const float y = topk_scaled(r.at(j), center, inv);
            slice_above[sl] += y >= y_above;
            if (y >= y_cand && !(y >= y_above)) {
                if (ncand < (uint32_t)cand_max) list.push_back(Cand{order_key(r.at(j)), j, 0});
                ++ncand;
            }
        }
    }
    // emit: the k-th key exactly, from the list or, if it overflowed, from the row
    *path = ncand <= (uint32_t)cand_max ? 1 : 2;
    std::vector<uint32_t> keys;
    if (*path == 1) {
        for (const Cand &c : list) keys.push_back(c.key);
    } else {
        for (int j = 0; j < n; ++j)
            if (topk_bin(r.at(j), center, inv) == kth_bin) keys.push_back(order_key(r.at(j)));
    }
    std::sort(keys.begin(), keys.end(), [](uint32_t a, uint32_t b) { return a > b; });
    const uint32_t kth = keys[remaining - 1];
    uint32_t above = 0;
    for (uint32_t key : keys) above += key > kth;
    const uint32_t need = remaining - above;
    const float kth_score = key_to_float(kth);
    for (int i = 0; i < k; ++i) dst[i] = -9;
    for (int sl = 0; sl < nslices; ++sl) {
        const int first = topk_slice_first_token(sl, r.mis);
        // selected for certain / equal to the k-th key, before this slice
        uint32_t gtb = 0, eqb = 0;
        for (int e = 0; e < sl; ++e) gtb += slice_above[e];
        if (*path == 1) {
            for (const Cand &c : list) {
                if (c.idx < first) {
                    gtb += c.key > kth;
                    eqb += c.key == kth;
                }
            }
        } else {
            for (int j = 0; j < std::min(first, n); ++j) {
                if (topk_bin(r.at(j), center, inv) == kth_bin) {
                    gtb += order_key(r.at(j)) > kth;
                    eqb += order_key(r.at(j)) == kth;
                }
            }
        }
        for (int t = 0; t < kTopkSliceScores; ++t) {
            const int j = first + t;
            if (j < 0 || j >= n) continue;
            const float f = r.at(j), y = topk_scaled(f, center, inv);
            const bool inbin = y >= y_cand;
            if (y >= y_above || (inbin && f > kth_score)) {
                const uint32_t at = gtb + std::min(eqb, need);
                if (at < (uint32_t)k) dst[at] = j;
                ++gtb;
            } else if (inbin && f == kth_score) {
                if (eqb < need && gtb + eqb < (uint32_t)k) dst[gtb + eqb] = j;
                ++eqb;
            }
        }
    }
}

}  // namespace

// rows of fp32 scores as td_topk takes them (host pointers); row r starts `row_stride * r +
// first_mis` floats into a 16-byte aligned buffer, which fixes how its slices are cut.  fused_bins:
// the bin map of a selection layer's attention launch (centred on zero) instead of the sampled
// one.  cand_max: capacity of the candidate list (kTopkCandMax in the kernels; smaller values
// exercise the fallback).  paths[r] receives 0 (k >= n), 1 (candidate list) or 2 (fallback).
extern "C" int topk_model(const float *scores, int64_t row_stride, int rows, const int32_t *row_lens, int rows_per_len,
                          int max_len, int k, int first_mis, int fused_bins, int cand_max, uint32_t order_seed,
                          int32_t *positions, int32_t *paths) {
    if (cand_max < 1 || k < 1) return 1;
    for (int row = 0; row < rows; ++row) {
        Row r;
        r.src = scores + (int64_t)row * row_stride;
        r.mis = (int)(((int64_t)row * row_stride + first_mis) & 3);
        r.n = std::min(std::max(row_lens[row / rows_per_len], 0), max_len);
        select_row(r, k, fused_bins != 0, cand_max, order_seed + (uint32_t)row, positions + (int64_t)row * k, paths + row);
    }
    return 0;
}

extern "C" int topk_model_bin(float x, float center, float inv) { return topk_bin(x, center, inv); }
extern "C" int topk_model_bin_of_scaled(float y) { return topk_bin_of_scaled(y); }
extern "C" float topk_model_bin_floor(int b) { return topk_bin_floor(b); }
extern "C" float topk_model_key_to_float(uint32_t key) { return key_to_float(key); }
extern "C" uint32_t topk_model_key(float x) { return order_key(x); }
