// Split-K decode attention for gfx950: Eq. 1 of the paper for one query row per head, over
// either the whole KV cache (full attention and token selection layers of Alg. 1) or the
// rows named by rho (position persistent sparse attention).
//
// Work decomposition.  grid = (token chunks, KV heads, sequences).  A workgroup of four
// wave64s streams one chunk of consecutive tokens of one (sequence, KV head) and serves all
// G query heads of the group from the same loaded rows, so each K/V byte is fetched once.  A row of head_dim
// elements is covered by LPR lanes holding 16 bytes each, so one wave-wide 128-bit load
// fetches 64/LPR whole rows, fully coalesced; a dot product is finished by a DPP reduction
// over those LPR lanes.  Each lane keeps an online-softmax state (running max, sum, its
// slice of the output) per query head; states are merged across row groups, waves and
// finally chunks with the usual rescaling rule.  Chunk partials go to a workspace; the
// workgroup that finishes last for a (sequence, KV head), found with a device-scope
// ticket counter, merges them and writes the output, so a layer is one launch.
//
// Token selection (Sec. 3.1): the scaled inner products are not turned into probabilities;
// their sum over the group's query heads is written once per token while the row is in
// registers, and top-k runs on those sums afterwards.
#include "attend_tail.h"

namespace tidal {
namespace {

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over the LPR consecutive lanes that hold one row; every lane gets the same bits.
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
    v += dpp_move<0xB1>(v);                        // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);                        // quad_perm [2,3,0,1]
    if constexpr (LPR >= 8) v += dpp_move<0x141>(v);   // row_half_mirror
    if constexpr (LPR >= 16) v += dpp_move<0x140>(v);  // row_mirror
    if constexpr (LPR >= 32) v += __shfl_xor(v, 16);
    return v;
}

template <int DT>
struct Elems;
template <>
struct Elems<TD_BF16> {
    static constexpr int kPerLane = 8;
    static constexpr int kBytes = 2;
    static __device__ __forceinline__ void unpack(const uint4 &r, float (&f)[8]) {
        f[0] = __uint_as_float(r.x << 16);
        f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16);
        f[3] = __uint_as_float(r.y & 0xffff0000u);
        f[4] = __uint_as_float(r.z << 16);
        f[5] = __uint_as_float(r.z & 0xffff0000u);
        f[6] = __uint_as_float(r.w << 16);
        f[7] = __uint_as_float(r.w & 0xffff0000u);
    }
};
template <>
struct Elems<TD_F32> {
    static constexpr int kPerLane = 4;
    static constexpr int kBytes = 4;
    static __device__ __forceinline__ void unpack(const uint4 &r, float (&f)[4]) {
        f[0] = __uint_as_float(r.x);
        f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z);
        f[3] = __uint_as_float(r.w);
    }
};

// Up to four query heads per group the streaming loop fits 128 registers, i.e. four
// workgroups per CU; the attribute keeps the rarely executed final merge from raising the
// kernel's register count above that.
//
// W is the number of wave64s per workgroup (4 or 8).  Eight-wave workgroups own chunks twice
// as long, so a (sequence, KV head) has half as many partials to merge across workgroups -
// the merge inside a workgroup goes through LDS and is much cheaper - which pays when the
// launch is short enough for its tail to matter.
//
// PAGED: the cache is a pool of pages behind a block table.  Logical token j of sequence b is
// in page block_table[b][j >> page_shift] at slot j & (page_size - 1); p.stride_batch is then
// the stride between pages.  Everything else (chunks, scores, positions) stays in logical
// token indices.  Full and selection layers stage the chunk's slice of the block table in
// LDS; sparse layers look the page of every position up while they stage the positions.
// Page ids are clamped into the pool, so a wrong table cannot cause an access outside it.
template <int DT, int D, int G, int MODE, int W, bool PAGED>
__global__ __launch_bounds__(W *kWave) __attribute__((amdgpu_waves_per_eu(G <= 4 && MODE != kSparse ? 4 : 1)))
void attend_split_kernel(const AttendParams p) {
    constexpr int T = W * kWave;  // threads per workgroup
    using E = Elems<DT>;
    constexpr int EPL = E::kPerLane;
    constexpr int LPR = D / EPL;        // lanes per row
    constexpr int TPW = kWave / LPR;    // rows per wave-wide load
    // row loads in flight per wave for each of K and V: the gather of a sparse layer is one
    // short burst, so it issues twice as many at once
    constexpr int kUnroll = MODE == kSparse && G <= 4 ? 8 : 4;
    constexpr int STEP = kUnroll * TPW; // rows per wave per iteration

    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int r = lane / LPR, c = lane % LPR;
    // the sequence whose cache row block b reads: b itself, except when the rows are the new tokens of a prefill
    const bool prefill = MODE == kDense && p.new_per_seq > 0;
    const int bc = prefill ? p.cache_first + b / p.new_per_seq : b;

    // A workgroup owns p.chunk consecutive tokens (a multiple of the 128-token granule): a
    // contiguous stream per workgroup keeps TLB and DRAM-page locality.
    constexpr int TILE = W * STEP;
    const int t0 = split * p.chunk;

    // The first loads depend on the launch arguments only.  They are issued here, ahead of the
    // read of the sequence length, so all of them are in flight together: this lane's slice of
    // the G queries of the group and, in sparse mode, the chunk's positions (staged in LDS
    // below, once the sequence length has said that the workgroup has work).
    uint4 qraw[G];
#pragma unroll
    for (int i = 0; i < G; ++i)
        qraw[i] = *(const uint4 *)((const char *)p.q +
                                   (((int64_t)b * p.num_q_heads + g * G + i) * D + c * EPL) * E::kBytes);
    constexpr int kPosPerThread = MODE == kSparse ? kSparseChunkMax / T : 1;
    int pstage[kPosPerThread];
    if constexpr (MODE == kSparse) {
        const int32_t *pos = p.positions + ((int64_t)b * p.num_kv_heads + g) * p.k;
        const int len = min(p.k - t0, p.chunk);
#pragma unroll
        for (int i = 0; i < kPosPerThread; ++i) {
            const int j = i * T + threadIdx.x;
            pstage[i] = i * T < len ? pos[t0 + min(j, len - 1)] : -1;  // the condition is workgroup-uniform
        }
    }
    // paged full / selection layers: the block-table entries of the chunk's pages (the chunk is
    // bounded by max_seq_len here, by the sequence length below)
    constexpr bool kStageTable = PAGED && MODE != kSparse;
    constexpr int kTablePerThread = kStageTable ? kPageStageMax / T : 1;
    int tstage[kTablePerThread];
    const int first_page = PAGED ? t0 >> p.page_shift : 0;
    if constexpr (kStageTable) {
        const int32_t *table = p.block_table + (int64_t)bc * p.bt_stride + first_page;
        const int pages = ((min(p.max_seq_len, t0 + p.chunk) - 1) >> p.page_shift) - first_page + 1;
#pragma unroll
        for (int i = 0; i < kTablePerThread; ++i) {
            const int j = i * T + threadIdx.x;
            tstage[i] = i * T < pages ? table[min(j, pages - 1)] : 0;  // workgroup-uniform condition
        }
    }
    asm volatile("" ::: "memory");  // the loads above stay above the branch on the sequence length

    int N = min(max(p.seq_lens[bc], 0), p.max_seq_len);
    if (prefill) {
        // the new token's own position + 1; a token before the start of the cache yields zeros
        N = N - p.num_new + p.new_first + b % p.new_per_seq + 1;
        if (N <= 0) {
            if (split == 0)
                for (int i = threadIdx.x; i < G * D; i += T) store_out<DT>(p.out, ((int64_t)b * p.num_q_heads + g * G) * D + i, 0.f);
            return;
        }
    }
    const int n_tok = MODE == kSparse ? (N > 0 ? p.k : 0) : N;
    if (t0 >= n_tok) return;
    const int t1 = min(n_tok, t0 + p.chunk);
    const int ns = (n_tok + p.chunk - 1) / p.chunk;  // workgroups of this (sequence, KV head) with work

    __shared__ int s_pos[MODE == kSparse ? kSparseChunkMax : 1];
    __shared__ int s_page[PAGED ? (MODE == kSparse ? kSparseChunkMax : kPageStageMax) : 1];
    if constexpr (MODE == kSparse) {
#pragma unroll
        for (int i = 0; i < kPosPerThread; ++i) {
            const int j = i * T + threadIdx.x;
            if (j < t1 - t0) {
                s_pos[j] = pstage[i];
                if constexpr (PAGED) {  // the page of the row that the gather will read (row 0 if masked)
                    const int pj = pstage[i] >= 0 && pstage[i] < N ? pstage[i] : 0;
                    s_page[j] = p.block_table[(int64_t)bc * p.bt_stride + (pj >> p.page_shift)];
                }
            }
        }
        __syncthreads();
    } else if constexpr (PAGED) {
        const int pages = ((t1 - 1) >> p.page_shift) - first_page + 1;
#pragma unroll
        for (int i = 0; i < kTablePerThread; ++i) {
            const int j = i * T + threadIdx.x;
            if (j < pages) s_page[j] = tstage[i];
        }
        __syncthreads();
    }
    float qf[G][EPL];
#pragma unroll
    for (int i = 0; i < G; ++i) E::unpack(qraw[i], qf[i]);

    const int64_t row_bytes = p.stride_tok * E::kBytes;
    const int64_t head_off =
        ((PAGED ? 0 : (int64_t)bc * p.stride_batch) + (int64_t)(g / p.kv_div) * p.stride_head) * E::kBytes + c * 16;
    const int64_t page_bytes = p.stride_batch * E::kBytes;  // paged only
    const int slot_mask = PAGED ? (1 << p.page_shift) - 1 : 0;
    const char *Kb = (const char *)p.K + head_off;
    const char *Vb = (const char *)p.V + head_off;

    // Fused C.append(k, v) of Alg. 1: the current token's row (index N - 1) comes from k_new /
    // v_new.  Whoever needs that row reads it there instead of from the cache, so nobody depends
    // on the one workgroup per KV head that stores it into the cache.
    const bool append = p.k_new != nullptr;
    const int last = N - 1;
    const int64_t new_off = (((int64_t)b * (p.num_kv_heads / p.kv_div) + g / p.kv_div) * D) * E::kBytes + c * 16;
    const char *Knew = (const char *)p.k_new + new_off, *Vnew = (const char *)p.v_new + new_off;
    if (append && split == 0 && g % p.kv_div == 0 && threadIdx.x < LPR) {
        int64_t dst = (int64_t)last * row_bytes;
        if constexpr (PAGED) {
            const int page = p.block_table[(int64_t)b * p.bt_stride + (last >> p.page_shift)];
            dst = (int64_t)min(max(page, 0), p.num_pages - 1) * page_bytes + (int64_t)(last & slot_mask) * row_bytes;
        }
        *(uint4 *)(const_cast<char *>(Kb) + dst) = *(const uint4 *)Knew;
        *(uint4 *)(const_cast<char *>(Vb) + dst) = *(const uint4 *)Vnew;
    }

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int i = 0; i < G; ++i) {
        m[i] = kEmptyMax;
        l[i] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[i][e] = 0.f;
    }
    const float scale2 = p.scale * kLog2e;

    // Selection layers with one score row per KV head collect the chunk's scores in LDS and write
    // them with one contiguous burst after the loop: writes that trickle out between the
    // streaming reads make HBM switch direction and row all the time (34 us per 16 MiB of
    // scores, measured).  The launch plan keeps such chunks within W * kScoreStagePerWave tokens.
    // The stage shares its LDS with the tail's state buffers, which are used only after it has
    // been written out.
    constexpr int RG = W * TPW;          // row groups per workgroup
    constexpr int GC = G < 4 ? G : 4;    // heads per pass of the tail
    using Tail = TailShared<D, GC, RG, T>;
    // While they sit there they are also binned for the top-k launch that follows (p.topk_rows);
    // the histogram lies behind the stage.
    constexpr size_t kStageBytes = MODE == kSelect ? W * kScoreStagePerWave * sizeof(float) : 0;
    constexpr size_t kHistBytes = MODE == kSelect ? kTopkBins * sizeof(uint32_t) : 0;
    __shared__ __align__(16) char lds_tail[sizeof(Tail) > kStageBytes + kHistBytes ? sizeof(Tail) : kStageBytes + kHistBytes];
    float *s_scores = reinterpret_cast<float *>(lds_tail);
    uint32_t *s_hist = reinterpret_cast<uint32_t *>(lds_tail + kStageBytes);
    const bool per_head = MODE == kSelect && p.select_rule == TD_SELECT_PER_HEAD;
    const bool fused_hist = MODE == kSelect && p.topk_rows != nullptr;  // never with the per-head rule
    if constexpr (MODE == kSelect) {
        if (fused_hist) {
            for (int i = threadIdx.x; i < kTopkBins; i += T) s_hist[i] = 0;
            __syncthreads();
        }
    }

    for (int base = t0 + wave * STEP; base < t1; base += TILE) {
        uint4 kraw[kUnroll], vraw[kUnroll];
        bool valid[kUnroll], fresh[kUnroll];
        int64_t off[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int t = base + u * TPW + r;
            bool ok = t < t1;
            int row, page = 0;
            if constexpr (MODE == kSparse) {
                // lanes beyond the chunk read what the chunk's first entry reads, masked
                const int idx = ok ? t - t0 : 0;
                const int pj = s_pos[idx];
                if constexpr (PAGED) page = s_page[idx];  // of row pj, or of row 0 if pj is not a token
                const bool token = pj >= 0 && pj < N;
                ok = ok && token;
                row = token ? pj : 0;
            } else {
                row = ok ? t : t1 - 1;
                if constexpr (PAGED) page = s_page[(row >> p.page_shift) - first_page];
            }
            valid[u] = ok;
            if constexpr (PAGED)
                off[u] = (int64_t)min(max(page, 0), p.num_pages - 1) * page_bytes + (int64_t)(row & slot_mask) * row_bytes;
            else
                off[u] = (int64_t)row * row_bytes;
            fresh[u] = append && row == last;
            kraw[u] = stream_load16(fresh[u] ? Knew : Kb + off[u]);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) vraw[u] = stream_load16(fresh[u] ? Vnew : Vb + off[u]);
        __builtin_amdgcn_sched_barrier(0);  // every load is issued before the first one is consumed

        float s2[kUnroll][G], gsum[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            float kf[EPL];
            E::unpack(kraw[u], kf);
            gsum[u] = 0.f;
#pragma unroll
            for (int i = 0; i < G; ++i) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) d = fmaf(kf[e], qf[i][e], d);
                d = row_sum<LPR>(d);
                if constexpr (MODE == kSelect) {
                    const float sv = d * p.scale;
                    gsum[u] = p.select_rule == TD_SELECT_GROUP_MAX ? (i ? fmaxf(gsum[u], sv) : sv) : gsum[u] + sv;
                }
                s2[u][i] = valid[u] ? d * scale2 : -INFINITY;
            }
        }
        if constexpr (MODE == kSelect) {
            // every lane of a row holds the row's sums; lane c < kUnroll writes the one of load c,
            // so the wave stores its kUnroll * TPW consecutive scores with one instruction
            static_assert(kUnroll <= LPR, "one writing lane per load");
            const int t = base + c * TPW + r;
            if (!per_head) {
                float mine = gsum[0];
#pragma unroll
                for (int u = 1; u < kUnroll; ++u) mine = c == u ? gsum[u] : mine;
                if (c < kUnroll && t < t1) {
                    s_scores[t - t0] = mine;
                    if (fused_hist) bin_score(s_hist, mine);
                }
            } else {  // one score row per query head: the head's own scaled logits
#pragma unroll
                for (int i = 0; i < G; ++i) {
                    float mine = s2[0][i];
#pragma unroll
                    for (int u = 1; u < kUnroll; ++u) mine = c == u ? s2[u][i] : mine;
                    if (c < kUnroll && t < t1)
                        p.scores[((int64_t)b * p.num_q_heads + g * G + i) * p.score_stride + t] = mine * kLn2;
                }
            }
        }

        float pr[kUnroll][G];
#pragma unroll
        for (int i = 0; i < G; ++i) {
            float mx = m[i];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) mx = fmaxf(mx, s2[u][i]);
            const float alpha = fast_exp2(m[i] - mx);
            m[i] = mx;
            l[i] *= alpha;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[i][e] *= alpha;
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                pr[u][i] = fast_exp2(s2[u][i] - mx);
                l[i] += pr[u][i];
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            float vf[EPL];
            E::unpack(vraw[u], vf);
#pragma unroll
            for (int i = 0; i < G; ++i)
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[i][e] = fmaf(pr[u][i], vf[e], acc[i][e]);
        }
    }

    if constexpr (MODE == kSelect) {
        if (!per_head) {
            write_staged_scores<T>(s_scores, t1 - t0, p.scores + ((int64_t)b * p.num_kv_heads + g) * p.score_stride + t0);
            if (fused_hist) flush_score_histogram<T>(p.topk_rows + (b * p.num_kv_heads + g), s_hist, split == 0);
            __syncthreads();  // the stage has been read; its LDS now takes the states
        }
    }

    // ---- merge the online-softmax states of the workgroup's row groups through LDS,
    // at most four heads at a time to bound the LDS footprint
    Tail &sm = *reinterpret_cast<Tail *>(lds_tail);
    const int rg = wave * TPW + r;
#pragma unroll
    for (int h0 = 0; h0 < G; h0 += GC) {
        if (h0) __syncthreads();
#pragma unroll
        for (int i = 0; i < GC; ++i) {
#pragma unroll
            for (int e = 0; e < EPL; e += 4)
                *reinterpret_cast<float4 *>(&sm.acc[(rg * GC + i) * D + c * EPL + e]) =
                    make_float4(acc[h0 + i][e], acc[h0 + i][e + 1], acc[h0 + i][e + 2], acc[h0 + i][e + 3]);
            if (c == 0) {
                sm.m[rg][i] = m[h0 + i];
                sm.l[rg][i] = l[h0 + i];
            }
        }
        __syncthreads();
        fold_states<DT, D, G, GC, RG, T>(p, sm, b, g, split, ns, h0);
    }
    if (ns == 1 || p.separate_merge) return;
    finish_chunks<DT, D, G, GC, RG, T>(p, sm, b, g, ns);
}

template <int DT, int D, int G, int W, bool PAGED>
hipError_t launch_mode(int mode, const AttendParams &p, hipStream_t stream) {
    const dim3 grid(p.num_splits, p.num_kv_heads, p.batch), block(W * kWave);
    switch (mode) {
    case kDense:
        hipLaunchKernelGGL((attend_split_kernel<DT, D, G, kDense, W, PAGED>), grid, block, 0, stream, p);
        break;
    case kSelect:
        hipLaunchKernelGGL((attend_split_kernel<DT, D, G, kSelect, W, PAGED>), grid, block, 0, stream, p);
        break;
    default:
        hipLaunchKernelGGL((attend_split_kernel<DT, D, G, kSparse, W, PAGED>), grid, block, 0, stream, p);
        break;
    }
    return hipGetLastError();
}

template <int DT, int D, int G, int W>
hipError_t launch_paged(int mode, const AttendParams &p, hipStream_t stream) {
    return p.block_table ? launch_mode<DT, D, G, W, true>(mode, p, stream)
                         : launch_mode<DT, D, G, W, false>(mode, p, stream);
}

template <int DT, int D, int G>
hipError_t launch_waves(int waves, int mode, const AttendParams &p, hipStream_t stream) {
    if (waves == 8) return launch_paged<DT, D, G, 8>(mode, p, stream);
    return launch_paged<DT, D, G, 4>(mode, p, stream);
}

template <int DT, int D>
hipError_t launch_group(int group, int waves, int mode, const AttendParams &p, hipStream_t stream) {
    switch (group) {
    case 1: return launch_waves<DT, D, 1>(waves, mode, p, stream);
    case 2: return launch_waves<DT, D, 2>(waves, mode, p, stream);
    case 4: return launch_waves<DT, D, 4>(waves, mode, p, stream);
    case 8: return launch_waves<DT, D, 8>(waves, mode, p, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool attend_supports_waves(int group, int waves) { return (waves == 4 || waves == 8) && group >= 1; }

hipError_t launch_attend(int dtype, int head_dim, int group, int waves, int mode, const AttendParams &p,
                         hipStream_t stream) {
    if (!attend_supports_waves(group, waves)) return hipErrorInvalidValue;
    if (dtype == TD_BF16 && head_dim == 128) return launch_group<TD_BF16, 128>(group, waves, mode, p, stream);
    if (dtype == TD_BF16 && head_dim == 64) return launch_group<TD_BF16, 64>(group, waves, mode, p, stream);
    if (dtype == TD_F32 && head_dim == 128) return launch_group<TD_F32, 128>(group, waves, mode, p, stream);
    if (dtype == TD_F32 && head_dim == 64) return launch_group<TD_F32, 64>(group, waves, mode, p, stream);
    return hipErrorInvalidValue;
}

}  // namespace tidal
