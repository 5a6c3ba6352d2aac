// Decode attention for bf16 caches with head_dim 128 on the gfx950 matrix cores.
//
// Same decomposition and the same tail as attend.hip (one workgroup per chunk of consecutive
// tokens of a (sequence, KV head), all G query heads of the group served from one fetch of K
// and V, partials + ticket + last-chunk merge), but both contractions of Eq. 1 run on MFMA so
// that the vector ALU only does the softmax bookkeeping, and the instruction count does not
// grow with G (a 16-row tile holds up to 16 heads).  With G = 4 the plain VALU kernel spends
// ~140 vector instructions per 2 KiB of K+V fetched, about 60 % of the issue slots at HBM
// speed, and still wins; with G = 8 it is bound by its arithmetic and this kernel is faster.
//
// A wave handles 16 tokens per iteration, lane = (n16 = lane % 16, kb = lane / 16):
//   S^T = K Q^T   4 x v_mfma_f32_16x16x32_bf16.  A = K tile: lane (n16, kb) loads 16 bytes of
//                 token n16 at d-octet 4s + kb (step s), exactly the A-operand layout, so K
//                 goes from memory to the matrix core untouched.  B = Q^T, loaded once
//                 (rows >= G are zero).  Result: lane (n16, kb) holds the logits of head n16
//                 for tokens 4kb .. 4kb+3 - already the A-operand layout of the second product.
//   softmax       per lane on those 4 logits; the tile maximum of a head is reduced over the
//                 four kb lanes with two cross-row shuffles; running max and sum per lane.
//   O += P V      16 x v_mfma_f32_16x16x16_bf16 (8 channel groups x {hi, lo}): P is split into
//                 two bf16 parts so that its rounding (2^-17) stays far below the tolerance.
//                 B = V: lane (n16, kb) loads 16 bytes of tokens 4kb+u (u = 0..3) at octet n16
//                 (whole 256-byte rows, coalesced) and builds, with byte permutes, for channel
//                 8 n16 + e the 4-token column the B operand wants; channel group e is the set
//                 {8 c + e}, which the matrix core does not care about.  No LDS in the loop.
//   The accumulators of head 4kb + i, channel 8 n16 + e live in lane (n16, kb), acc[e][i].
#include "attend_tail.h"
#include "mfma_util.h"

namespace tidal {
namespace {

constexpr int kD = 128;
constexpr int kWaveTokens = 16;  // tokens per wave per iteration

// W wave64s per workgroup (4 or 8) and PAGED as in attend.hip.  A sparse layer is one short
// burst per wave, so with four waves a wave takes two 16-token tiles per iteration (all 16 row
// loads in flight at once); full and selection layers, and eight-wave sparse layers, take one.
template <int G, int MODE, int W, bool PAGED>
__global__ __launch_bounds__(W *kWave) __attribute__((amdgpu_waves_per_eu(MODE != kSparse ? 4 : 1)))
void attend_mfma_kernel(const AttendParams p) {
    constexpr int T = W * kWave;
    constexpr int kTiles = MODE == kSparse && W == 4 ? 2 : 1;
    constexpr int STEP = kTiles * kWaveTokens;  // tokens per wave per iteration
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int n16 = lane & 15, kb = lane >> 4;

    const int t0 = split * p.chunk;

    // Loads that depend on the launch arguments only, issued ahead of the read of the sequence
    // length: Q^T as B operand (lane (n16 = head, kb) holds d-octet 4s + kb of head n16), the
    // chunk's positions (sparse) or block-table entries (paged full / selection layers).
    bf16x8 qfrag[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (n16 < G)
            v = *reinterpret_cast<const uint4 *>(static_cast<const char *>(p.q) +
                                                 (((int64_t)b * p.num_q_heads + g * G + n16) * kD + (4 * s + kb) * 8) * 2);
        qfrag[s] = __builtin_bit_cast(bf16x8, v);
    }
    constexpr int kPosPerThread = MODE == kSparse ? kSparseChunkMax / T : 1;
    int pstage[kPosPerThread];
    if constexpr (MODE == kSparse) {
        const int32_t *pos = p.positions + ((int64_t)b * p.num_kv_heads + g) * p.k;
        const int len = min(p.k - t0, p.chunk);
#pragma unroll
        for (int i = 0; i < kPosPerThread; ++i) {
            const int j = i * T + threadIdx.x;
            pstage[i] = i * T < len ? pos[t0 + min(j, len - 1)] : -1;  // workgroup-uniform condition
        }
    }
    constexpr bool kStageTable = PAGED && MODE != kSparse;
    constexpr int kTablePerThread = kStageTable ? kPageStageMax / T : 1;
    int tstage[kTablePerThread];
    const int first_page = PAGED ? t0 >> p.page_shift : 0;
    if constexpr (kStageTable) {
        const int32_t *table = p.block_table + (int64_t)b * p.bt_stride + first_page;
        const int pages = ((min(p.max_seq_len, t0 + p.chunk) - 1) >> p.page_shift) - first_page + 1;
#pragma unroll
        for (int i = 0; i < kTablePerThread; ++i) {
            const int j = i * T + threadIdx.x;
            tstage[i] = i * T < pages ? table[min(j, pages - 1)] : 0;
        }
    }
    asm volatile("" ::: "memory");  // the loads above stay above the branch on the sequence length

    const int N = min(max(p.seq_lens[b], 0), p.max_seq_len);
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
                    s_page[j] = p.block_table[(int64_t)b * p.bt_stride + (pj >> p.page_shift)];
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

    const int64_t row_bytes = p.stride_tok * 2;
    const int64_t head_off = ((PAGED ? 0 : (int64_t)b * p.stride_batch) + (int64_t)(g / p.kv_div) * p.stride_head) * 2;
    const int64_t page_bytes = p.stride_batch * 2;  // paged only
    const int slot_mask = PAGED ? (1 << p.page_shift) - 1 : 0;
    const char *Kb = static_cast<const char *>(p.K) + head_off + kb * 16;   // + 64 s per step
    const char *Vb = static_cast<const char *>(p.V) + head_off + n16 * 16;
    float *score_row = nullptr;  // of the KV head, or of the group's first query head (per-head rule)
    if constexpr (MODE == kSelect)
        score_row = p.scores + (p.select_rule == TD_SELECT_PER_HEAD ? (int64_t)b * p.num_q_heads + g * G
                                                                    : (int64_t)b * p.num_kv_heads + g) * p.score_stride;

    // Where the row for slot t of the chunk lives (byte offset inside the head's cache); lanes
    // beyond the chunk, and positions that are no token, read a row that exists and are masked.
    // Fused C.append(k, v) of Alg. 1: the current token's row (index N - 1) comes from k_new /
    // v_new.  Whoever needs that row reads it there instead of from the cache, so nobody depends
    // on the one workgroup per KV head that stores it into the cache.
    const bool append = p.k_new != nullptr;
    const int last = N - 1;
    const int64_t new_off = (((int64_t)b * (p.num_kv_heads / p.kv_div) + g / p.kv_div) * kD) * 2;
    const char *Knew = static_cast<const char *>(p.k_new) + new_off + kb * 16;
    const char *Vnew = static_cast<const char *>(p.v_new) + new_off + n16 * 16;
    if (append && split == 0 && g % p.kv_div == 0 && threadIdx.x < 16) {
        int64_t dst = (int64_t)last * row_bytes;
        if constexpr (PAGED) {
            const int page = p.block_table[(int64_t)b * p.bt_stride + (last >> p.page_shift)];
            dst = (int64_t)min(max(page, 0), p.num_pages - 1) * page_bytes + (int64_t)(last & slot_mask) * row_bytes;
        }
        *reinterpret_cast<uint4 *>(const_cast<char *>(Vb) + dst) = *reinterpret_cast<const uint4 *>(Vnew);
        *reinterpret_cast<uint4 *>(static_cast<char *>(const_cast<void *>(p.K)) + head_off + n16 * 16 + dst) =
            *reinterpret_cast<const uint4 *>(static_cast<const char *>(p.k_new) + new_off + n16 * 16);
    }

    auto locate = [&](int t, bool &ok, int &row) -> int64_t {
        ok = t < t1;
        int page = 0;
        if constexpr (MODE == kSparse) {
            const int idx = ok ? t - t0 : 0;
            const int pj = s_pos[idx];
            if constexpr (PAGED) page = s_page[idx];
            const bool token = pj >= 0 && pj < N;
            ok = ok && token;
            row = token ? pj : 0;
        } else {
            row = ok ? t : t1 - 1;
            if constexpr (PAGED) page = s_page[(row >> p.page_shift) - first_page];
        }
        if constexpr (PAGED)
            return (int64_t)min(max(page, 0), p.num_pages - 1) * page_bytes + (int64_t)(row & slot_mask) * row_bytes;
        else
            return (int64_t)row * row_bytes;
    };

    float m_run = kEmptyMax, l_run = 0.f;  // head n16, the same in the four kb lanes
    f32x4 acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
    const float scale2 = p.scale * kLog2e;

    // Selection layers with one score row per KV head collect the chunk's scores in LDS and write
    // them with one contiguous burst after the loop: writes that trickle out between the
    // streaming reads make HBM switch direction and row all the time (34 us per 16 MiB of
    // scores, measured).  The launch plan keeps such chunks within W * kScoreStagePerWave tokens.
    // While they sit there they are also binned for the top-k launch that follows (p.topk_rows).
    // Stage and histogram share their LDS with the tail's state buffers, which are used only
    // after both have been read.
    constexpr int RG = W;
    using Tail = TailShared<kD, G, RG, T>;
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

    for (int base = t0 + wave * STEP; base < t1; base += W * STEP) {
        uint4 kraw[kTiles][4], vraw[kTiles][4];
        bool valid[kTiles][4];
        int tok[kTiles][4];
#pragma unroll
        for (int x = 0; x < kTiles; ++x) {
            // K: token base + 16x + n16
            bool okk;
            int rowk;
            const int64_t koff = locate(base + kWaveTokens * x + n16, okk, rowk);
            const char *kp = append && rowk == last ? Knew : Kb + koff;
#pragma unroll
            for (int s = 0; s < 4; ++s) kraw[x][s] = stream_load16(kp + 64 * s);
            // V: tokens base + 16x + 4kb + u; their validity is also the validity of this lane's logits
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t voff = locate(base + kWaveTokens * x + 4 * kb + u, valid[x][u], tok[x][u]);
                vraw[x][u] = stream_load16(append && tok[x][u] == last ? Vnew : Vb + voff);
            }
        }
        __builtin_amdgcn_sched_barrier(0);  // every load is issued before the first one is consumed

#pragma unroll
        for (int x = 0; x < kTiles; ++x) {
            f32x4 st = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s)
                st = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kraw[x][s]), qfrag[s], st, 0, 0, 0);

            if constexpr (MODE == kSelect) {
                // per token, the group's scaled logits sit in lanes n16 = 0..G-1 of a 16-lane row
                // (lanes >= G hold zeros): their sum, their maximum, or each head's own value
                float gs[4];
                if (p.select_rule == TD_SELECT_GROUP_MAX) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        gs[i] = n16 < G ? st[i] * p.scale : -INFINITY;
                        gs[i] = fmaxf(gs[i], dpp_f<0xB1>(gs[i]));                       // quad_perm [1,0,3,2]
                        gs[i] = fmaxf(gs[i], dpp_f<0x4E>(gs[i]));                       // quad_perm [2,3,0,1]
                        if constexpr (G > 4) gs[i] = fmaxf(gs[i], dpp_f<0x141>(gs[i])); // row_half_mirror
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        gs[i] = st[i] * p.scale;
                        if (!per_head) {
                            gs[i] += dpp_f<0xB1>(gs[i]);
                            gs[i] += dpp_f<0x4E>(gs[i]);
                            if constexpr (G > 4) gs[i] += dpp_f<0x141>(gs[i]);
                        }
                    }
                }
                // lane (head, kb) holds the values of the four consecutive tokens base + 4kb ..
                if (!per_head) {
                    if (n16 == 0 && valid[x][0]) {  // a lane's valid tokens are a prefix of its four
                        if (valid[x][3]) {
                            *reinterpret_cast<float4 *>(&s_scores[tok[x][0] - t0]) = make_float4(gs[0], gs[1], gs[2], gs[3]);
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (valid[x][i]) s_scores[tok[x][i] - t0] = gs[i];
                        }
                    }
                    // every lane of a quad holds the four reduced values: lane i of the first quad bins token i
                    if (fused_hist && n16 < 4) {
                        const float mine = n16 == 0 ? gs[0] : n16 == 1 ? gs[1] : n16 == 2 ? gs[2] : gs[3];
                        const bool ok = n16 == 0 ? valid[x][0] : n16 == 1 ? valid[x][1] : n16 == 2 ? valid[x][2] : valid[x][3];
                        if (ok) bin_score(s_hist, mine);
                    }
                } else if (n16 < G) {  // one 16-byte store per head where the row allows it
                    float *dst = score_row + (int64_t)n16 * p.score_stride + tok[x][0];
                    if (valid[x][3] && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
                        *reinterpret_cast<float4 *>(dst) = make_float4(gs[0], gs[1], gs[2], gs[3]);
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (valid[x][i]) dst[tok[x][i] - tok[x][0]] = gs[i];
                    }
                }
            }

            float s2[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) s2[i] = valid[x][i] ? st[i] * scale2 : -INFINITY;
            float tm = fmaxf(fmaxf(s2[0], s2[1]), fmaxf(s2[2], s2[3]));
            tm = cross_rows_max(tm);
            const float m_new = fmaxf(m_run, tm);
            const float alpha = fast_exp2(m_run - m_new);
            float pr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) pr[i] = fast_exp2(s2[i] - m_new);
            l_run = l_run * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3]));
            if (__any(m_new != m_run)) {  // some head's maximum moved: rescale its accumulators
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float a = __shfl(alpha, 4 * kb + i);  // head 4kb + i keeps its state in lane 4kb + i
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[e][i] *= a;
                }
            }
            m_run = m_new;

            // P (tokens 4kb .. 4kb+3 of head n16) as two bf16 parts
            uint32_t ph[4], pl[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ph[i] = __float_as_uint(pr[i]) & 0xffff0000u;
                pl[i] = __float_as_uint(pr[i] - __uint_as_float(ph[i]));
            }
            const s16x4 p_hi = pack_pairs(ph[1], ph[0], ph[3], ph[2], kHighHalves);
            const s16x4 p_lo = pack_pairs(pl[1], pl[0], pl[3], pl[2], kHighHalves);
            const uint32_t vw[4][4] = {{vraw[x][0].x, vraw[x][0].y, vraw[x][0].z, vraw[x][0].w},
                                       {vraw[x][1].x, vraw[x][1].y, vraw[x][1].z, vraw[x][1].w},
                                       {vraw[x][2].x, vraw[x][2].y, vraw[x][2].z, vraw[x][2].w},
                                       {vraw[x][3].x, vraw[x][3].y, vraw[x][3].z, vraw[x][3].w}};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t sel = (e & 1) ? kHighHalves : kLowHalves;
                const s16x4 vf = pack_pairs(vw[1][e >> 1], vw[0][e >> 1], vw[3][e >> 1], vw[2][e >> 1], sel);
                acc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_hi, vf, acc[e], 0, 0, 0);
                acc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_lo, vf, acc[e], 0, 0, 0);
            }
        }
    }

    if constexpr (MODE == kSelect) {
        if (!per_head) {
            write_staged_scores<T>(s_scores, t1 - t0, score_row + t0);
            if (fused_hist) flush_score_histogram<T>(p.topk_rows + (b * p.num_kv_heads + g), s_hist, split == 0);
            __syncthreads();  // stage and histogram have been read; their LDS now takes the states
        }
    }

    // ---- one state per wave into LDS, then the common tail
    l_run = cross_rows_sum(l_run);
    Tail &sm = *reinterpret_cast<Tail *>(lds_tail);
    if (kb == 0 && n16 < G) {
        sm.m[wave][n16] = m_run;
        sm.l[wave][n16] = l_run;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int h = 4 * kb + i;
        if (h < G) {
            float *dst = &sm.acc[(wave * G + h) * kD + 8 * n16];
            *reinterpret_cast<float4 *>(dst) = make_float4(acc[0][i], acc[1][i], acc[2][i], acc[3][i]);
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(acc[4][i], acc[5][i], acc[6][i], acc[7][i]);
        }
    }
    __syncthreads();
    fold_states<TD_BF16, kD, G, G, RG, T>(p, sm, b, g, split, ns, 0);
    if (ns == 1 || p.separate_merge) return;
    finish_chunks<TD_BF16, kD, G, G, RG, T>(p, sm, b, g, ns);
}

template <int G, int W, bool PAGED>
hipError_t launch_mfma_mode(int mode, const AttendParams &p, hipStream_t stream) {
    const dim3 grid(p.num_splits, p.num_kv_heads, p.batch), block(W * kWave);
    switch (mode) {
    case kDense:
        hipLaunchKernelGGL((attend_mfma_kernel<G, kDense, W, PAGED>), grid, block, 0, stream, p);
        break;
    case kSelect:
        hipLaunchKernelGGL((attend_mfma_kernel<G, kSelect, W, PAGED>), grid, block, 0, stream, p);
        break;
    default:
        hipLaunchKernelGGL((attend_mfma_kernel<G, kSparse, W, PAGED>), grid, block, 0, stream, p);
        break;
    }
    return hipGetLastError();
}

template <int G>
hipError_t launch_mfma_group(int waves, int mode, const AttendParams &p, hipStream_t stream) {
    if (waves == 8)
        return p.block_table ? launch_mfma_mode<G, 8, true>(mode, p, stream) : launch_mfma_mode<G, 8, false>(mode, p, stream);
    return p.block_table ? launch_mfma_mode<G, 4, true>(mode, p, stream) : launch_mfma_mode<G, 4, false>(mode, p, stream);
}

}  // namespace

hipError_t launch_attend_mfma(int group, int waves, int mode, const AttendParams &p, hipStream_t stream) {
    if (waves != 4 && waves != 8) return hipErrorInvalidValue;
    switch (group) {
    case 1: return launch_mfma_group<1>(waves, mode, p, stream);
    case 2: return launch_mfma_group<2>(waves, mode, p, stream);
    case 4: return launch_mfma_group<4>(waves, mode, p, stream);
    case 8: return launch_mfma_group<8>(waves, mode, p, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tidal
