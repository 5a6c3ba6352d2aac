// Decode attention for bf16 caches with head_dim 128 on the gfx950 matrix cores.
//
// Same decomposition and the same tail as attend.hip (one workgroup of four wave64s per chunk
// of consecutive tokens of a (sequence, KV head), all G query heads of the group served from
// one fetch of K and V, partials + ticket + last-chunk merge), but both contractions of Eq. 1
// run on MFMA so that the vector ALU only does the softmax bookkeeping.  With G = 4 the plain
// VALU kernel spends ~140 vector instructions per 2 KiB of K+V fetched, which is about 60 %
// of the issue slots at HBM speed; here it is ~70 per 8 KiB.
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

namespace tidal {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kWaveTokens = 16;  // tokens per wave per iteration

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

__device__ __forceinline__ s16x4 pack_pairs(uint32_t a1, uint32_t a0, uint32_t b1, uint32_t b0, uint32_t sel) {
    const uint32_t d0 = __builtin_amdgcn_perm(a1, a0, sel), d1 = __builtin_amdgcn_perm(b1, b0, sel);
    return __builtin_bit_cast(s16x4, make_uint2(d0, d1));
}

constexpr uint32_t kLowHalves = 0x05040100u;   // (x1.lo16 << 16) | x0.lo16
constexpr uint32_t kHighHalves = 0x07060302u;  // (x1.hi16 << 16) | x0.hi16

template <int G, int MODE>
__global__ __launch_bounds__(kThreads) void attend_mfma_kernel(const AttendParams p) {
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int n16 = lane & 15, kb = lane >> 4;

    if constexpr (MODE == kSelect) {  // leave the row's top-k state clear for the kernels that follow
        TopkRow *row = static_cast<TopkRow *>(p.topk_scratch) + (b * p.num_kv_heads + g);
        for (int i = split * kThreads + threadIdx.x; i < kTopkBins; i += p.num_splits * kThreads) row->hist[i] = 0;
        if (split == 0 && threadIdx.x == 0) row->ncand = 0;
    }
    const int N = min(max(p.seq_lens[b], 0), p.max_seq_len);
    const int n_tok = MODE == kSparse ? (N > 0 ? p.k : 0) : N;
    const int t0 = split * p.chunk;
    if (t0 >= n_tok) return;
    const int t1 = min(n_tok, t0 + p.chunk);
    const int ns = (n_tok + p.chunk - 1) / p.chunk;  // workgroups of this (sequence, KV head) with work

    __shared__ int s_pos[MODE == kSparse ? kSparseChunkMax : 1];
    if constexpr (MODE == kSparse) {
        const int32_t *pos = p.positions + ((int64_t)b * p.num_kv_heads + g) * p.k;
        for (int i = threadIdx.x; i < t1 - t0; i += kThreads) s_pos[i] = pos[t0 + i];
        __syncthreads();
    }

    // Q^T as B operand: lane (n16 = head, kb) holds d-octet 4s + kb of head n16
    bf16x8 qfrag[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (n16 < G)
            v = *reinterpret_cast<const uint4 *>(static_cast<const char *>(p.q) +
                                                 (((int64_t)b * p.num_q_heads + g * G + n16) * kD + (4 * s + kb) * 8) * 2);
        qfrag[s] = __builtin_bit_cast(bf16x8, v);
    }

    const int64_t row_bytes = p.stride_tok * 2;
    const int64_t head_off = ((int64_t)b * p.stride_batch + (int64_t)g * p.stride_head) * 2;
    const char *Kb = static_cast<const char *>(p.K) + head_off + kb * 16;   // + 64 s per step
    const char *Vb = static_cast<const char *>(p.V) + head_off + n16 * 16;
    float *score_row = MODE == kSelect ? p.scores + ((int64_t)b * p.num_kv_heads + g) * p.score_stride : nullptr;

    float m_run = kEmptyMax, l_run = 0.f;  // head n16, the same in the four kb lanes
    f32x4 acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
    const float scale2 = p.scale * kLog2e;

    for (int base = t0 + wave * kWaveTokens; base < t1; base += kWavesPerGroup * kWaveTokens) {
        // K: token base + n16
        int rowk;
        {
            const int t = base + n16;
            bool ok = t < t1;
            if constexpr (MODE == kSparse) {
                const int pj = ok ? s_pos[t - t0] : -1;
                ok = pj >= 0 && pj < N;
                rowk = ok ? pj : 0;
            } else {
                rowk = ok ? t : t1 - 1;
            }
        }
        const char *kp = Kb + (int64_t)rowk * row_bytes;
        uint4 kraw[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) kraw[s] = stream_load16(kp + 64 * s);
        // V: tokens base + 4kb + u; their validity is also the validity of this lane's logits
        uint4 vraw[4];
        bool valid[4];
        int tok[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = base + 4 * kb + u;
            bool ok = t < t1;
            int row;
            if constexpr (MODE == kSparse) {
                const int pj = ok ? s_pos[t - t0] : -1;
                ok = pj >= 0 && pj < N;
                row = ok ? pj : 0;
            } else {
                row = ok ? t : t1 - 1;
            }
            valid[u] = ok;
            tok[u] = row;
            vraw[u] = stream_load16(Vb + (int64_t)row * row_bytes);
        }

        f32x4 st = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 4; ++s)
            st = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kraw[s]), qfrag[s], st, 0, 0, 0);

        if constexpr (MODE == kSelect) {
            // sum of the group's scaled logits per token: heads sit in lanes n16 = 0..G-1 of a
            // 16-lane row (lanes >= G hold zeros)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float gs = st[i] * p.scale;
                gs += dpp_f<0xB1>(gs);                       // quad_perm [1,0,3,2]
                gs += dpp_f<0x4E>(gs);                       // quad_perm [2,3,0,1]
                if constexpr (G > 4) gs += dpp_f<0x141>(gs); // row_half_mirror
                if (n16 == 0 && valid[i]) score_row[tok[i]] = gs;
            }
        }

        float s2[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) s2[i] = valid[i] ? st[i] * scale2 : -INFINITY;
        float tm = fmaxf(fmaxf(s2[0], s2[1]), fmaxf(s2[2], s2[3]));
        tm = fmaxf(tm, __shfl_xor(tm, 16));
        tm = fmaxf(tm, __shfl_xor(tm, 32));
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
        const uint32_t vw[4][4] = {{vraw[0].x, vraw[0].y, vraw[0].z, vraw[0].w},
                                   {vraw[1].x, vraw[1].y, vraw[1].z, vraw[1].w},
                                   {vraw[2].x, vraw[2].y, vraw[2].z, vraw[2].w},
                                   {vraw[3].x, vraw[3].y, vraw[3].z, vraw[3].w}};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t sel = (e & 1) ? kHighHalves : kLowHalves;
            const s16x4 vf = pack_pairs(vw[1][e >> 1], vw[0][e >> 1], vw[3][e >> 1], vw[2][e >> 1], sel);
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_hi, vf, acc[e], 0, 0, 0);
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_lo, vf, acc[e], 0, 0, 0);
        }
    }

    // ---- one state per wave into LDS, then the common tail
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    constexpr int RG = kWavesPerGroup;
    __shared__ TailShared<kD, G, RG, kThreads> sm;
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
    fold_states<TD_BF16, kD, G, G, RG, kThreads>(p, sm, b, g, split, ns, 0);
    if (ns == 1) return;
    finish_chunks<TD_BF16, kD, G, G, RG, kThreads>(p, sm, b, g, ns);
}

template <int G>
hipError_t launch_mfma_mode(int mode, const AttendParams &p, hipStream_t stream) {
    const dim3 grid(p.num_splits, p.num_kv_heads, p.batch), block(kThreads);
    switch (mode) {
    case kDense:
        hipLaunchKernelGGL((attend_mfma_kernel<G, kDense>), grid, block, 0, stream, p);
        break;
    case kSelect:
        hipLaunchKernelGGL((attend_mfma_kernel<G, kSelect>), grid, block, 0, stream, p);
        break;
    default:
        hipLaunchKernelGGL((attend_mfma_kernel<G, kSparse>), grid, block, 0, stream, p);
        break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attend_mfma(int group, int mode, const AttendParams &p, hipStream_t stream) {
    switch (group) {
    case 1: return launch_mfma_mode<1>(mode, p, stream);
    case 2: return launch_mfma_mode<2>(mode, p, stream);
    case 4: return launch_mfma_mode<4>(mode, p, stream);
    case 8: return launch_mfma_mode<8>(mode, p, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tidal
