// Attention of a prefill over the last P tokens of every sequence (the cache-correction step of
// Sec. 3.2 re-runs full attention for the tokens that were decoded sparsely): token j sits at
// position N - P + j and attends, with Eq. 1, to the positions up to its own.  bf16, head_dim 128,
// contiguous cache.
//
// The query rows of a KV head are the (token, head) pairs, row = token * G + head.  A workgroup
// of four wave64s takes R * 16 consecutive rows and streams the cache once for all of them, up to
// the last position any of its rows may see; the waves split the tokens (16-token tiles,
// interleaved) and every wave keeps an online-softmax state for all R * 16 rows, so a K or V tile
// is loaded once per wave and used by R row tiles.  The tile arithmetic is that of
// attend_mfma.hip: S^T = K Q^T with v_mfma_f32_16x16x32_bf16 (K from memory straight into the A
// operand), O += P V with v_mfma_f32_16x16x16_bf16 - here with P rounded to bf16 once, as prefill
// kernels commonly do - and per-row causal masks on the logits.  The four waves' states are
// folded through LDS, one row tile at a time, and the rows are written out; there is no split
// across workgroups, so no partials and no workspace.
//
// Per 16-token tile and wave: 8 loads of 16 bytes per lane, R * 12 MFMAs (R * 98304 flop) and
// about 60 + R * 45 vector instructions, so for R = 4 the vector ALU, not the matrix core, sets
// the pace: at best ~40 % of the MFMA peak.
#include "attend_tail.h"
#include "mfma_util.h"

namespace tidal {
namespace {

constexpr int kPD = 128;
constexpr int kPWaves = 4;
constexpr int kPThreads = kPWaves * kWave;

template <int G, int R>
__global__ __launch_bounds__(kPThreads) void prefill_mfma_kernel(const PrefillParams p) {
    // Workgroups are handed to the eight XCDs round-robin by their linear index.  The row blocks of
    // one (sequence, KV head) stream the same keys and values at about the same pace, so they
    // should share an L2: with a multiple of eight (sequence, KV head) pairs, the linear index is
    // unpacked pair-first, and all row blocks of a pair land on XCD (pair % 8).
    const int pairs = p.num_kv_heads * p.batch;
    int rb, pair;
    if (pairs % 8 == 0) {
        pair = blockIdx.x % pairs;
        rb = blockIdx.x / pairs;
    } else {
        rb = blockIdx.x % p.row_blocks;
        pair = blockIdx.x / p.row_blocks;
    }
    const int g = pair % p.num_kv_heads, b = pair / p.num_kv_heads;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int n16 = lane & 15, kb = lane >> 4;
    const int P = p.num_new, rows_total = P * G, row0 = rb * (16 * R);

    // Q^T fragments: lane (n16, kb) holds d-octet 4s + kb of row row0 + 16r + n16; rows beyond the
    // last one are zero and never written
    bf16x8 qfrag[R][4];
    int tkn[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int row = row0 + 16 * r + n16;
        tkn[r] = row / G;
        const int head = row - tkn[r] * G;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (row < rows_total)
                v = *reinterpret_cast<const uint4 *>(
                    static_cast<const char *>(p.q) +
                    ((((int64_t)b * P + tkn[r]) * p.num_q_heads + g * G + head) * kPD + (4 * s + kb) * 8) * 2);
            qfrag[r][s] = __builtin_bit_cast(bf16x8, v);
        }
    }
    asm volatile("" ::: "memory");  // the loads above are issued before the sequence length is needed

    const int N = min(max(p.seq_lens[b], 0), p.max_seq_len);
    // row (tile r, n16) sees tokens t < limit[r]; a token before the start of the cache sees none
    int limit[R];
#pragma unroll
    for (int r = 0; r < R; ++r) limit[r] = row0 + 16 * r + n16 < rows_total ? max(N - P + tkn[r] + 1, 0) : 0;
    const int last_tkn = min(P - 1, (row0 + 16 * R - 1) / G);
    const int t_end = max(N - P + last_tkn + 1, 0);  // tokens this workgroup streams

    const int64_t row_bytes = p.stride_tok * 2;
    const int64_t head_off = ((int64_t)b * p.stride_batch + (int64_t)g * p.stride_head) * 2;
    const char *Kb = static_cast<const char *>(p.K) + head_off + kb * 16;  // + 64 s per step
    const char *Vb = static_cast<const char *>(p.V) + head_off + n16 * 16;

    float m_run[R], l_run[R];
    f32x4 acc[R][8];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        m_run[r] = kEmptyMax;
        l_run[r] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float scale2 = p.scale * kLog2e;

    // K: token base + n16; V: tokens base + 4kb + u.  Lanes beyond the streamed range read its last
    // row and are masked by the rows' limits.  The next tile's loads are issued before the current
    // tile is consumed (one wave per SIMD fits the registers, so nothing else hides the latency).
    auto load_tile = [&](int base, uint4 (&kr)[4], uint4 (&vr)[4]) {
        const char *kp = Kb + (int64_t)min(base + n16, t_end - 1) * row_bytes;
#pragma unroll
        for (int s = 0; s < 4; ++s) kr[s] = stream_load16(kp + 64 * s);
#pragma unroll
        for (int u = 0; u < 4; ++u) vr[u] = stream_load16(Vb + (int64_t)min(base + 4 * kb + u, t_end - 1) * row_bytes);
    };
    uint4 kraw[4], vraw[4];
    if (wave * 16 < t_end) load_tile(wave * 16, kraw, vraw);
    for (int base = wave * 16; base < t_end; base += kPWaves * 16) {
        uint4 knext[4], vnext[4];
        const bool more = base + kPWaves * 16 < t_end;
        if (more) load_tile(base + kPWaves * 16, knext, vnext);
        __builtin_amdgcn_sched_barrier(0);  // the next tile's loads are issued before this tile is consumed

        // V as B operand: for channel group e the 4-token column of channels {8 c + e}
        s16x4 vf[8];
        {
            const uint32_t vw[4][4] = {{vraw[0].x, vraw[0].y, vraw[0].z, vraw[0].w},
                                       {vraw[1].x, vraw[1].y, vraw[1].z, vraw[1].w},
                                       {vraw[2].x, vraw[2].y, vraw[2].z, vraw[2].w},
                                       {vraw[3].x, vraw[3].y, vraw[3].z, vraw[3].w}};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                vf[e] = pack_pairs(vw[1][e >> 1], vw[0][e >> 1], vw[3][e >> 1], vw[2][e >> 1],
                                   (e & 1) ? kHighHalves : kLowHalves);
        }
        const int t_lane = base + 4 * kb;  // this lane's logits are for tokens t_lane .. t_lane + 3
#pragma unroll
        for (int r = 0; r < R; ++r) {
            f32x4 st = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s)
                st = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kraw[s]), qfrag[r][s], st, 0, 0, 0);
            float s2[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) s2[i] = t_lane + i < limit[r] ? st[i] * scale2 : -INFINITY;
            float tm = fmaxf(fmaxf(s2[0], s2[1]), fmaxf(s2[2], s2[3]));
            tm = cross_rows_max(tm);
            const float m_new = fmaxf(m_run[r], tm);
            const float alpha = fast_exp2(m_run[r] - m_new);
            float pr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) pr[i] = fast_exp2(s2[i] - m_new);
            l_run[r] = l_run[r] * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3]));
            if (__any(m_new != m_run[r])) {  // some row's maximum moved: rescale its accumulators
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float a = __shfl(alpha, 4 * kb + i);  // row 4kb + i keeps its state in lane 4kb + i
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[r][e][i] *= a;
                }
            }
            m_run[r] = m_new;
            // P (tokens 4kb .. 4kb+3 of row n16), rounded to bf16 (half up on the magnitude)
            uint32_t ph[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) ph[i] = __float_as_uint(pr[i]) + 0x8000u;
            const s16x4 pa = pack_pairs(ph[1], ph[0], ph[3], ph[2], kHighHalves);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, vf[e], acc[r][e], 0, 0, 0);
        }
        if (more) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                kraw[s] = knext[s];
                vraw[s] = vnext[s];
            }
        }
    }

    // ---- fold the four waves' states of one row tile at a time through LDS and write the rows
    __shared__ float s_m[kPWaves][16], s_l[kPWaves][16];
    __shared__ __align__(16) float s_acc[kPWaves][16][kPD];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float lr = cross_rows_sum(l_run[r]);
        if (r) __syncthreads();
        if (kb == 0) {
            s_m[wave][n16] = m_run[r];
            s_l[wave][n16] = lr;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // row 4kb + i, channels 8 n16 + e
            float *dst = &s_acc[wave][4 * kb + i][8 * n16];
            *reinterpret_cast<float4 *>(dst) = make_float4(acc[r][0][i], acc[r][1][i], acc[r][2][i], acc[r][3][i]);
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(acc[r][4][i], acc[r][5][i], acc[r][6][i], acc[r][7][i]);
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < 16 * kPD; idx += kPThreads) {
            const int i = idx / kPD, ch = idx % kPD;
            const int row = row0 + 16 * r + i;
            if (row >= rows_total) continue;
            float mx = s_m[0][i];
#pragma unroll
            for (int w = 1; w < kPWaves; ++w) mx = fmaxf(mx, s_m[w][i]);
            float ls = 0.f, as = 0.f;
#pragma unroll
            for (int w = 0; w < kPWaves; ++w) {
                const float wgt = fast_exp2(s_m[w][i] - mx);
                ls = fmaf(s_l[w][i], wgt, ls);
                as = fmaf(s_acc[w][i][ch], wgt, as);
            }
            const int t = row / G, head = row - t * G;
            store_out<TD_BF16>(p.out, ((((int64_t)b * P + t) * p.num_q_heads + g * G + head) * kPD + ch),
                               ls > 0.f ? as / ls : 0.f);
        }
    }
}

template <int G, int R>
hipError_t launch_prefill_rows(PrefillParams p, hipStream_t stream) {
    p.row_blocks = (p.num_new * G + 16 * R - 1) / (16 * R);
    const dim3 grid(p.row_blocks * p.num_kv_heads * p.batch), block(kPThreads);
    hipLaunchKernelGGL((prefill_mfma_kernel<G, R>), grid, block, 0, stream, p);
    return hipGetLastError();
}

// Rows per workgroup: 64 when that still gives every CU a workgroup, else 32 or 16 (more
// workgroups, each streaming the keys and values for fewer rows).
template <int G>
hipError_t launch_prefill_group(const PrefillParams &p, hipStream_t stream) {
    const int64_t rows = (int64_t)p.num_new * G, pairs = (int64_t)p.num_kv_heads * p.batch;
    if ((rows + 63) / 64 * pairs >= 256) return launch_prefill_rows<G, 4>(p, stream);
    if ((rows + 31) / 32 * pairs >= 256) return launch_prefill_rows<G, 2>(p, stream);
    return launch_prefill_rows<G, 1>(p, stream);
}

}  // namespace

hipError_t launch_prefill(int group, const PrefillParams &p, hipStream_t stream) {
    switch (group) {
    case 1: return launch_prefill_group<1>(p, stream);
    case 2: return launch_prefill_group<2>(p, stream);
    case 4: return launch_prefill_group<4>(p, stream);
    case 8: return launch_prefill_group<8>(p, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tidal
