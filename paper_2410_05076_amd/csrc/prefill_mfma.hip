// Attention of a prefill over the last P tokens of every sequence (the cache-correction step of
// Sec. 3.2 re-runs full attention for the tokens that were decoded sparsely): token j sits at
// position N - P + j and attends, with Eq. 1, to the positions up to its own.  bf16, head_dim 128,
// contiguous cache.
//
// The query rows of a KV head are the (token, head) pairs, row = token * G + head.  A workgroup
// of four wave64s takes R * 16 consecutive rows (R = 4 or 2) and one chunk of the tokens, up to
// the last position any of its rows may see; the waves split the chunk's 32-token tiles
// (interleaved) and every wave keeps an online-softmax state for all R * 16 rows, so a K or V tile
// is loaded once per wave and used by R row tiles.  Per tile half: S^T = K Q^T with
// v_mfma_f32_16x16x32_bf16 (K from memory straight into the A operand; a lane then holds four
// tokens of one query row); then P = exp2(S^T scale log2(e) - m) rounded to bf16 once
// (v_cvt_pk_bf16_f32), and O^T += V^T P^T over the tile's 32 tokens, again with
// v_mfma_f32_16x16x32_bf16 (twice the rate of the 16-deep form), so that a lane's accumulators
// all belong to its own query row and the row's state (m, l) needs no shuffle.
//
// The reference maximum m of a row is lazy: it is raised (and the row's accumulators rescaled)
// only when a logit exceeds it by more than kLazyMax in log2 units, so p <= 2^kLazyMax, far
// inside the range of fp32 sums and bf16 operands, and the check is one compare per lane with no
// cross-lane step; after the first tile the rescale branch is practically never taken.  Tiles
// that every row of the workgroup sees in full run without masks and with wave-uniform load
// addresses; only the last tiles (the causal diagonal and the ragged end) take the masked path.
// The four waves' states are folded through LDS, one row tile at a time.  With one chunk the rows
// are written out; with more, the folded state goes to the workspace and prefill_merge_kernel
// combines the chunks.
//
// Per 32-token tile and wave: 16 loads of 16 bytes per lane, R * 17 MFMAs (R * 196608 flop, 272
// matrix-core cycles per row tile) and about 40 + R * 45 vector instructions, eight of them
// quarter-rate exponentials per row tile: the vector ALU and the matrix core are about balanced,
// and with one wave per SIMD they overlap only as far as the instruction order lets them.
#include "attend_tail.h"
#include "mfma_util.h"

#include <algorithm>
#include <type_traits>

namespace tidal {
namespace {

constexpr int kPD = 128;
constexpr int kPWaves = 4;
constexpr int kPThreads = kPWaves * kWave;
constexpr int kPTile = 32;                // tokens per tile
constexpr int kPStep = kPWaves * kPTile;  // tokens between two tiles of one wave
constexpr float kLazyMax = 8.f;       // a row's reference maximum may trail its true one by this (log2 units)

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t bf16_pair(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){lo, hi}, bf16x2));
}

template <int G, int R, bool PAGED>
__global__ __launch_bounds__(kPThreads)
void prefill_mfma_kernel(const PrefillParams p) {
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
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n16 = lane & 15, kb = lane >> 4;
    const int P = p.num_new, rows_total = P * G, row0 = rb * (16 * R);

    // Q^T fragments: lane (n16, kb) of fragment (r, s) holds d-octet 4s + kb of row row0 + 16r + n16;
    // rows beyond the last one are zero and never written.  All four waves use the same fragments,
    // tile after tile, so they live in LDS (16 bytes per lane and fragment, read back lane by lane)
    // and leave the registers to the tiles in flight; wave w fetches the fragments with s = w.
    __shared__ uint4 s_q[R * 4 * kWave];
    int tkn[R];
    uint4 qv[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int row = row0 + 16 * r + n16;
        tkn[r] = row / G;
        const int head = row - tkn[r] * G;
        qv[r] = make_uint4(0u, 0u, 0u, 0u);
        if (row < rows_total)
            qv[r] = *reinterpret_cast<const uint4 *>(
                static_cast<const char *>(p.q) +
                ((((int64_t)b * P + tkn[r]) * p.num_q_heads + g * G + head) * kPD + (4 * wave + kb) * 8) * 2);
    }
    asm volatile("" ::: "memory");  // the loads above are issued before the sequence length is needed

    const int N = min(max(p.seq_lens[b], 0), p.max_seq_len);
    // row (tile r, n16) sees tokens t < limit[r]; a token before the start of the cache sees none
    int limit[R];
#pragma unroll
    for (int r = 0; r < R; ++r) limit[r] = row0 + 16 * r + n16 < rows_total ? max(N - P + tkn[r] + 1, 0) : 0;
    const int last_tkn = min(P - 1, (row0 + 16 * R - 1) / G);
    const int t_end = max(N - P + last_tkn + 1, 0);   // tokens the rows of this block may see
    const int t_full = max(N - P + row0 / G + 1, 0);  // tokens below this one are seen by every row
    // this workgroup's chunk of them
    const int c0 = blockIdx.y * p.chunk, c1 = min(c0 + p.chunk, t_end);
    if (p.chunks > 1 && c0 >= t_end) return;  // the merge kernel knows that this chunk is empty
#pragma unroll
    for (int r = 0; r < R; ++r) s_q[(r * 4 + wave) * kWave + lane] = qv[r];
    __syncthreads();

    const int64_t row_bytes = p.stride_tok * 2;
    const int64_t head_off = ((PAGED ? 0 : (int64_t)b * p.stride_batch) + (int64_t)g * p.stride_head) * 2;
    const char *Kh = static_cast<const char *>(p.K) + head_off;  // wave-uniform
    const char *Vh = static_cast<const char *>(p.V) + head_off;
    // Paged cache (pages of at least 16 tokens): a 16-token half of a tile lies in one page, so a
    // whole tile needs two block-table entries, read one tile before the loads that use them.
    const int64_t page_bytes = p.stride_batch * 2;
    const int slot_mask = PAGED ? (1 << p.page_shift) - 1 : 0;
    const int32_t *table = PAGED ? p.block_table + (int64_t)b * p.bt_stride : nullptr;
    auto page_of = [&](int t) -> int {  // table entry of token t (any t: clamped into the table)
        if constexpr (PAGED) return table[min(max(t, 0), p.max_seq_len - 1) >> p.page_shift];
        return 0;
    };
    // The entry of a 16-token half is looked up by every lane for its own key token of the half
    // (t16 + n16: the same entry for all of them).  A wave-uniform lookup would be turned into a
    // scalar value on the spot, which means waiting for the vector load right behind the tile
    // loads it was issued after; the per-lane value is only waited for where the next tile's
    // addresses are formed, a tile later.
    auto page_of_half = [&](int t16) -> int { return page_of(t16 + n16); };
    auto row_off = [&](int t, int page) -> int64_t {  // byte offset of token t's row inside the head's cache
        if constexpr (PAGED)
            return (int64_t)min(max(page, 0), p.num_pages - 1) * page_bytes + (int64_t)(t & slot_mask) * row_bytes;
        return (int64_t)t * row_bytes;
    };

    // The softmax denominator is accumulated on the matrix core as well, as one more "channel" of
    // ones: it then sums the same bf16-rounded probabilities as the numerator, which keeps a row
    // that one token dominates exact, and costs no vector instruction.
    float m_use[R];   // reference maximum of row n16 (the same in its four lanes)
    f32x4 acc[R][8];  // acc[r][e][i]: row n16 of tile r, channel 8 (4 kb + i) + e
    f32x4 lacc[R];    // every element: l of row n16
    const uint32_t one2 = 0x3f803f80u;  // bf16 (1, 1)
    const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(one2, one2, one2, one2));
#pragma unroll
    for (int r = 0; r < R; ++r) {
        m_use[r] = kEmptyMax;
        lacc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float scale2 = p.scale * kLog2e;

    // A tile is 32 tokens, two halves h of 16.  K: token base + 16 h + n16, d-octets kb + 4 s;
    // V: tokens base + 16 h + 4 kb + u, channels 8 n16 .. + 7.  A tile whose tokens all exist is
    // addressed as a wave-uniform base plus a constant lane offset; the last, partial tile clamps
    // its tokens to the last one streamed (masked below).
    const uint32_t k_lane = (uint32_t)(n16 * row_bytes) + kb * 16, v_lane = (uint32_t)(4 * kb * row_bytes) + n16 * 16;
    uint4 kr[2][4], vr[2][4];
    auto load_full = [&](int base, uint4 (&kr)[2][4], uint4 (&vr)[2][4], const int (&pages)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int64_t off = row_off(base + 16 * h, pages[h]);
            const char *kt = Kh + off, *vt = Vh + off;
#pragma unroll
            for (int s = 0; s < 4; ++s) kr[h][s] = *reinterpret_cast<const uint4 *>(kt + k_lane + 64 * s);
#pragma unroll
            for (int u = 0; u < 4; ++u) vr[h][u] = *reinterpret_cast<const uint4 *>(vt + u * row_bytes + v_lane);
        }
    };
    auto load_tile = [&](int base, uint4 (&kr)[2][4], uint4 (&vr)[2][4]) {
        if (base + kPTile <= t_end) {
            const int pages[2] = {page_of_half(base), page_of_half(base + 16)};
            load_full(base, kr, vr, pages);
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int tk = min(base + 16 * h + n16, t_end - 1);
                const char *kp = Kh + row_off(tk, page_of(tk)) + kb * 16;
#pragma unroll
                for (int s = 0; s < 4; ++s) kr[h][s] = *reinterpret_cast<const uint4 *>(kp + 64 * s);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int tv = min(base + 16 * h + 4 * kb + u, t_end - 1);
                    vr[h][u] = *reinterpret_cast<const uint4 *>(Vh + row_off(tv, page_of(tv)) + n16 * 16);
                }
            }
        }
    };

    // One 32-token tile against the R row tiles.  kMasked: per-row causal limits apply; kSteady:
    // the wave's next tile exists and is whole, so its loads need no branch (and its block-table
    // entries are in pages_next already).  Returns false, with nothing accumulated, when some
    // reference maximum has to be raised first (the caller then loads the tile again: its
    // registers may already be receiving the next one).  The next tile's loads: with R = 4 (one
    // wave per SIMD fits the registers, a long tile) they go into the registers of this tile as
    // soon as its keys are multiplied and its values are in operand order (both before the maxima
    // are looked at, so the byte permutes run under the K Q^T MFMAs and the loads get the rest of
    // the tile to land); the smaller variant, whose tiles are too short to cover the latency that
    // way, loads into a second set of registers before anything else.
    int pages_next[2] = {0, 0};
    auto look_ahead = [&](int t) {  // block-table entries of the tile that starts at token t
        pages_next[0] = page_of_half(t);
        pages_next[1] = page_of_half(t + 16);
    };
    float top[R];  // largest scaled logit of this lane in the tile, per row tile
    int base = c0 + wave * kPTile;
    auto consume = [&](auto masked, auto steady) -> bool {
        constexpr bool kMasked = decltype(masked)::value, kSteady = decltype(steady)::value;
        constexpr bool kInPlace = R == 4;
        const bool more = kSteady || base + kPStep < c1;
        uint4 kn[kInPlace ? 1 : 2][4], vn[kInPlace ? 1 : 2][4];
        if constexpr (!kInPlace) {
            if constexpr (kSteady) {
                load_full(base + kPStep, kn, vn, pages_next);
                look_ahead(base + 2 * kPStep);
            } else {
                if (more) load_tile(base + kPStep, kn, vn);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        const int t_lane = base + 4 * kb;  // this lane's logits are for tokens t_lane + 16 h + i
        f32x4 st[R][2];
        bool grow = false;
        // the 2 R chains of four dependent MFMAs advance together, so that none waits for its own result
#pragma unroll
        for (int r = 0; r < R; ++r) st[r][0] = st[r][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        asm volatile("" ::: "memory");  // the fragments are read from LDS in every tile, not kept in registers
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const bf16x8 qf = __builtin_bit_cast(bf16x8, s_q[(r * 4 + s) * kWave + lane]);
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    st[r][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kr[h][s]), qf, st[r][h], 0, 0, 0);
            }
        // V^T as A operand: for channel group e, the lane's eight tokens (4kb .. 4kb+3 of either
        // half) of channel 8 n16 + e
        bf16x8 vf[8];
        {
            uint32_t vw[2][4][4];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    vw[h][u][0] = vr[h][u].x;
                    vw[h][u][1] = vr[h][u].y;
                    vw[h][u][2] = vr[h][u].z;
                    vw[h][u][3] = vr[h][u].w;
                }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t sel = (e & 1) ? kHighHalves : kLowHalves;
                const int w = e >> 1;
                vf[e] = __builtin_bit_cast(
                    bf16x8, make_uint4(__builtin_amdgcn_perm(vw[0][1][w], vw[0][0][w], sel), __builtin_amdgcn_perm(vw[0][3][w], vw[0][2][w], sel),
                                       __builtin_amdgcn_perm(vw[1][1][w], vw[1][0][w], sel), __builtin_amdgcn_perm(vw[1][3][w], vw[1][2][w], sel)));
                asm volatile("" : "+v"(vf[e]));  // computed here, under the MFMAs above, not sunk below the branch
            }
        }
        if constexpr (kInPlace) {
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (kSteady) {
                load_full(base + kPStep, kr, vr, pages_next);
                look_ahead(base + 2 * kPStep);
            } else {
                if (more) load_tile(base + kPStep, kr, vr);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (kMasked) {
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i) st[r][h][i] = t_lane + 16 * h + i < limit[r] ? st[r][h][i] : -INFINITY;
            }
            top[r] = fmaxf(fmaxf(fmaxf(st[r][0][0], st[r][0][1]), fmaxf(st[r][0][2], st[r][0][3])),
                           fmaxf(fmaxf(st[r][1][0], st[r][1][1]), fmaxf(st[r][1][2], st[r][1][3]))) * scale2;  // scale2 > 0
            grow |= top[r] > m_use[r] + kLazyMax;
        }
        if (__builtin_expect(__any(grow), 0)) return false;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float pr[2][4];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 4; ++i) pr[h][i] = fast_exp2(fmaf(st[r][h][i], scale2, -m_use[r]));
            // P^T as B operand: the lane's eight tokens of row n16, as two bf16 parts (the upper
            // half of the float, and the rest rounded to bf16), so that the probabilities carry
            // 16 bits like those of the decode kernels: with a single bf16 rounding, two or three
            // comparable tokens with far-apart values put up to 2^-10 of that distance on the
            // output, a quarter of the stated tolerance on top of the output's own rounding
            uint32_t ph[2][4];
            float pl[2][4];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    ph[h][i] = __float_as_uint(pr[h][i]);
                    pl[h][i] = pr[h][i] - __uint_as_float(ph[h][i] & 0xffff0000u);
                }
            const bf16x8 pb = __builtin_bit_cast(
                bf16x8, make_uint4(__builtin_amdgcn_perm(ph[0][1], ph[0][0], kHighHalves), __builtin_amdgcn_perm(ph[0][3], ph[0][2], kHighHalves),
                                   __builtin_amdgcn_perm(ph[1][1], ph[1][0], kHighHalves), __builtin_amdgcn_perm(ph[1][3], ph[1][2], kHighHalves)));
            const bf16x8 pb_lo = __builtin_bit_cast(bf16x8, make_uint4(bf16_pair(pl[0][0], pl[0][1]), bf16_pair(pl[0][2], pl[0][3]),
                                                                      bf16_pair(pl[1][0], pl[1][1]), bf16_pair(pl[1][2], pl[1][3])));
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                acc[r][e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[e], pb, acc[r][e], 0, 0, 0);
                acc[r][e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[e], pb_lo, acc[r][e], 0, 0, 0);
            }
            lacc[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb, lacc[r], 0, 0, 0);
            lacc[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb_lo, lacc[r], 0, 0, 0);
        }
        if constexpr (!kInPlace) {
            if (more) {
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        kr[h][s] = kn[h][s];
                        vr[h][s] = vn[h][s];
                    }
            }
        }
        base += kPStep;
        return true;
    };
    // Rare (after a row's first tile practically never): bring every row's reference maximum up
    // to date and rescale its state.  Kept outside the tile loops so that the accumulators stay in
    // their matrix-core registers there.
    auto raise = [&]() {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float m_new = fmaxf(m_use[r], cross_rows_max(top[r]));
            const float alpha = fast_exp2(m_use[r] - m_new);
            m_use[r] = m_new;
            lacc[r] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] *= alpha;
        }
    };

    // First the tiles that need no mask and whose successor is whole, then the rest through the
    // general path; a tile that needs a higher reference maximum leaves the loops, and is taken
    // again after the rescale.
    if (base < c1) load_tile(base, kr, vr);
    for (;;) {
        bool done = true;
        if (base + kPTile <= t_full && base + kPStep + kPTile <= c1) look_ahead(base + kPStep);
        while (done && base + kPTile <= t_full && base + kPStep + kPTile <= c1) done = consume(std::false_type{}, std::true_type{});
        while (done && base < c1) done = consume(std::true_type{}, std::false_type{});
        if (done) break;
        raise();
        load_tile(base, kr, vr);
    }

    // ---- fold the four waves' states of one row tile at a time through LDS and write the rows
    constexpr int kPitch = kPD + 4;  // rows of one wave's tile start in different banks
    __shared__ float s_m[kPWaves][16], s_l[kPWaves][16];
    __shared__ __align__(16) float s_acc[kPWaves][16][kPitch];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r) __syncthreads();
        if (kb == 0) {
            s_m[wave][n16] = m_use[r];
            s_l[wave][n16] = lacc[r][0];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // row n16, channels 8 (4 kb + i) + e
            float *dst = &s_acc[wave][n16][8 * (4 * kb + i)];
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
            if (p.chunks > 1) {  // partial state of (row, chunk): maximum, denominator, numerators
                const int64_t slot = (((int64_t)pair * p.row_blocks + rb) * p.chunks + blockIdx.y) * (16 * R) + 16 * r + i;
                p.part_acc[slot * kPD + ch] = as;
                if (ch == 0) *reinterpret_cast<float2 *>(p.part_ml + slot * 2) = make_float2(mx, ls);
            } else {
                const int t = row / G, head = row - t * G;
                store_out<TD_BF16>(p.out, ((((int64_t)b * P + t) * p.num_q_heads + g * G + head) * kPD + ch),
                                   ls > 0.f ? as / ls : 0.f);
            }
        }
    }
}

// Merge of the chunks' partial states: one workgroup per row, thread = (channel, one of four
// interleaved sets of chunks), so that every thread's loads are independent and few.
constexpr int kMergeSets = 4;
constexpr int kPrefillChunksMax = 512;
template <int G>
__global__ __launch_bounds__(kMergeSets * kPD) void prefill_merge_kernel(const PrefillParams p) {
    __shared__ float s_m[kPrefillChunksMax], s_l[kPrefillChunksMax], s_part[kMergeSets][kPD];
    const int rpw = p.rows_per_wg, P = p.num_new;
    const int64_t rid = blockIdx.x;  // over (pair, row block, row in block)
    const int ch = threadIdx.x % kPD, set = threadIdx.x / kPD;
    const int64_t wg = rid / rpw;
    const int i = (int)(rid - wg * rpw);
    const int pair = (int)(wg / p.row_blocks), rb = (int)(wg - (int64_t)pair * p.row_blocks);
    const int row = rb * rpw + i;
    if (row >= P * G) return;
    const int g = pair % p.num_kv_heads, b = pair / p.num_kv_heads;
    const int N = min(max(p.seq_lens[b], 0), p.max_seq_len);
    const int last_tkn = min(P - 1, (rb * rpw + rpw - 1) / G);
    const int t_end = max(N - P + last_tkn + 1, 0);
    const int nch = min(p.chunks, (t_end + p.chunk - 1) / p.chunk);  // chunks that hold tokens for this row block
    const float *ml = p.part_ml + (wg * p.chunks * rpw + i) * 2;
    const float *pa = p.part_acc + (wg * p.chunks * rpw + i) * kPD + ch;
    for (int c = threadIdx.x; c < nch; c += kMergeSets * kPD) {
        const float2 s = *reinterpret_cast<const float2 *>(ml + (int64_t)c * rpw * 2);
        s_m[c] = s.x;
        s_l[c] = s.y;
    }
    __syncthreads();
    float mx = kEmptyMax;
    for (int c = 0; c < nch; ++c) mx = fmaxf(mx, s_m[c]);
    float as = 0.f;
#pragma unroll 8
    for (int c = set; c < nch; c += kMergeSets) as = fmaf(pa[(int64_t)c * rpw * kPD], fast_exp2(s_m[c] - mx), as);
    s_part[set][ch] = as;
    __syncthreads();
    if (set) return;
    float ls = 0.f;
    for (int c = 0; c < nch; ++c) ls = fmaf(s_l[c], fast_exp2(s_m[c] - mx), ls);
#pragma unroll
    for (int s = 1; s < kMergeSets; ++s) as += s_part[s][ch];
    const int t = row / G, head = row - t * G;
    store_out<TD_BF16>(p.out, ((((int64_t)b * P + t) * p.num_q_heads + g * G + head) * kPD + ch), ls > 0.f ? as / ls : 0.f);
}

template <int G, int R>
hipError_t launch_prefill_rows(const PrefillParams &p, hipStream_t stream) {
    const int pairs = p.num_kv_heads * p.batch;
    const dim3 grid(p.row_blocks * pairs, p.chunks), block(kPThreads);
    if (p.block_table)
        hipLaunchKernelGGL((prefill_mfma_kernel<G, R, true>), grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL((prefill_mfma_kernel<G, R, false>), grid, block, 0, stream, p);
    if (p.chunks > 1) {
        const int64_t rows = (int64_t)p.row_blocks * pairs * p.rows_per_wg;
        hipLaunchKernelGGL((prefill_merge_kernel<G>), dim3((unsigned)rows), dim3(kMergeSets * kPD), 0, stream, p);
    }
    return hipGetLastError();
}

template <int G>
hipError_t launch_prefill_group(const PrefillParams &p, hipStream_t stream) {
    switch (p.rows_per_wg) {
    case 64: return launch_prefill_rows<G, 4>(p, stream);
    case 32: return launch_prefill_rows<G, 2>(p, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

// Rows per workgroup: 64 (the keys and values are streamed once per row block, and the R = 4
// kernel does the most arithmetic per byte loaded), but 32 for a pair with no more than 128
// rows: such a prefill is bound by the stream of the cache, like a decode step, and the R = 2
// kernel has the registers to load a whole tile ahead.  Few row blocks leave most of the chip
// idle, so the tokens are cut into chunks until every CU has a workgroup; more chunks than that
// measured slower at every size (each adds a partial state of rows_per_wg * 520 bytes, an
// epilogue and merge work).  A chunk is at least 512 tokens.
PrefillPlan plan_prefill(int64_t rows, int64_t pairs, int32_t max_seq_len, size_t part_avail) {
    PrefillPlan pl;
    pl.rows_per_wg = rows <= 128 ? 32 : 64;
    pl.row_blocks = (int32_t)((rows + pl.rows_per_wg - 1) / pl.rows_per_wg);
    const int64_t wgs = (int64_t)pl.row_blocks * pairs;
    constexpr int64_t kTargetWgs = 256, kMinChunk = 512;
    int64_t chunks = (kTargetWgs + wgs - 1) / wgs;
    chunks = std::min<int64_t>({chunks, std::max<int64_t>(1, max_seq_len / kMinChunk), (int64_t)kPrefillChunksMax});
    const size_t per_chunk = (size_t)wgs * pl.rows_per_wg * (kPD + 2) * sizeof(float);
    if (chunks > 1 && per_chunk * chunks > part_avail) chunks = (int64_t)(part_avail / per_chunk);
    if (chunks <= 1) {
        pl.chunks = 1;
        pl.chunk = (max_seq_len + kPStep - 1) / kPStep * kPStep;
        pl.part_bytes = 0;
        return pl;
    }
    pl.chunk = (int32_t)(((max_seq_len + chunks - 1) / chunks + kPStep - 1) / kPStep * kPStep);
    pl.chunks = (max_seq_len + pl.chunk - 1) / pl.chunk;
    pl.part_bytes = per_chunk * pl.chunks;
    return pl;
}

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
