// Host-side exerciser of the C ABI for a sanitizer build (address + undefined behaviour) of the
// library's host code: validation, workspace sizing and launch planning over a grid of shapes,
// including invalid and extreme ones.  Calls only entry points that never touch a GPU.
// Built and run by tests/test_abi.py::test_host_logic_under_sanitizers; prints "ok" on success.
#include <stdio.h>
#include <string.h>

#include "tidal.h"

static int32_t fake_lens[4] = {1, 2, 3, 4};

static td_shape base_shape() {
    td_shape s;
    memset(&s, 0, sizeof s);
    s.batch = 1;
    s.num_q_heads = 32;
    s.num_kv_heads = 8;
    s.head_dim = 128;
    s.dtype = TD_BF16;
    s.kv_stride_tok = 128;
    s.kv_stride_head = 128 * 4096;
    s.kv_stride_batch = 128 * 4096 * 8;
    s.seq_lens = fake_lens;  // never dereferenced by the host-only calls
    s.max_seq_len = 4096;
    return s;
}

int main() {
    long calls = 0, accepted = 0;
    const int32_t batches[] = {-1, 0, 1, 4, 16, 4096, 65535, 65536, 2147483647};
    const int32_t heads[][2] = {{32, 8}, {32, 32}, {64, 8}, {8, 2}, {30, 8}, {0, 0}, {8, 16}, {65536, 65536}, {128, 8}};
    const int32_t lens[] = {-5, 0, 1, 127, 128, 129, 4096, 32768, 131072, 1048576, 1048577, 2147483647};
    const int32_t ks[] = {-1, 0, 1, 128, 2048, 16384, 524288, 524289, 2147483647};
    const int32_t dims[] = {64, 128, 96, 0, -8};
    const int32_t pages[] = {0, 1, 16, 64, 12, -16, 1 << 30};
    for (int32_t b : batches)
        for (auto &h : heads)
            for (int32_t n : lens)
                for (int32_t d : dims)
                    for (int32_t pg : pages)
                        for (int sel = -1; sel <= 4; ++sel) {
                            td_shape s = base_shape();
                            s.batch = b;
                            s.num_q_heads = h[0];
                            s.num_kv_heads = h[1];
                            s.max_seq_len = n;
                            s.head_dim = d;
                            s.kv_stride_tok = d > 0 ? d : 8;
                            s.selection = sel;
                            s.total_seq_len = (int64_t)b * (n / 2);
                            int32_t table[4] = {0, 1, 2, 3};
                            if (pg) {
                                s.page_size = pg;
                                s.num_pages = 4;
                                s.block_table = table;
                                s.block_table_stride = pg > 0 ? ((int64_t)n + pg - 1) / pg : 1;
                            }
                            for (int32_t k : ks) {
                                const td_status v = td_validate(&s, k);
                                const size_t ws = td_workspace_bytes(&s, k);
                                calls += 2;
                                if ((v == TD_OK) != (ws != 0)) {
                                    printf("validate %d but workspace %zu\n", (int)v, ws);
                                    return 1;
                                }
                                if (v != TD_OK) continue;
                                ++accepted;
                                for (int kind = TD_LAYER_DENSE; kind <= TD_LAYER_SPARSE; ++kind) {
                                    td_launch_plan plan;
                                    const td_status ps = td_plan_launch(nullptr, &s, kind, k, &plan);
                                    ++calls;
                                    if (kind != TD_LAYER_DENSE && k < 1) {
                                        if (ps == TD_OK) return 2;
                                        continue;
                                    }
                                    if (ps != TD_OK || plan.chunk_tokens < 1 || plan.chunks_per_row < 1 || plan.chunks_per_row > 256 ||
                                        (plan.waves_per_workgroup != 4 && plan.waves_per_workgroup != 8) ||
                                        (int64_t)plan.chunk_tokens * plan.chunks_per_row < (kind == TD_LAYER_SPARSE ? k : n)) {
                                        printf("bad plan: status %d chunk %d chunks %d waves %d for n %d k %d kind %d\n", (int)ps,
                                               plan.chunk_tokens, plan.chunks_per_row, plan.waves_per_workgroup, n, k, kind);
                                        return 3;
                                    }
                                }
                                if (d == 128) {
                                    (void)td_prefill_workspace_bytes(&s, 1);
                                    (void)td_prefill_workspace_bytes(&s, 16);
                                    (void)td_prefill_workspace_bytes(&s, n);
                                    calls += 3;
                                }
                            }
                        }
    (void)td_topk_workspace_bytes(0, 0);
    (void)td_topk_workspace_bytes(65535, 1048576);
    (void)td_validate(nullptr, 1);
    (void)td_status_string(TD_ERR_HIP);
    (void)td_last_error(nullptr);
    printf("ok %ld calls, %ld shapes accepted\n", calls, accepted);
    return 0;
}
