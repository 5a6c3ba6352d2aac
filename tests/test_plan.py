"""Host-side launch planning (td_plan_launch), no GPU: the documented decisions, and the
bounds the kernels rely on (chunks per row within the workspace, staged positions / scores /
block-table entries within their LDS buffers) over a sweep of shapes."""
import ctypes
import itertools

import pytest

from paper_2410_05076_amd import tidal
from test_abi import good_shape, paged

DENSE, SELECT, SPARSE = 0, 1, 2
SPLITS_MAX, SPARSE_CHUNK_MAX, PAGE_STAGE_MAX, SCORE_STAGE_PER_WAVE = 256, 2048, 1024, 1024


def shape(batch=1, hq=32, hkv=8, n=32768, total=0, **over):
    return good_shape(batch=batch, num_q_heads=hq, num_kv_heads=hkv, max_seq_len=n, total_seq_len=total,
                      kv_stride_batch=hkv * n * 128, kv_stride_head=n * 128, **over)


def test_benchmark_shapes_get_the_documented_plans():
    c2 = shape()
    p = tidal.plan_launch(c2, DENSE, 2048)
    assert (p.matrix_core, p.waves_per_workgroup, p.chunk_tokens, p.chunks_per_row, p.workgroups) == (1, 8, 1024, 32, 256)
    p = tidal.plan_launch(c2, SPARSE, 2048)
    assert (p.matrix_core, p.waves_per_workgroup, p.chunk_tokens, p.chunks_per_row) == (1, 4, 128, 16)
    c3 = shape(hq=32, hkv=32, n=131072)
    assert tidal.plan_launch(c3, DENSE, 4096).matrix_core == 1          # full layers of small groups
    p = tidal.plan_launch(c3, SELECT, 4096)
    assert (p.matrix_core, p.waves_per_workgroup) == (0, 8)
    assert tidal.plan_launch(c3, SPARSE, 4096).matrix_core == 0
    assert tidal.plan_launch(c3, SPARSE, 4096).waves_per_workgroup == 8                 # large gathers: eight waves
    c5 = shape(batch=4, n=131072)
    assert [tidal.plan_launch(c5, SPARSE, k).waves_per_workgroup for k in (256, 1024, 2048, 4096, 16384)] == [4, 4, 8, 8, 8]
    assert tidal.plan_launch(c2, SPARSE, 4096).waves_per_workgroup == 8
    c6 = shape(hq=64, hkv=8)
    assert all(tidal.plan_launch(c6, kind, 2048).matrix_core == 1 for kind in (DENSE, SELECT, SPARSE))
    f32 = shape(dtype=tidal.F32)
    assert tidal.plan_launch(f32, DENSE, 128).matrix_core == 0


def test_ragged_hint_switches_to_many_small_chunks():
    even = tidal.plan_launch(shape(batch=16, n=65536, total=16 * 65536), DENSE, 2048)
    ragged = tidal.plan_launch(shape(batch=16, n=65536, total=16 * 36000), DENSE, 2048)
    assert even.waves_per_workgroup == 8 and ragged.waves_per_workgroup == 4
    assert ragged.chunk_tokens < even.chunk_tokens and ragged.workgroups > even.workgroups


def test_ragged_batches_get_odd_chunk_granules_and_a_fold_launch_of_their_own():
    """A slot serves several chunks there: chunk starts must not agree modulo a power of two, and no chunk waits for a ticket."""
    for batch, n, frac in itertools.product((4, 16, 64), (8192, 65536, 131072, 100000), (0.3, 0.6, 0.85)):
        s = shape(batch=batch, n=n, total=int(batch * n * frac))
        for kind in (DENSE, SELECT):
            p = tidal.plan_launch(s, kind, 2048)
            assert p.waves_per_workgroup == 4
            if p.chunks_per_row > 1:
                assert p.merge_launch == 1
                if p.chunk_tokens < 4 * SCORE_STAGE_PER_WAVE:        # the selection chunk's LDS limit wins over the rule
                    assert (p.chunk_tokens // 128) % 2 == 1, (batch, n, frac, kind, p.chunk_tokens)
            assert p.chunk_tokens * p.chunks_per_row >= n and p.chunks_per_row <= SPLITS_MAX
        assert tidal.plan_launch(s, SPARSE, 2048).merge_launch == 0
    even = shape(batch=16, n=65536, total=16 * 65536)
    assert all(tidal.plan_launch(even, kind, 2048).merge_launch == 0 for kind in (DENSE, SELECT, SPARSE))


def test_per_head_rule_gives_sparse_layers_one_grid_row_per_query_head():
    s = shape(selection=tidal.SELECT_PER_HEAD)
    assert tidal.plan_launch(s, SPARSE, 2048).grid_rows == 32
    assert tidal.plan_launch(s, SELECT, 2048).grid_rows == 8
    assert tidal.plan_launch(shape(), SPARSE, 2048).grid_rows == 8


@pytest.mark.parametrize("kind", [DENSE, SELECT, SPARSE])
def test_plans_stay_within_the_kernels_buffers(kind):
    for batch, (hq, hkv), n, k in itertools.product((1, 3, 64), ((8, 8), (32, 8), (64, 8), (16, 2)),
                                                   (1, 100, 4099, 32768, 131072, 1000000), (1, 64, 2048, 100000)):
        if batch * n > 2 ** 27:
            continue
        s = shape(batch=batch, hq=hq, hkv=hkv, n=n)
        p = tidal.plan_launch(s, kind, k)
        tokens = k if kind == SPARSE else n
        assert p.chunk_tokens % 128 == 0 and p.chunk_tokens >= 128
        assert 1 <= p.chunks_per_row <= SPLITS_MAX
        assert p.chunk_tokens * p.chunks_per_row >= tokens > p.chunk_tokens * (p.chunks_per_row - 1)
        if kind == SPARSE:
            assert p.chunk_tokens <= SPARSE_CHUNK_MAX
        if kind == SELECT:
            assert p.chunk_tokens <= p.waves_per_workgroup * SCORE_STAGE_PER_WAVE


@pytest.mark.parametrize("page_size", [1, 2, 16, 256, 4096])
def test_paged_plans_keep_a_chunks_table_entries_within_the_stage(page_size):
    for n in (100, 4099, 131072, 200000):
        pages = (n + page_size - 1) // page_size
        s = paged(page_size=page_size, max_seq_len=n, block_table_stride=pages, num_pages=pages,
                  kv_stride_batch=8 * page_size * 128, kv_stride_head=page_size * 128)
        for kind in (DENSE, SELECT):
            p = tidal.plan_launch(s, kind, 64)
            assert p.chunk_tokens // page_size + 1 <= PAGE_STAGE_MAX
            assert p.chunks_per_row <= SPLITS_MAX


def test_plan_rejects_bad_arguments():
    L = tidal.lib()
    plan = tidal.LaunchPlan()
    assert L.td_plan_launch(None, ctypes.byref(shape()), 3, 64, ctypes.byref(plan)) == tidal.ERR_INVALID_ARG
    assert L.td_plan_launch(None, ctypes.byref(shape()), SPARSE, 0, ctypes.byref(plan)) == tidal.ERR_INVALID_ARG
    assert L.td_plan_launch(None, ctypes.byref(shape(head_dim=96, kv_stride_tok=96)), DENSE, 0,
                            ctypes.byref(plan)) == tidal.ERR_UNSUPPORTED
    assert L.td_plan_launch(None, ctypes.byref(shape()), DENSE, 0, None) == tidal.ERR_INVALID_ARG


def test_prefill_workspace_covers_token_chunks_only_when_rows_are_few():
    L = tidal.lib()
    c2 = shape()
    # 16 new tokens x 4 heads per KV head = 64 rows = two row blocks of 32 per (sequence, KV head): 16
    # workgroups, so the tokens are cut into 16 chunks of 2048 and every chunk leaves 32 rows x 130 floats
    need = L.td_prefill_workspace_bytes(ctypes.byref(c2), 16)
    parts = 16 * 16 * 32 * 130 * 4
    fixed = 65536 * 4 + 256 * (2048 + 8) * 4     # ticket counters and the top-k state of 256 rows, always there
    assert parts <= need <= parts + fixed + 1024
    # 4096 new tokens fill the GPU with row blocks alone: no chunks, no workspace
    assert L.td_prefill_workspace_bytes(ctypes.byref(c2), 4096) == 0
    # a short cache cannot be cut below 512 tokens per chunk
    assert L.td_prefill_workspace_bytes(ctypes.byref(shape(n=600)), 16) == 0
    # invalid arguments
    assert L.td_prefill_workspace_bytes(ctypes.byref(c2), 0) == 0
    assert L.td_prefill_workspace_bytes(ctypes.byref(c2), 40000) == 0
