"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2410_05076_amd import tidal

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good_shape(**over):
    lens = ctypes.c_int32(100)
    f = dict(batch=1, num_q_heads=32, num_kv_heads=8, head_dim=128, dtype=tidal.BF16, sm_scale=0.0,
             kv_stride_batch=8 * 100 * 128, kv_stride_head=100 * 128, kv_stride_tok=128,
             seq_lens=ctypes.addressof(lens), max_seq_len=100, total_seq_len=0)
    f.update(over)
    s = tidal.Shape(**f)
    s._keep = lens
    return s


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "tidal.h")) as f:
        text = f.read()
    declared = set(re.findall(r"\b(td_[a-z_]+)\s*\(", text))
    assert declared == set(tidal.EXPORTS)
    L = tidal.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_validate_accepts_the_benchmark_shapes():
    L = tidal.lib()
    assert L.td_validate(ctypes.byref(good_shape()), 2048) == tidal.OK
    assert L.td_validate(ctypes.byref(good_shape(num_kv_heads=32)), 4096) == tidal.OK
    assert L.td_validate(ctypes.byref(good_shape(num_q_heads=8, num_kv_heads=2, head_dim=64, dtype=tidal.F32,
                                                 kv_stride_tok=64)), 128) == tidal.OK


def paged(**over):
    table = (ctypes.c_int32 * 8)(*range(8))
    f = dict(page_size=16, num_pages=8, block_table=ctypes.addressof(table), block_table_stride=8,
             kv_stride_batch=8 * 16 * 128, kv_stride_head=16 * 128)
    f.update(over)
    s = good_shape(**f)
    s._table = table
    return s


def test_validate_accepts_a_paged_shape():
    L = tidal.lib()
    assert L.td_validate(ctypes.byref(paged()), 64) == tidal.OK
    assert L.td_validate(ctypes.byref(paged(page_size=1, block_table_stride=100)), 64) == tidal.OK


@pytest.mark.parametrize("over,code", [
    (dict(page_size=12), tidal.ERR_INVALID_ARG),              # not a power of two
    (dict(page_size=-16), tidal.ERR_INVALID_ARG),
    (dict(block_table=None), tidal.ERR_INVALID_ARG),
    (dict(num_pages=0), tidal.ERR_INVALID_ARG),
    (dict(block_table_stride=6), tidal.ERR_INVALID_ARG),      # 100 tokens need 7 pages of 16
    (dict(page_size=1, block_table_stride=400000, max_seq_len=400000), tidal.ERR_UNSUPPORTED),
])
def test_validate_rejects_paged(over, code):
    L = tidal.lib()
    assert L.td_validate(ctypes.byref(paged(**over)), 64) == code


@pytest.mark.parametrize("over,k,code", [
    (dict(batch=0), 1, tidal.ERR_INVALID_ARG),
    (dict(num_q_heads=30), 1, tidal.ERR_INVALID_ARG),
    (dict(max_seq_len=0), 1, tidal.ERR_INVALID_ARG),
    (dict(seq_lens=None), 1, tidal.ERR_INVALID_ARG),
    (dict(dtype=7), 1, tidal.ERR_INVALID_ARG),
    (dict(sm_scale=-1.0), 1, tidal.ERR_INVALID_ARG),
    (dict(kv_stride_tok=64), 1, tidal.ERR_INVALID_ARG),
    (dict(kv_stride_tok=132), 1, tidal.ERR_INVALID_ARG),
    (dict(total_seq_len=-5), 1, tidal.ERR_INVALID_ARG),
    (dict(selection=4), 1, tidal.ERR_INVALID_ARG),
    (dict(selection=-1), 1, tidal.ERR_INVALID_ARG),
    (dict(), 600000, tidal.ERR_INVALID_ARG),
    (dict(head_dim=96, kv_stride_tok=96), 1, tidal.ERR_UNSUPPORTED),
    (dict(max_seq_len=(1 << 30) + 1), 0, tidal.ERR_UNSUPPORTED),
    (dict(num_q_heads=24, num_kv_heads=8), 1, tidal.ERR_UNSUPPORTED),
    (dict(num_q_heads=128, num_kv_heads=8), 1, tidal.ERR_UNSUPPORTED),
])
def test_validate_rejects(over, k, code):
    L = tidal.lib()
    assert L.td_validate(ctypes.byref(good_shape(**over)), k) == code
    assert L.td_workspace_bytes(ctypes.byref(good_shape(**over)), k) == 0
    assert L.td_validate(None, 1) == tidal.ERR_INVALID_ARG


def test_workspace_bytes_covers_partials_and_scores():
    L = tidal.lib()
    s = good_shape(max_seq_len=32768)
    dense_only = L.td_workspace_bytes(ctypes.byref(s), 0)
    with_k = L.td_workspace_bytes(ctypes.byref(s), 2048)
    assert dense_only >= 32 * 256 * (128 + 2) * 4          # 256 chunk partials per query head
    assert with_k - dense_only >= 8 * 32768 * 4            # one fp32 score per (KV head, token)
    assert with_k % 256 == 0


def test_calls_without_a_context_fail_cleanly():
    L = tidal.lib()
    s = good_shape()
    assert L.td_full_attend(None, ctypes.byref(s), None, None, None, None, None) == tidal.ERR_INVALID_ARG
    assert L.td_sparse_attend(None, ctypes.byref(s), None, None, None, None, 4, None, None) == tidal.ERR_INVALID_ARG
    assert L.td_destroy(None) == tidal.ERR_INVALID_ARG
    assert L.td_create(None, 0, 0) == tidal.ERR_INVALID_ARG
    assert L.td_status_string(tidal.ERR_WORKSPACE) == b"workspace too small"
    assert L.td_last_error(None) == b"context is NULL"


def test_host_logic_under_sanitizers():
    """Argument checks, workspace layout and launch planning, compiled with AddressSanitizer and
    UndefinedBehaviorSanitizer (host code only), over a grid of valid, invalid and extreme shapes."""
    from paper_2410_05076_amd import build
    if not all(os.path.exists(os.path.join(build.OBJ_DIR, os.path.basename(s)[:-4] + ".o")) for s in build.SOURCES):
        build.build()
    exe = build.build_sanitized_host_check()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0 and r.stdout.startswith("ok"), (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
