"""ctypes binding of libtidal.so (include/tidal.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels; torch is used for
device memory and the current stream.  If the library has not been built this
module raises: there is no fallback path.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
# TIDAL_LIBRARY names another build of the same library (A/B timing of two builds in one run)
LIB_PATH = os.environ.get("TIDAL_LIBRARY") or os.path.join(HERE, "libtidal.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = range(5)
BF16, F32 = 0, 1
LAYER_DENSE, LAYER_SELECT, LAYER_SPARSE = 0, 1, 2

EXPORTS = ("td_validate", "td_workspace_bytes", "td_topk_workspace_bytes", "td_create", "td_destroy", "td_full_attend",
           "td_select_tokens", "td_sparse_attend", "td_prefill_attend", "td_prefill_workspace_bytes", "td_topk", "td_decode_step", "td_decode_step_append",
           "td_decode_step_static", "td_plan_launch", "td_set_tuning", "td_probe_stream", "td_reset",
           "td_status_string", "td_last_error")


class Shape(ctypes.Structure):
    """td_shape of include/tidal.h."""
    _fields_ = [("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("sm_scale", ctypes.c_float),
                ("kv_stride_batch", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64),
                ("kv_stride_tok", ctypes.c_int64),
                ("seq_lens", ctypes.c_void_p), ("max_seq_len", ctypes.c_int32),
                ("total_seq_len", ctypes.c_int64),
                ("page_size", ctypes.c_int32), ("num_pages", ctypes.c_int32),
                ("block_table", ctypes.c_void_p), ("block_table_stride", ctypes.c_int64),
                ("selection", ctypes.c_int32)]


class LaunchPlan(ctypes.Structure):
    """td_launch_plan of include/tidal.h."""
    _fields_ = [("chunk_tokens", ctypes.c_int32), ("chunks_per_row", ctypes.c_int32),
                ("waves_per_workgroup", ctypes.c_int32), ("matrix_core", ctypes.c_int32),
                ("grid_rows", ctypes.c_int32), ("merge_launch", ctypes.c_int32),
                ("workgroups", ctypes.c_int64)]


def plan_launch(shape, layer_kind, k, ctx=None):
    """td_plan_launch: the launch plan of one layer (host only, nothing is enqueued)."""
    plan = LaunchPlan()
    st = lib().td_plan_launch(ctx, ctypes.byref(shape), int(layer_kind), int(k), ctypes.byref(plan))
    if st != OK:
        raise TidalError(st, "td_plan_launch")
    return plan


class TidalError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("td_status %d: %s" % (status, message))
        self.status = status


_lib = None


def lib():
    """Opens libtidal.so (built by paper_2410_05076_amd/build.py) and declares its signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: run `python paper_2410_05076_amd/build.py` "
                          "(there is no non-HIP fallback)" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    shp = ctypes.POINTER(Shape)
    L.td_validate.argtypes, L.td_validate.restype = [shp, i32], ctypes.c_int
    L.td_workspace_bytes.argtypes, L.td_workspace_bytes.restype = [shp, i32], sz
    L.td_topk_workspace_bytes.argtypes, L.td_topk_workspace_bytes.restype = [i32, i32], sz
    L.td_create.argtypes, L.td_create.restype = [ctypes.POINTER(vp), ctypes.c_int, sz], ctypes.c_int
    L.td_destroy.argtypes, L.td_destroy.restype = [vp], ctypes.c_int
    L.td_full_attend.argtypes, L.td_full_attend.restype = [vp, shp, vp, vp, vp, vp, vp], ctypes.c_int
    L.td_select_tokens.argtypes = [vp, shp, vp, vp, vp, i32, vp, vp, vp, vp]
    L.td_select_tokens.restype = ctypes.c_int
    L.td_sparse_attend.argtypes = [vp, shp, vp, vp, vp, vp, i32, vp, vp]
    L.td_sparse_attend.restype = ctypes.c_int
    L.td_prefill_attend.argtypes = [vp, shp, i32, vp, vp, vp, vp, vp]
    L.td_prefill_attend.restype = ctypes.c_int
    L.td_prefill_workspace_bytes.argtypes, L.td_prefill_workspace_bytes.restype = [shp, i32], sz
    L.td_topk.argtypes = [vp, vp, i64, i32, vp, i32, i32, i32, vp, vp]
    L.td_topk.restype = ctypes.c_int
    L.td_decode_step.argtypes = [vp, shp, i32, ctypes.POINTER(i32), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                 ctypes.POINTER(vp), i32, ctypes.POINTER(vp), vp, vp]
    L.td_decode_step.restype = ctypes.c_int
    pv = ctypes.POINTER(vp)
    L.td_decode_step_append.argtypes = [vp, shp, i32, ctypes.POINTER(i32), pv, pv, pv, pv, pv, i32, pv, vp, vp]
    L.td_decode_step_append.restype = ctypes.c_int
    L.td_decode_step_static.argtypes = [shp, i32, ctypes.POINTER(i32), pv, pv, pv, i32, pv, vp, vp]
    L.td_decode_step_static.restype = ctypes.c_int
    L.td_plan_launch.argtypes = [vp, shp, i32, i32, ctypes.POINTER(LaunchPlan)]
    L.td_plan_launch.restype = ctypes.c_int
    L.td_set_tuning.argtypes, L.td_set_tuning.restype = [vp, i32, i32, i32, i32, i32], ctypes.c_int
    L.td_probe_stream.argtypes, L.td_probe_stream.restype = [vp, vp, vp, sz, vp], ctypes.c_int
    L.td_reset.argtypes, L.td_reset.restype = [vp, vp], ctypes.c_int
    L.td_status_string.argtypes, L.td_status_string.restype = [ctypes.c_int], ctypes.c_char_p
    L.td_last_error.argtypes, L.td_last_error.restype = [vp], ctypes.c_char_p
    _lib = L
    return L


def _dtype_code(t):
    if t == torch.bfloat16:
        return BF16
    if t == torch.float32:
        return F32
    raise TypeError("q, K, V must be bfloat16 or float32, got %s" % t)


SELECT_GROUP_SUM, SELECT_GROUP_MAX, SELECT_PER_HEAD, SELECT_GROUP_MEAN_PROB = 0, 1, 2, 3


def make_shape(q, K, seq_lens, sm_scale=0.0, total_seq_len=0, selection=0):
    """td_shape for q [B][Hq][d] and a cache tensor K [B][Hkv][N_max][d] (any strides with d contiguous).

    total_seq_len: the host's knowledge of sum(seq_lens), 0 if unknown (a launch-plan hint only)."""
    assert q.dim() == 3 and K.dim() == 4 and q.is_contiguous() and K.stride(3) == 1
    assert seq_lens.dtype == torch.int32 and seq_lens.is_contiguous() and seq_lens.numel() == q.shape[0]
    return Shape(q.shape[0], q.shape[1], K.shape[1], q.shape[2], _dtype_code(q.dtype), float(sm_scale),
                 K.stride(0), K.stride(1), K.stride(2), seq_lens.data_ptr(), K.shape[2], int(total_seq_len),
                 0, 0, None, 0, int(selection))


def make_paged_shape(q, pool, block_table, seq_lens, max_seq_len, sm_scale=0.0, total_seq_len=0, selection=0):
    """td_shape for a paged cache: pool indexed [page][Hkv][slot][d] (any strides with d contiguous;
    a token-major pool is passed as a permuted view), block_table int32 [B][entries per sequence]."""
    assert q.dim() == 3 and pool.dim() == 4 and q.is_contiguous() and pool.stride(3) == 1
    assert seq_lens.dtype == torch.int32 and seq_lens.is_contiguous() and seq_lens.numel() == q.shape[0]
    assert block_table.dtype == torch.int32 and block_table.dim() == 2 and block_table.stride(1) == 1
    assert block_table.shape[0] == q.shape[0]
    return Shape(q.shape[0], q.shape[1], pool.shape[1], q.shape[2], _dtype_code(q.dtype), float(sm_scale),
                 pool.stride(0), pool.stride(1), pool.stride(2), seq_lens.data_ptr(), int(max_seq_len),
                 int(total_seq_len), pool.shape[2], pool.shape[0], block_table.data_ptr(), block_table.stride(0),
                 int(selection))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


STATIC_SCRATCH_BYTES = 64 << 20


def decode_step_static(shape, schedule, qs, Ks, Vs, k, outs, positions):
    """td_decode_step_static: the decode step on the library's static scratch, no context, no allocation."""
    n = len(schedule)
    arr = ctypes.c_void_p * n
    sched = (ctypes.c_int32 * n)(*[int(x) for x in schedule])
    st = lib().td_decode_step_static(
        ctypes.byref(shape), n, sched, arr(*[t.data_ptr() for t in qs]), arr(*[t.data_ptr() for t in Ks]),
        arr(*[t.data_ptr() for t in Vs]), k, arr(*[t.data_ptr() for t in outs]), positions.data_ptr(), _stream())
    if st != OK:
        raise TidalError(st, lib().td_last_error(None).decode())
    return outs, positions


class Tidal:
    """A td_ctx with a workspace sized for one shape and budget."""

    def __init__(self, shape, k, device=None, topk_rows=0, topk_max_len=0, prefill_new=0, workspace_bytes=None):
        L = lib()
        self.device = torch.cuda.current_device() if device is None else device
        need = L.td_workspace_bytes(ctypes.byref(shape), k)
        if need == 0:
            raise TidalError(L.td_validate(ctypes.byref(shape), k), "invalid or unsupported shape")
        if topk_rows:       # also room for stand-alone td_topk calls of this size
            need = max(need, L.td_topk_workspace_bytes(topk_rows, topk_max_len))
        if prefill_new:     # also room for the token chunks of prefill_attend over this many new tokens
            need = max(need, L.td_prefill_workspace_bytes(ctypes.byref(shape), prefill_new))
        if workspace_bytes is not None:   # the caller's own size (td_create's argument as it is)
            need = workspace_bytes
        self.workspace_bytes = need
        self._ctx = ctypes.c_void_p()
        st = L.td_create(ctypes.byref(self._ctx), self.device, need)
        if st != OK:
            raise TidalError(st, "td_create failed")

    def close(self):
        # (at interpreter shutdown the module's globals may already be gone: then the process's exit frees the context)
        if getattr(self, "_ctx", None) and lib is not None:
            lib().td_destroy(self._ctx)
            self._ctx = None

    __del__ = close

    def _check(self, st):
        if st != OK:
            raise TidalError(st, lib().td_last_error(self._ctx).decode())

    def set_tuning(self, target_workgroups=0, min_chunk_dense=0, min_chunk_sparse=0, max_splits=0,
                   kernel_variant=0):
        self._check(lib().td_set_tuning(self._ctx, target_workgroups, min_chunk_dense, min_chunk_sparse,
                                        max_splits, kernel_variant))

    def reset(self):
        """td_reset: zeroes the ticket counters on the current stream."""
        self._check(lib().td_reset(self._ctx, _stream()))

    def full_attend(self, shape, q, K, V, out):
        self._check(lib().td_full_attend(self._ctx, ctypes.byref(shape), q.data_ptr(), K.data_ptr(),
                                         V.data_ptr(), out.data_ptr(), _stream()))
        return out

    def select_tokens(self, shape, q, K, V, k, out, positions, group_scores=None):
        self._check(lib().td_select_tokens(self._ctx, ctypes.byref(shape), q.data_ptr(), K.data_ptr(),
                                           V.data_ptr(), k, out.data_ptr(), positions.data_ptr(),
                                           group_scores.data_ptr() if group_scores is not None else None,
                                           _stream()))
        return out, positions

    def sparse_attend(self, shape, q, K, V, positions, k, out):
        self._check(lib().td_sparse_attend(self._ctx, ctypes.byref(shape), q.data_ptr(), K.data_ptr(),
                                           V.data_ptr(), positions.data_ptr(), k, out.data_ptr(), _stream()))
        return out

    def topk(self, scores, row_lens, rows_per_len, k, positions):
        rows, stride = scores.shape[0], scores.stride(0)
        self._check(lib().td_topk(self._ctx, scores.data_ptr(), stride, rows, row_lens.data_ptr(),
                                  rows_per_len, scores.shape[1], k, positions.data_ptr(), _stream()))
        return positions

    def probe_stream(self, src, dst=None):
        """Streams the bytes of `src` (copying them to `dst` when given) with a plain kernel."""
        nbytes = src.numel() * src.element_size()
        self._check(lib().td_probe_stream(self._ctx, dst.data_ptr() if dst is not None else None,
                                          src.data_ptr(), nbytes, _stream()))

    def prefill_attend(self, shape, q, K, V, out):
        """td_prefill_attend: q, out [B][num_new][Hq][d]; causal attention of the last num_new tokens."""
        assert q.dim() == 4 and q.is_contiguous() and out.is_contiguous() and out.shape == q.shape
        self._check(lib().td_prefill_attend(self._ctx, ctypes.byref(shape), q.shape[1], q.data_ptr(), K.data_ptr(),
                                            V.data_ptr(), out.data_ptr(), _stream()))
        return out

    def decode_step(self, shape, schedule, qs, Ks, Vs, k, outs, positions):
        n = len(schedule)
        arr = ctypes.c_void_p * n
        sched = (ctypes.c_int32 * n)(*[int(x) for x in schedule])
        self._check(lib().td_decode_step(
            self._ctx, ctypes.byref(shape), n, sched, arr(*[t.data_ptr() for t in qs]),
            arr(*[t.data_ptr() for t in Ks]), arr(*[t.data_ptr() for t in Vs]), k,
            arr(*[t.data_ptr() for t in outs]), positions.data_ptr(), _stream()))
        return outs, positions

    def decode_step_append(self, shape, schedule, qs, k_news, v_news, Ks, Vs, k, outs, positions):
        """td_decode_step_append: every layer appends k_news[i], v_news[i] [B][Hkv][d] to its cache first."""
        n = len(schedule)
        arr = ctypes.c_void_p * n
        sched = (ctypes.c_int32 * n)(*[int(x) for x in schedule])
        self._check(lib().td_decode_step_append(
            self._ctx, ctypes.byref(shape), n, sched, arr(*[t.data_ptr() for t in qs]),
            arr(*[t.data_ptr() for t in k_news]), arr(*[t.data_ptr() for t in v_news]),
            arr(*[t.data_ptr() for t in Ks]), arr(*[t.data_ptr() for t in Vs]), k,
            arr(*[t.data_ptr() for t in outs]), positions.data_ptr(), _stream()))
        return outs, positions
