"""ctypes front end of the C oracle (oracle/tidal_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the bench's cpu_baseline
leg use it; nothing in the product path may import it.

Every function takes CPU torch tensors:
  q        [B][Hq][d]            bf16 or fp32
  K, V     [B][Hkv][N_max][d]    same dtype, last dim contiguous (strides passed on)
  seq_lens list/array of B ints, each N_b >= 1 and including the current token
and returns fp32 outputs [B][Hq][d] and int32 positions [B][Hkv][k], following
Eq. 1 and Alg. 1 of the paper (see the C file's header for the readings taken
where the paper is silent).
"""
import ctypes
import os

import numpy as np
import torch

from . import build as _build

DENSE, SELECT, SPARSE = 0, 1, 2

_ERR = {1: "bad argument", 2: "out of memory", 3: "position >= sequence length",
        4: "sparse layer before any selection layer"}


class _Shape(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("sm_scale", ctypes.c_float),
                ("kv_stride_batch", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64),
                ("kv_stride_tok", ctypes.c_int64),
                ("seq_lens", ctypes.c_void_p), ("max_seq_len", ctypes.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        _lib = ctypes.CDLL(path)
        for name in ("tdo_full", "tdo_select", "tdo_sparse", "tdo_step", "tdo_topk_row", "tdo_gather_pages",
                     "tdo_select_variant", "tdo_sparse_per_head", "tdo_append", "tdo_prefill"):
            getattr(_lib, name).restype = ctypes.c_int
        _lib.tdo_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    return lib().tdo_num_threads()


def _check(code):
    if code:
        raise RuntimeError("oracle: " + _ERR.get(code, "error %d" % code))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _shape(q, K, V, seq_lens, sm_scale):
    assert q.device.type == "cpu" and K.device.type == "cpu" and V.device.type == "cpu"
    assert q.dtype == K.dtype == V.dtype and q.dtype in (torch.bfloat16, torch.float32)
    assert q.dim() == 3 and K.dim() == 4 and K.shape == V.shape and K.stride() == V.stride()
    assert q.is_contiguous() and K.stride(3) == 1
    B, Hq, d = q.shape
    assert K.shape[0] == B and K.shape[3] == d
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    assert lens.shape == (B,)
    s = _Shape(B, Hq, K.shape[1], d, 0 if q.dtype == torch.bfloat16 else 1, float(sm_scale),
               K.stride(0), K.stride(1), K.stride(2), lens.ctypes.data, K.shape[2])
    return s, lens  # lens must stay alive while s is in use


def full(q, K, V, seq_lens, sm_scale=0.0, return_logits=False):
    """FullAttention(q, C[:]) of Alg. 1; optionally also the scaled logits [B][Hq][N_max]."""
    s, lens = _shape(q, K, V, seq_lens, sm_scale)
    out = torch.zeros(q.shape, dtype=torch.float32)
    logits = torch.full((q.shape[0], q.shape[1], K.shape[2]), float("-inf")) if return_logits else None
    _check(lib().tdo_full(ctypes.byref(s), _ptr(q), _ptr(K), _ptr(V), _ptr(out),
                          _ptr(logits) if return_logits else None))
    return (out, logits) if return_logits else out


def select(q, K, V, seq_lens, k, sm_scale=0.0, return_scores=False):
    """Token selection layer of Alg. 1: (out, positions[, group scores [B][Hkv][N_max]])."""
    s, lens = _shape(q, K, V, seq_lens, sm_scale)
    out = torch.zeros(q.shape, dtype=torch.float32)
    pos = torch.zeros((q.shape[0], K.shape[1], k), dtype=torch.int32)
    scores = torch.full((q.shape[0], K.shape[1], K.shape[2]), float("-inf")) if return_scores else None
    _check(lib().tdo_select(ctypes.byref(s), _ptr(q), _ptr(K), _ptr(V), ctypes.c_int32(k),
                            _ptr(out), _ptr(pos), _ptr(scores) if return_scores else None))
    return (out, pos, scores) if return_scores else (out, pos)


def sparse(q, K, V, seq_lens, positions, sm_scale=0.0):
    """SparseAttention(q, C[rho]) of Alg. 1 for positions int32 [B][Hkv][k] (-1 entries skipped)."""
    s, lens = _shape(q, K, V, seq_lens, sm_scale)
    positions = positions.to(torch.int32).contiguous()
    assert positions.dim() == 3 and positions.shape[:2] == (q.shape[0], K.shape[1])
    out = torch.zeros(q.shape, dtype=torch.float32)
    _check(lib().tdo_sparse(ctypes.byref(s), _ptr(q), _ptr(K), _ptr(V), _ptr(positions),
                            ctypes.c_int32(positions.shape[2]), _ptr(out)))
    return out


REDUCE_SUM, REDUCE_MAX, PER_HEAD, REDUCE_MEAN_PROB = 0, 1, 2, 3


def select_variant(q, K, V, seq_lens, k, variant, sm_scale=0.0):
    """Selection layer with another grouped-query rule: REDUCE_MAX (max of the group's logits, one
    rho per KV head), REDUCE_MEAN_PROB (mean of the heads' softmax probabilities, one rho per KV head)
    or PER_HEAD (the paper's per-head rule: positions and scores per query head).
    Returns (out, positions, scores)."""
    s, lens = _shape(q, K, V, seq_lens, sm_scale)
    rows = q.shape[1] if variant == PER_HEAD else K.shape[1]
    out = torch.zeros(q.shape, dtype=torch.float32)
    pos = torch.zeros((q.shape[0], rows, k), dtype=torch.int32)
    scores = torch.full((q.shape[0], rows, K.shape[2]), float("-inf"))
    _check(lib().tdo_select_variant(ctypes.byref(s), ctypes.c_int(variant), _ptr(q), _ptr(K), _ptr(V),
                                    ctypes.c_int32(k), _ptr(out), _ptr(pos), _ptr(scores)))
    return out, pos, scores


def sparse_per_head(q, K, V, seq_lens, positions, sm_scale=0.0):
    """Sparse attention with one rho per query head: positions int32 [B][Hq][k]."""
    s, lens = _shape(q, K, V, seq_lens, sm_scale)
    positions = positions.to(torch.int32).contiguous()
    assert positions.dim() == 3 and positions.shape[:2] == (q.shape[0], q.shape[1])
    out = torch.zeros(q.shape, dtype=torch.float32)
    _check(lib().tdo_sparse_per_head(ctypes.byref(s), _ptr(q), _ptr(K), _ptr(V), _ptr(positions),
                                     ctypes.c_int32(positions.shape[2]), _ptr(out)))
    return out


def topk_row(scores, k):
    """argTopK over one fp32 row: ascending indices of the min(k, n) largest, -1 padded."""
    scores = scores.to(torch.float32).contiguous()
    pos = torch.zeros(k, dtype=torch.int32)
    _check(lib().tdo_topk_row(_ptr(scores), ctypes.c_int(scores.numel()), ctypes.c_int(k), _ptr(pos)))
    return pos


def step(schedule, qs, Ks, Vs, seq_lens, k, sm_scale=0.0):
    """Alg. 1's layer loop (attention only).  Returns (list of fp32 outs, positions [n_select][B][Hkv][k])."""
    L = len(schedule)
    assert len(qs) == len(Ks) == len(Vs) == L
    s, lens = _shape(qs[0], Ks[0], Vs[0], seq_lens, sm_scale)
    for i in range(1, L):
        assert qs[i].shape == qs[0].shape and Ks[i].shape == Ks[0].shape
        assert Ks[i].stride() == Ks[0].stride() and Vs[i].stride() == Ks[0].stride()
    outs = [torch.zeros(qs[0].shape, dtype=torch.float32) for _ in range(L)]
    n_sel = max(1, sum(1 for x in schedule if x == SELECT))
    pos = torch.full((n_sel, qs[0].shape[0], Ks[0].shape[1], k), -1, dtype=torch.int32)
    arr = ctypes.c_void_p * L
    sched = (ctypes.c_int32 * L)(*[int(x) for x in schedule])
    _check(lib().tdo_step(ctypes.byref(s), ctypes.c_int32(L), sched,
                          arr(*[t.data_ptr() for t in qs]), arr(*[t.data_ptr() for t in Ks]),
                          arr(*[t.data_ptr() for t in Vs]), ctypes.c_int32(k),
                          arr(*[t.data_ptr() for t in outs]), _ptr(pos)))
    return outs, pos


def gather_pages(pool, block_table, seq_lens, max_seq_len, fill=float("nan")):
    """Logical cache [B][Hkv][max_seq_len][d] of a paged cache.

    pool is indexed [page][KV head][slot][c] (any strides with c contiguous, so a
    token-major pool is passed as a permuted view); block_table int32 [B][>= pages per
    sequence].  Token j of sequence b is pool[block_table[b][j // page_size], :, j % page_size].
    Rows j >= seq_lens[b] are set to `fill`."""
    assert pool.device.type == "cpu" and pool.dim() == 4 and pool.stride(3) == 1
    assert pool.dtype in (torch.bfloat16, torch.float32)
    bt = block_table.to(torch.int32).contiguous()
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    B = lens.shape[0]
    assert bt.dim() == 2 and bt.shape[0] == B
    num_pages, Hkv, page_size, d = pool.shape
    logical = torch.full((B, Hkv, max_seq_len, d), fill, dtype=pool.dtype)
    _check(lib().tdo_gather_pages(
        ctypes.c_int32(B), ctypes.c_int32(Hkv), ctypes.c_int32(d), ctypes.c_int32(pool.element_size()),
        ctypes.c_void_p(lens.ctypes.data), ctypes.c_int32(max_seq_len), ctypes.c_int32(page_size),
        ctypes.c_int32(num_pages), _ptr(bt), ctypes.c_int64(bt.stride(0)), ctypes.c_int64(pool.stride(0)),
        ctypes.c_int64(pool.stride(1)), ctypes.c_int64(pool.stride(2)), _ptr(pool), _ptr(logical)))
    return logical


def append(K, V, k_new, v_new, seq_lens):
    """C.append(k, v) of Alg. 1, in place: row seq_lens[b] - 1 of K and V takes k_new, v_new [B][Hkv][d]."""
    assert k_new.dim() == 3 and k_new.shape == v_new.shape and k_new.is_contiguous() and v_new.is_contiguous()
    assert k_new.dtype == K.dtype == V.dtype == v_new.dtype
    q_like = torch.zeros((K.shape[0], K.shape[1], K.shape[3]), dtype=K.dtype)
    s, lens = _shape(q_like, K, V, seq_lens, 0.0)
    assert k_new.shape == q_like.shape
    _check(lib().tdo_append(ctypes.byref(s), _ptr(K), _ptr(V), _ptr(k_new), _ptr(v_new)))


def prefill(q, K, V, seq_lens, sm_scale=0.0):
    """Attention of a prefill over the last P tokens (cache correction, Sec. 3.2): q [B][P][Hq][d];
    token j of sequence b sits at position seq_lens[b] - P + j and sees positions up to its own."""
    assert q.dim() == 4 and q.is_contiguous()
    B, P_new, Hq, d = q.shape
    s, lens = _shape(q.view(B * P_new, Hq, d)[:B], K, V, seq_lens, sm_scale)
    out = torch.zeros(q.shape, dtype=torch.float32)
    _check(lib().tdo_prefill(ctypes.byref(s), ctypes.c_int32(P_new), _ptr(q), _ptr(K), _ptr(V), _ptr(out)))
    return out
