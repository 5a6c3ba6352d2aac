"""One context, many launch shapes.  Split launches of one (sequence, KV head) meet through ticket
counters and partial slots in the context's workspace, and every launch must leave the counters at
zero whatever its grid was.  These tests interleave launches that differ in the number of chunks,
group size, workgroup size, kernel (matrix-core / vector-ALU), dtype, batch raggedness and cache
layout (contiguous / paged) on ONE context and check every result against the oracle, and against
the bits the same case produced on its first visit."""
import ctypes

import pytest
import torch

from oracle import tidal_oracle as O
from paper_2410_05076_amd import tidal
import workloads as W
from parity_util import check_output, check_positions
from test_gpu_parity import DEV, device_layers, host, say

pytestmark = pytest.mark.gpu


class Visit:
    """One workload (one layer of it) with its inputs on the device and the oracle's answers."""

    def __init__(self, name, w, page_size=0, tuning=None):
        self.name, self.w, self.tuning = name, w, tuning or {}
        (self.q, K, V), = device_layers(w, [0])
        self.lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
        qh, Kh, Vh = host(self.q), host(K), host(V)
        if page_size:
            table, num_pages = W.page_table(w, page_size, device=DEV)
            self.K, Kview = W.paginate(K, table, num_pages, page_size, "HND")
            self.V, _ = W.paginate(V, table, num_pages, page_size, "HND")
            self.keep = table
            self.shape = tidal.make_paged_shape(self.q, Kview, table, self.lens, w.max_seq_len,
                                                total_seq_len=sum(w.seq_lens))
        else:
            self.K, self.V = K, V
            self.shape = tidal.make_shape(self.q, K, self.lens, total_seq_len=sum(w.seq_lens))
        self.o_full = O.full(qh, Kh, Vh, w.seq_lens)
        _, self.o_pos, self.o_scores = O.select(qh, Kh, Vh, w.seq_lens, w.k, return_scores=True)
        self.o_sparse = O.sparse(qh, Kh, Vh, w.seq_lens, self.o_pos)
        self.first = None

    def workspace_bytes(self):
        return tidal.lib().td_workspace_bytes(ctypes.byref(self.shape), self.w.k)

    def run(self, td, tag):
        w = self.w
        td.set_tuning(**self.tuning)
        nan = float("nan")
        out_f, out_s, out_p = (torch.full_like(self.q, nan) for _ in range(3))
        pos = torch.full((w.batch, w.num_kv_heads, w.k), -7, dtype=torch.int32, device=DEV)
        say("%s: %s full, select, sparse" % (tag, self.name))
        td.full_attend(self.shape, self.q, self.K, self.V, out_f)
        td.select_tokens(self.shape, self.q, self.K, self.V, w.k, out_s, pos)
        td.sparse_attend(self.shape, self.q, self.K, self.V, pos, w.k, out_p)
        torch.cuda.synchronize()
        check_output(out_f, self.o_full, "%s %s full" % (tag, self.name))
        check_output(out_s, self.o_full, "%s %s select" % (tag, self.name))
        check_positions(pos, self.o_scores, w.seq_lens, w.k, "%s %s" % (tag, self.name))
        if torch.equal(pos.cpu(), self.o_pos):
            check_output(out_p, self.o_sparse, "%s %s sparse" % (tag, self.name))
        else:   # a legal difference inside the band: the oracle on the GPU's own rho
            check_output(out_p, O.sparse(host(self.q), *self.logical(), w.seq_lens, pos.cpu()),
                         "%s %s sparse" % (tag, self.name))
        got = (out_f.clone(), out_s.clone(), out_p.clone(), pos.clone())
        if self.first is None:
            self.first = got
        else:
            for a, b in zip(got, self.first):
                assert torch.equal(a, b), "%s %s: bits differ from the first visit" % (tag, self.name)

    def logical(self):
        (_, K, V), = device_layers(self.w, [0])
        return host(K), host(V)


def visits():
    mk = W.workload
    return [
        # matrix-core kernel, eight waves, ~20 chunks per KV head
        Visit("G4 bf16 5000", mk("c2", context=5000, k=300, n_heavy=32)),
        # ragged batch: four waves, small chunks, sequences of very different chunk counts
        Visit("G1 bf16 ragged", mk("c3", seq_lens=(4100, 130, 2777), num_q_heads=4, num_kv_heads=4, k=200,
                                   tau=256.0)),
        # vector-ALU kernel, fp32, head_dim 64
        Visit("G4 f32 d64 2048", mk("c1")),
        # the same tokens as the first case behind a block table, four waves: twice the chunks
        Visit("G4 bf16 5000 paged16", mk("c2", context=5000, k=300, n_heavy=32), page_size=16,
              tuning=dict(kernel_variant=4, max_splits=128, target_workgroups=2048)),
        # groups of eight (sparse layer with eight waves), one chunk only for the sparse layer
        Visit("G8 bf16 3000", mk("c6", context=3000, k=128, n_heavy=16)),
        # forced vector-ALU kernel with eight waves on the first shape: other chunk length, same counters
        Visit("G4 bf16 5000 valu8", mk("c2", context=5000, k=300, n_heavy=32), tuning=dict(kernel_variant=3)),
        # few long chunks
        Visit("G2 bf16 d64 9000", mk("c2", context=9000, k=1000, num_q_heads=4, num_kv_heads=2, head_dim=64,
                                     n_heavy=32), tuning=dict(max_splits=3)),
    ]


def test_one_context_serves_alternating_shapes():
    vs = visits()
    td = tidal.Tidal(vs[0].shape, vs[0].w.k, workspace_bytes=max(v.workspace_bytes() for v in vs))
    order = [0, 1, 2, 3, 4, 5, 6, 3, 0, 6, 2, 5, 1, 4, 0, 3, 3, 1, 6, 4, 2, 0]
    for step, i in enumerate(order):
        vs[i].run(td, "visit %d" % step)
    td.close()


def test_reset_between_launches_changes_nothing():
    vs = visits()[:3]
    td = tidal.Tidal(vs[0].shape, vs[0].w.k, workspace_bytes=max(v.workspace_bytes() for v in vs))
    for step, i in enumerate([0, 1, 2, 0, 1, 2]):
        if step % 2:
            td.reset()
        vs[i].run(td, "reset visit %d" % step)
    td.close()


def test_probe_leaves_the_workspace_alone():
    """The streaming probe between attention launches: same bits before and after."""
    v = visits()[0]
    td = tidal.Tidal(v.shape, v.w.k)
    v.run(td, "before probe")
    src = torch.full((1 << 22,), 0x9E, dtype=torch.uint8, device=DEV)
    dst = torch.empty_like(src)
    td.probe_stream(src)
    td.probe_stream(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    v.run(td, "after probe")
    td.close()
