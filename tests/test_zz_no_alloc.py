"""td_decode_step_static (the entry point that allocates nothing) against td_decode_step on the same
inputs, through the C ABI: two calls in a row on the static scratch, the second with a smaller
input, each compared bit for bit with the context-based call and with the oracle."""
import ctypes

import pytest
import torch

from oracle import tidal_oracle as O
from paper_2410_05076_amd import tidal
import workloads as W
from parity_util import check_output, check_positions
from test_gpu_parity import DEV, device_layers, host, say

pytestmark = pytest.mark.gpu
D, S, P = W.DENSE, W.SELECT, W.SPARSE


def both_ways(w, tag):
    layers = device_layers(w, range(w.num_layers))
    qs, Ks, Vs = zip(*layers)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(qs[0], Ks[0], lens, total_seq_len=sum(w.seq_lens))
    n_sel = sum(1 for x in w.schedule if x == S)
    need = tidal.lib().td_workspace_bytes(ctypes.byref(shape), w.k)
    assert 0 < need <= tidal.STATIC_SCRATCH_BYTES, need

    def fresh():
        return ([torch.full_like(q, float("nan")) for q in qs],
                torch.full((n_sel, w.batch, w.num_kv_heads, w.k), -7, dtype=torch.int32, device=DEV))

    say("%s: static entry point" % tag)
    outs_s, pos_s = fresh()
    tidal.decode_step_static(shape, w.schedule, qs, Ks, Vs, w.k, outs_s, pos_s)
    torch.cuda.synchronize()
    say("%s: context entry point" % tag)
    td = tidal.Tidal(shape, w.k)
    outs_c, pos_c = fresh()
    td.decode_step(shape, w.schedule, qs, Ks, Vs, w.k, outs_c, pos_c)
    torch.cuda.synchronize()
    td.close()
    assert torch.equal(pos_s, pos_c), "%s: positions differ between the two entry points" % tag
    for i in range(w.num_layers):
        assert torch.equal(outs_s[i], outs_c[i]), "%s: layer %d differs between the two entry points" % (tag, i)
    # and against the oracle, so that two equal wrong answers cannot pass
    o_outs, o_pos = O.step(w.schedule, [host(t) for t in qs], [host(t) for t in Ks], [host(t) for t in Vs],
                           w.seq_lens, w.k)
    sel = 0
    for i, kind in enumerate(w.schedule):
        if kind == S:
            _, _, scores = O.select(host(qs[i]), host(Ks[i]), host(Vs[i]), w.seq_lens, w.k, return_scores=True)
            check_positions(pos_s[sel], scores, w.seq_lens, w.k, "%s L%d" % (tag, i))
            sel += 1
    if torch.equal(pos_s.cpu(), o_pos):
        for i in range(w.num_layers):
            check_output(outs_s[i], o_outs[i], "%s L%d" % (tag, i))
    else:
        for i, kind in enumerate(w.schedule):
            if kind != P:
                check_output(outs_s[i], o_outs[i], "%s L%d" % (tag, i))


def test_static_entry_matches_the_context_entry_twice_in_a_row():
    sched = (D, S, P, P, S, P)
    # first a batch of three ragged sequences, then a single shorter one: the second call finds the
    # scratch as the first one left it
    both_ways(W.workload("c2", seq_lens=(6000, 4097, 2500), k=384, n_heavy=48, schedule=sched), "first call")
    both_ways(W.workload("c2", context=1500, k=200, n_heavy=32, schedule=sched), "second, smaller call")
    both_ways(W.workload("c1"), "third call, fp32")


def test_static_entry_refuses_what_does_not_fit():
    w = W.workload("c4", schedule=(D, S, P))
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    q = torch.zeros((w.batch, w.num_q_heads, w.head_dim), dtype=torch.bfloat16, device=DEV)
    K = torch.zeros((16,), dtype=torch.bfloat16, device=DEV)   # never read: the call must refuse on the host
    n, d = w.max_seq_len, w.head_dim
    shape = tidal.Shape(w.batch, w.num_q_heads, w.num_kv_heads, d, tidal.BF16, 0.0, w.num_kv_heads * n * d, n * d, d,
                        lens.data_ptr(), n, 0, 0, 0, None, 0, 0)
    assert tidal.lib().td_workspace_bytes(ctypes.byref(shape), w.k) > tidal.STATIC_SCRATCH_BYTES
    out = torch.zeros_like(q)
    pos = torch.zeros((1, w.batch, w.num_kv_heads, w.k), dtype=torch.int32, device=DEV)
    with pytest.raises(tidal.TidalError) as e:
        tidal.decode_step_static(shape, w.schedule, [q] * 3, [K] * 3, [K] * 3, w.k, [out] * 3, pos)
    assert e.value.status == tidal.ERR_WORKSPACE
    assert "TD_STATIC_SCRATCH_BYTES" in str(e.value)
