"""GPU parity at the benchmark configurations' full sizes, through td_decode_step in the
launch configuration bench.py times (one call for all layers, eager and as a HIP graph).

The oracle checks one layer at a time (one layer's K and V on the host at once): every layer of
c2, c3, c4, c6 and of c5 at k = 4096 (the other budgets of c5 and the paged c2 run a sample).  Sparse
layers are compared with the oracle run on the positions the GPU selected, after those
positions have passed the position rule against the oracle's own scores (rows whose k-th score is
clear of the (k+1)-th by more than the band must be the oracle's bit for bit); the first sparse layer
checked after each selection layer is also compared with the oracle run on the oracle's own positions.
"""
import gc
import sys
import time

import pytest
import torch

from oracle import tidal_oracle as O
from paper_2410_05076_amd import tidal
import workloads as W
from parity_util import check_output, check_positions, same_positions

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def free():
    gc.collect()
    torch.cuda.empty_cache()


def run_step(w, sparse_to_check, graph=False, tag="", page_size=0):
    t0 = time.time()
    heavy = W.heavy_positions(w)
    ranks = W.zipf_ranks(w) if w.structure == "zipf" else None
    layers = [W.make_layer(w, i, DEV, heavy=heavy, ranks=ranks) for i in range(w.num_layers)]
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    if page_size:   # the same tokens in a shuffled page pool; the oracle gathers them back itself
        table, num_pages = W.page_table(w, page_size, device=DEV)
        paged = []
        for q, K, V in layers:
            Kp, Kv = W.paginate(K, table, num_pages, page_size)
            Vp, _ = W.paginate(V, table, num_pages, page_size)
            paged.append((q, Kp, Vp))
        layers = paged
        del paged, K, V
        shape = tidal.make_paged_shape(layers[0][0], Kv, table, lens, w.max_seq_len, total_seq_len=sum(w.seq_lens))
    qs, Ks, Vs = zip(*layers)
    del layers
    if not page_size:
        shape = tidal.make_shape(qs[0], Ks[0], lens, total_seq_len=sum(w.seq_lens))
    td = tidal.Tidal(shape, w.k)
    outs = [torch.full_like(q, float("nan")) for q in qs]
    n_sel = sum(1 for x in w.schedule if x == W.SELECT)
    pos = torch.full((n_sel, w.batch, w.num_kv_heads, w.k), -7, dtype=torch.int32, device=DEV)
    torch.cuda.synchronize()
    say("%s: inputs ready after %.1f s" % (tag, time.time() - t0))
    td.decode_step(shape, w.schedule, qs, Ks, Vs, w.k, outs, pos)
    torch.cuda.synchronize()
    if graph:
        # replay a captured step several times with eager work in between; every replay must
        # reproduce the eager result bit for bit
        eager_outs = [o.clone() for o in outs]
        eager_pos = pos.clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            td.decode_step(shape, w.schedule, qs, Ks, Vs, w.k, outs, pos)
        for rep in range(3):
            for o in outs:
                o.fill_(float("nan"))
            pos.fill_(-7)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(pos, eager_pos), "replay %d: positions differ from eager" % rep
            for i in range(w.num_layers):
                assert torch.equal(outs[i], eager_outs[i]), "replay %d: layer %d differs from eager" % (rep, i)
        say("%s: 3 graph replays identical to eager" % tag)
        del g
    slot = -1
    exact, decided, own_rho = [], [], {}
    for i, kind in enumerate(w.schedule):
        if kind == W.SPARSE and i not in sparse_to_check:
            continue
        q, K, V = qs[i].cpu(), Ks[i].cpu(), Vs[i].cpu()
        if page_size:
            K = O.gather_pages(K, table.cpu(), w.seq_lens, w.max_seq_len)
            V = O.gather_pages(V, table.cpu(), w.seq_lens, w.max_seq_len)
        if kind == W.DENSE:
            ref = O.full(q, K, V, w.seq_lens)
        elif kind == W.SELECT:
            slot += 1
            ref, o_pos, o_scores = O.select(q, K, V, w.seq_lens, w.k, return_scores=True)
            rows, clear = check_positions(pos[slot], o_scores, w.seq_lens, w.k, "%s L%d" % (tag, i), oracle_pos=o_pos)
            exact.append(same_positions(pos[slot], o_pos))
            decided.append("%d of %d rows clear of the band" % (clear, rows))
            own_rho[slot] = o_pos
        else:
            cur = sum(1 for x in w.schedule[:i] if x == W.SELECT) - 1
            ref = O.sparse(q, K, V, w.seq_lens, pos[cur].cpu())
            if cur in own_rho:   # once per selection layer: the oracle on its own positions
                check_output(outs[i], O.sparse(q, K, V, w.seq_lens, own_rho.pop(cur)), "%s L%d, oracle's own rho" % (tag, i))
        ma, rel = check_output(outs[i], ref, "%s L%d" % (tag, i))
        say("%s: layer %2d kind %d max-abs %.2e rel-L2 %.2e" % (tag, i, kind, ma, rel))
    say("%s: positions identical to the oracle's per selection layer: %s, %s (%.1f s)"
        % (tag, exact, decided, time.time() - t0))
    td.close()
    del qs, Ks, Vs, outs, pos
    free()


def test_c2_full_decode_step_eager_and_graph():
    w = W.workload("c2")
    run_step(w, set(range(w.num_layers)), graph=True, tag="c2")


def test_c2_paged_decode_step_eager_and_graph():
    w = W.workload("c2")
    run_step(w, {3, 12, 14, 31}, graph=True, tag="c2 pages of 16", page_size=16)


def test_c3_full_size():
    w = W.workload("c3")
    run_step(w, set(range(w.num_layers)), tag="c3")


def test_c4_full_size_ragged_batch():
    w = W.workload("c4")
    run_step(w, set(range(w.num_layers)), tag="c4")


def test_c6_sixty_four_layers_eight_heads_per_group():
    # the 64-layer schedule of Sec. 4.3 with the 70B head shape: 2 full, selection at layers 2 and 31, 60 sparse
    w = W.workload("c6")
    run_step(w, set(range(w.num_layers)), graph=True, tag="c6")


def test_c5_whole_schedule_at_the_middle_budget():
    w = W.workload("c5", k=4096)
    run_step(w, set(range(w.num_layers)), tag="c5 k=4096, 32 layers")


@pytest.mark.parametrize("k", [256, 1024, 4096, 16384])
def test_c5_budget_sweep(k):
    # the cache does not depend on k; a shorter schedule keeps one full, both kinds of
    # selection-to-sparse hand-over and the re-selection in the step
    w = W.workload("c5", k=k, schedule=(W.DENSE, W.SELECT, W.SPARSE, W.SELECT, W.SPARSE, W.SPARSE))
    run_step(w, {2, 4, 5}, tag="c5 k=%d" % k)
