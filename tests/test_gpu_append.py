"""GPU parity for the fused C.append(k, v) of Alg. 1 (td_decode_step_append): every layer's
launch first stores the current token's key and value as row seq_lens[b] - 1 of its cache and
attends over the cache including it.  The caches start with garbage (NaN) in that row; the
oracle appends with its own function and then runs its ordinary step."""
import pytest
import torch

from oracle import tidal_oracle as O
from paper_2410_05076_amd import tidal
import workloads as W
from parity_util import check_output, check_positions, same_positions
from test_gpu_parity import DEV, device_layers, host, say

pytestmark = pytest.mark.gpu
D, S, P = W.DENSE, W.SELECT, W.SPARSE


def split_last_row(w, K, V):
    """Takes the current token's row out of a cache: returns (k_new, v_new) [B][Hkv][d] and leaves NaN."""
    kn = torch.stack([K[b, :, n - 1].clone() for b, n in enumerate(w.seq_lens)])
    vn = torch.stack([V[b, :, n - 1].clone() for b, n in enumerate(w.seq_lens)])
    for b, n in enumerate(w.seq_lens):
        K[b, :, n - 1] = float("nan")
        V[b, :, n - 1] = float("nan")
    return kn.contiguous(), vn.contiguous()


def favour_current_token(w, q, K):
    """Rewrites the current token's key so that every head of the group scores it far above the rest
    (6 standard deviations for the group sum): it is then in every rho and sparse layers gather it."""
    G = w.group
    for b, n in enumerate(w.seq_lens):
        u = q[b].float().view(w.num_kv_heads, G, w.head_dim).sum(1)
        K[b, :, n - 1] = (6.0 * u / u.norm(dim=-1, keepdim=True)).to(K.dtype)


def run_append(w, schedule, page_size=0, layout="HND", kernel_variant=0, selection=0, force_last=True):
    layers = device_layers(w, range(len(schedule)))
    if force_last:
        for q, K, V in layers:
            favour_current_token(w, q, K)
    full = [(host(K), host(V)) for _, K, V in layers]            # what the caches must become
    qs = [q for q, _, _ in layers]
    news = [split_last_row(w, K, V) for _, K, V in layers]
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    rows = w.num_q_heads if selection == tidal.SELECT_PER_HEAD else w.num_kv_heads
    if page_size:
        table, num_pages = W.page_table(w, page_size, device=DEV)
        pools = [(W.paginate(K, table, num_pages, page_size, layout), W.paginate(V, table, num_pages, page_size, layout))
                 for _, K, V in layers]
        Ks, Vs = [k[0] for k, _ in pools], [v[0] for _, v in pools]
        views = [(k[1], v[1]) for k, v in pools]
        shape = tidal.make_paged_shape(qs[0], views[0][0], table, lens, w.max_seq_len, selection=selection,
                                       total_seq_len=sum(w.seq_lens))
    else:
        Ks, Vs = [K for _, K, _ in layers], [V for _, _, V in layers]
        shape = tidal.make_shape(qs[0], Ks[0], lens, selection=selection, total_seq_len=sum(w.seq_lens))
    td = tidal.Tidal(shape, w.k)
    if kernel_variant:
        td.set_tuning(kernel_variant=kernel_variant)
    outs = [torch.full_like(q, float("nan")) for q in qs]
    n_sel = max(1, sum(1 for x in schedule if x == S))
    pos = torch.full((n_sel, w.batch, rows, w.k), -7, dtype=torch.int32, device=DEV)
    tag = "append %s page %d v%d sel %d" % (w.name, page_size, kernel_variant, selection)
    say(tag)
    td.decode_step_append(shape, schedule, qs, [a for a, _ in news], [b for _, b in news], Ks, Vs, w.k, outs, pos)
    torch.cuda.synchronize()
    slot = -1
    for i, kind in enumerate(schedule):
        # the cache now holds the appended row, bit for bit, and nothing else changed
        if page_size:
            Kl = O.gather_pages(host(views[i][0]), host(table), w.seq_lens, w.max_seq_len)
            Vl = O.gather_pages(host(views[i][1]), host(table), w.seq_lens, w.max_seq_len)
        else:
            Kl, Vl = host(Ks[i]), host(Vs[i])
        for b, n in enumerate(w.seq_lens):
            assert torch.equal(Kl[b, :, :n].view(torch.int16 if Kl.dtype == torch.bfloat16 else torch.int32),
                               full[i][0][b, :, :n].view(torch.int16 if Kl.dtype == torch.bfloat16 else torch.int32))
            assert torch.equal(Vl[b, :, :n].view(torch.int16 if Kl.dtype == torch.bfloat16 else torch.int32),
                               full[i][1][b, :, :n].view(torch.int16 if Kl.dtype == torch.bfloat16 else torch.int32))
        # the oracle: its own append into a cache whose last row is garbage, then its ordinary functions
        Ko, Vo = full[i][0].clone(), full[i][1].clone()
        for b, n in enumerate(w.seq_lens):
            Ko[b, :, n - 1] = float("nan")
            Vo[b, :, n - 1] = float("nan")
        O.append(Ko, Vo, host(news[i][0]), host(news[i][1]), w.seq_lens)
        qh = host(qs[i])
        if kind == D:
            ref = O.full(qh, Ko, Vo, w.seq_lens)
        elif kind == S:
            slot += 1
            if selection:
                ref, o_pos, o_scores = O.select_variant(qh, Ko, Vo, w.seq_lens, w.k, selection)
            else:
                ref, o_pos, o_scores = O.select(qh, Ko, Vo, w.seq_lens, w.k, return_scores=True)
            check_positions(pos[slot], o_scores, w.seq_lens, w.k, tag)
            if force_last:      # the current token is among the selected ones, so sparse layers gather the new row
                for b, n in enumerate(w.seq_lens):
                    assert (host(pos[slot])[b] == n - 1).any(dim=-1).all(), "%s: current token not selected" % tag
        else:
            sp = O.sparse_per_head if selection == tidal.SELECT_PER_HEAD else O.sparse
            ref = sp(qh, Ko, Vo, w.seq_lens, host(pos[slot]))
        check_output(outs[i], ref, "%s L%d" % (tag, i))
    td.close()


def recent(name, **over):
    # recency-weighted keys: the current token scores highest, so every rho contains it
    return W.workload("c3", **over) if name == "c3" else W.workload(name, **over)


@pytest.mark.parametrize("name,over,force_last", [
    ("c3", dict(context=5000, k=300, tau=64.0), True),                                   # G = 1
    ("c3", dict(context=4099, k=256, tau=64.0, num_kv_heads=8), True),                  # G = 4, matrix-core kernel
    ("c3", dict(context=3000, k=200, tau=64.0, num_q_heads=64, num_kv_heads=8), True),  # G = 8
    ("c3", dict(seq_lens=(777, 64, 1, 2500), k=128, tau=32.0, num_kv_heads=8), False),  # ragged, N = 1
    ("c1", dict(context=1500, k=128), False),                                           # fp32: vector-ALU kernel
])
def test_append_step(name, over, force_last):
    run_append(recent(name, **over), (D, S, P, P), force_last=force_last)


@pytest.mark.parametrize("variant", [2, 3, 4, 5])
def test_append_on_each_kernel(variant):
    run_append(W.workload("c3", context=4500, k=300, tau=64.0, num_kv_heads=8), (D, S, P), kernel_variant=variant)


@pytest.mark.parametrize("page_size,layout", [(16, "HND"), (16, "NHD"), (1, "HND"), (256, "HND")])
def test_append_paged(page_size, layout):
    run_append(W.workload("c3", context=4099, k=256, tau=64.0, num_kv_heads=8), (D, S, P), page_size=page_size,
               layout=layout)
    run_append(W.workload("c1", context=700, k=64), (D, S, P), page_size=page_size, layout=layout, force_last=False)


def test_append_with_per_head_selection():
    run_append(W.workload("c3", context=3000, k=200, tau=64.0, num_kv_heads=8), (S, P, P),
               selection=tidal.SELECT_PER_HEAD)


def test_append_step_as_a_hip_graph():
    # the fused append rewrites the same cache row on every replay: replays reproduce the eager result
    w = W.workload("c3", context=3000, k=200, tau=64.0, num_kv_heads=8)
    schedule = (D, S, P, P)
    layers = device_layers(w, range(len(schedule)))
    qs = [q for q, _, _ in layers]
    news = [split_last_row(w, K, V) for _, K, V in layers]
    Ks, Vs = [K for _, K, _ in layers], [V for _, _, V in layers]
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(qs[0], Ks[0], lens)
    td = tidal.Tidal(shape, w.k)
    outs = [torch.full_like(q, float("nan")) for q in qs]
    pos = torch.full((1, w.batch, w.num_kv_heads, w.k), -7, dtype=torch.int32, device=DEV)
    args = (shape, schedule, qs, [a for a, _ in news], [b for _, b in news], Ks, Vs, w.k, outs, pos)
    td.decode_step_append(*args)
    torch.cuda.synchronize()
    eager_outs, eager_pos = [o.clone() for o in outs], pos.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        td.decode_step_append(*args)
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan"))
        pos.fill_(-7)
        for K, V in zip(Ks, Vs):            # forget the appended row: the replay must write it again
            K[0, :, w.seq_lens[0] - 1] = float("nan")
            V[0, :, w.seq_lens[0] - 1] = float("nan")
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(pos, eager_pos), "replay %d" % rep
        for a, b in zip(outs, eager_outs):
            assert torch.equal(a, b), "replay %d" % rep
        for (kn, vn), K, V in zip(news, Ks, Vs):
            assert torch.equal(K[0, :, w.seq_lens[0] - 1], kn[0]) and torch.equal(V[0, :, w.seq_lens[0] - 1], vn[0])
    td.close()
