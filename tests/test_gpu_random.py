"""Seeded random sweep over small shapes: context lengths around chunk and tile boundaries, ragged
batches, every group size, both dtypes and head dims, paged or contiguous caches, every selection
rule, with and without the fused append, one decode step each (full, selection, two sparse layers)
against the oracle."""
import random

import pytest
import torch

from oracle import tidal_oracle as O
from paper_2410_05076_amd import tidal
import workloads as W
from parity_util import check_output, check_positions
from test_gpu_parity import DEV, device_layers, host, say

pytestmark = pytest.mark.gpu
D, S, P = W.DENSE, W.SELECT, W.SPARSE
SCHEDULE = (D, S, P, P)
EDGE_LENGTHS = [1, 2, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025,
                2047, 2048, 2049, 4095, 4096, 4097]


def draw_case(rng):
    dtype = rng.choice(["bf16", "bf16", "f32"])
    head_dim = rng.choice([64, 128])
    group = rng.choice([1, 2, 4, 8])
    hkv = rng.choice([1, 2, 3])
    batch = rng.choice([1, 1, 2, 5])
    lens = tuple(rng.choice(EDGE_LENGTHS) if rng.random() < 0.7 else rng.randint(1, 6000) for _ in range(batch))
    k = rng.choice([1, 7, 64, 128, 129, 300, 2048, 2500])
    return dict(dtype=dtype, head_dim=head_dim, num_q_heads=group * hkv, num_kv_heads=hkv, seq_lens=lens, k=k,
                page_size=rng.choice([0, 0, 1, 8, 16, 128]), layout=rng.choice(["HND", "NHD"]),
                selection=rng.choice([0, 0, 1, 2, 3]), append=rng.random() < 0.5,
                variant=rng.choice([0, 0, 0, 2, 3, 4, 5]))


def run_case(c, tag):
    w = W.workload("c4", seq_lens=c["seq_lens"], k=c["k"], dtype=c["dtype"], head_dim=c["head_dim"],
                   num_q_heads=c["num_q_heads"], num_kv_heads=c["num_kv_heads"], schedule=SCHEDULE,
                   n_heavy=min(8, min(c["seq_lens"])))
    layers = device_layers(w, range(len(SCHEDULE)))
    truth = [(host(K), host(V)) for _, K, V in layers]
    qs = [q for q, _, _ in layers]
    news = None
    if c["append"]:                    # take the current token's rows out of the caches
        news = []
        for _, K, V in layers:
            kn = torch.stack([K[b, :, n - 1].clone() for b, n in enumerate(w.seq_lens)]).contiguous()
            vn = torch.stack([V[b, :, n - 1].clone() for b, n in enumerate(w.seq_lens)]).contiguous()
            for b, n in enumerate(w.seq_lens):
                K[b, :, n - 1] = float("nan")
                V[b, :, n - 1] = float("nan")
            news.append((kn, vn))
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    if c["page_size"]:
        table, num_pages = W.page_table(w, c["page_size"], device=DEV)
        pools = [(W.paginate(K, table, num_pages, c["page_size"], c["layout"]),
                  W.paginate(V, table, num_pages, c["page_size"], c["layout"])) for _, K, V in layers]
        Ks, Vs = [a[0] for a, _ in pools], [b[0] for _, b in pools]
        shape = tidal.make_paged_shape(qs[0], pools[0][0][1], table, lens, w.max_seq_len, selection=c["selection"],
                                       total_seq_len=sum(w.seq_lens))
    else:
        Ks, Vs = [K for _, K, _ in layers], [V for _, _, V in layers]
        shape = tidal.make_shape(qs[0], Ks[0], lens, selection=c["selection"], total_seq_len=sum(w.seq_lens))
    td = tidal.Tidal(shape, w.k)
    if c["variant"]:
        td.set_tuning(kernel_variant=c["variant"])
    rows = w.num_q_heads if c["selection"] == tidal.SELECT_PER_HEAD else w.num_kv_heads
    outs = [torch.full_like(q, float("nan")) for q in qs]
    pos = torch.full((1, w.batch, rows, w.k), -7, dtype=torch.int32, device=DEV)
    say("%s: %s" % (tag, c))
    if news:
        td.decode_step_append(shape, SCHEDULE, qs, [a for a, _ in news], [b for _, b in news], Ks, Vs, w.k, outs, pos)
    else:
        td.decode_step(shape, SCHEDULE, qs, Ks, Vs, w.k, outs, pos)
    torch.cuda.synchronize()
    for i, kind in enumerate(SCHEDULE):
        qh, (Kh, Vh) = host(qs[i]), truth[i]
        if kind == D:
            ref = O.full(qh, Kh, Vh, w.seq_lens)
        elif kind == S:
            if c["selection"]:
                ref, o_pos, o_scores = O.select_variant(qh, Kh, Vh, w.seq_lens, w.k, c["selection"])
            else:
                ref, o_pos, o_scores = O.select(qh, Kh, Vh, w.seq_lens, w.k, return_scores=True)
            check_positions(pos[0], o_scores, w.seq_lens, w.k, tag, relative_band=c["selection"] == 3)
        else:
            sp = O.sparse_per_head if c["selection"] == tidal.SELECT_PER_HEAD else O.sparse
            ref = sp(qh, Kh, Vh, w.seq_lens, host(pos[0]))
        check_output(outs[i], ref, "%s L%d" % (tag, i))
    td.close()


@pytest.mark.parametrize("seed", range(120))
def test_random_small_step(seed):
    run_case(draw_case(random.Random(1000 + seed)), "random %d" % seed)
