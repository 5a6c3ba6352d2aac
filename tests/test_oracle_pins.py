"""Pins for the CPU oracle: brute force in float64, closed forms, invariants.

The paper prints no scores, positions or outputs, so the oracle is pinned to
the mathematics of Eq. 1 and Alg. 1 instead: an independent float64 NumPy
evaluation on tiny inputs, cases whose answer is known in closed form, and
the invariants the method states (ordering invariance of softmax, k = N
sparse attention equals full attention).
"""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import tidal_oracle as O
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_case(seed, B=2, Hq=4, Hkv=2, d=8, N=33, dtype=torch.float32, lens=None):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn((B, Hq, d), generator=g).to(dtype)
    K = torch.randn((B, Hkv, N, d), generator=g).to(dtype)
    V = torch.randn((B, Hkv, N, d), generator=g).to(dtype)
    return q, K, V, (lens if lens is not None else [N] * B)


def brute_logits(q, K, lens, scale=None):
    """float64 scaled logits [B][Hq][N] (NaN beyond a sequence's length), by definition."""
    q64, K64 = q.double().numpy(), K.double().numpy()
    B, Hq, d = q64.shape
    G = Hq // K64.shape[1]
    scale = scale if scale else 1.0 / math.sqrt(d)
    s = np.full((B, Hq, K64.shape[2]), np.nan)
    for b in range(B):
        for h in range(Hq):
            s[b, h, :lens[b]] = (K64[b, h // G, :lens[b]] @ q64[b, h]) * scale
    return s


def brute_attention(q, K, V, lens, rows=None, scale=None):
    """float64 softmax(q K^T / sqrt d) V restricted to rows[b][g] (default: all rows)."""
    s = brute_logits(q, K, lens, scale)
    V64 = V.double().numpy()
    B, Hq, d = q.shape
    G = Hq // K.shape[1]
    out = np.zeros((B, Hq, d))
    for b in range(B):
        for h in range(Hq):
            idx = np.arange(lens[b]) if rows is None else np.asarray(rows[b][h // G])
            idx = idx[idx >= 0]
            if len(idx) == 0:
                continue
            z = s[b, h, idx]
            p = np.exp(z - z.max())
            p /= p.sum()
            out[b, h] = p @ V64[b, h // G, idx]
    return out


# ---------------------------------------------------------------- full attention

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [dict(B=2, Hq=4, Hkv=2, d=8, N=33),
                                   dict(B=1, Hq=6, Hkv=6, d=16, N=17),
                                   dict(B=3, Hq=8, Hkv=2, d=4, N=29, lens=[29, 1, 13])])
def test_full_matches_float64_brute_force(dtype, shape):
    q, K, V, lens = rand_case(1, dtype=dtype, **shape)
    out = O.full(q, K, V, lens)
    ref = brute_attention(q, K, V, lens)
    assert np.abs(out.numpy() - ref).max() <= 1e-5


def test_full_hand_worked_example():
    # d = 2, scale chosen so that the logits are ln 1, ln 2, ln 3: the softmax weights are
    # exactly 1/6, 2/6, 3/6 and the output is a rational combination of the V rows.
    q = torch.tensor([[[1.0, 0.0]]])
    K = torch.tensor([[[[math.log(1.0), 5.0], [math.log(2.0), -3.0], [math.log(3.0), 0.5]]]])
    V = torch.tensor([[[[6.0, 0.0], [0.0, 12.0], [-6.0, 2.0]]]])
    out = O.full(q, K, V, [3], sm_scale=1.0)
    np.testing.assert_allclose(out.numpy()[0, 0], [1.0 - 3.0, 4.0 + 1.0], atol=2e-6)
    # default scale is 1/sqrt(d): feeding sqrt(2) q gives the same logits
    out2 = O.full(q * math.sqrt(2.0), K, V, [3])
    np.testing.assert_allclose(out2.numpy()[0, 0], [-2.0, 5.0], atol=5e-6)


def test_full_closed_forms():
    q, K, V, lens = rand_case(2, B=1, Hq=2, Hkv=1, d=8, N=40)
    # all keys equal: uniform weights, output is the mean of the V rows
    Ke = K[:, :, :1].expand(-1, -1, 40, -1).contiguous()
    out = O.full(q, Ke, V, lens)
    np.testing.assert_allclose(out.numpy()[0, 0], V[0, 0].double().mean(0).numpy(), atol=2e-6)
    # one key far above the rest (logit gap > 50 for head 0): output is that V row
    Kd = K.clone()
    Kd[0, 0, 7] = q[0, 0] * (80.0 * math.sqrt(8) / float(q[0, 0] @ q[0, 0]))
    out = O.full(q, Kd, V, lens)
    np.testing.assert_allclose(out.numpy()[0, 0], V[0, 0, 7].numpy(), atol=1e-6)


def test_full_shift_invariance_and_gqa_mapping():
    # adding the same vector to every key shifts each head's logits by a constant
    q, K, V, lens = rand_case(3, B=1, Hq=4, Hkv=2, d=8, N=21)
    w = torch.randn(8, generator=torch.Generator().manual_seed(9))
    a, b = O.full(q, K, V, lens), O.full(q, K + w, V, lens)
    assert (a - b).abs().max() <= 1e-5
    # GQA: head h reads KV head h // G - repeat the KV heads and run as MHA
    Kr, Vr = K.repeat_interleave(2, dim=1), V.repeat_interleave(2, dim=1)
    c = O.full(q, Kr, Vr, lens)
    assert torch.equal(a, c)


def test_full_honours_strides_and_ignores_rows_beyond_length():
    q, K, V, lens = rand_case(4, B=2, Hq=4, Hkv=2, d=8, N=24, lens=[24, 10])
    ref = O.full(q, K, V, lens)
    Kp, Vp = K.clone(), V.clone()
    Kp[1, :, 10:], Vp[1, :, 10:] = float("nan"), float("nan")
    assert torch.equal(O.full(q, Kp, Vp, lens), ref)
    # token-major storage [B][N][Hkv][d] viewed as [B][Hkv][N][d]
    Kt = K.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    Vt = V.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not Kt.is_contiguous()
    assert torch.equal(O.full(q, Kt, Vt, lens), ref)


def test_split_merge_identity():
    # (m, l, o) of two halves merged by the softmax rescaling rule equals the whole; this is
    # the identity a split-K evaluation of Eq. 1 relies on, derived here from Eq. 1 itself.
    q, K, V, lens = rand_case(5, B=1, Hq=2, Hkv=1, d=8, N=50)
    whole, logits = O.full(q, K, V, lens, return_logits=True)
    first = torch.arange(0, 23, dtype=torch.int32).view(1, 1, -1)
    second = torch.arange(23, 50, dtype=torch.int32).view(1, 1, -1)
    o1, o2 = O.sparse(q, K, V, lens, first), O.sparse(q, K, V, lens, second)
    for h in range(2):
        s = logits[0, h].double()
        m1, m2 = s[:23].max(), s[23:].max()
        l1, l2 = torch.exp(s[:23] - m1).sum(), torch.exp(s[23:] - m2).sum()
        m = max(m1, m2)
        w1, w2 = l1 * torch.exp(m1 - m), l2 * torch.exp(m2 - m)
        merged = (w1 * o1[0, h].double() + w2 * o2[0, h].double()) / (w1 + w2)
        assert (merged - whole[0, h].double()).abs().max() <= 1e-6


# ---------------------------------------------------------------- selection

def test_select_g1_equals_topk_of_softmax_probabilities():
    # Sec. 3.1: top-k on the inner products equals top-k on the post-softmax scores
    q, K, V, lens = rand_case(6, B=2, Hq=3, Hkv=3, d=16, N=64)
    out, pos = O.select(q, K, V, lens, 9)
    s = brute_logits(q, K, lens)
    for b in range(2):
        for h in range(3):
            p = np.exp(s[b, h] - s[b, h].max())
            p /= p.sum()
            want = np.sort(np.argsort(-p, kind="stable")[:9])
            assert pos[b, h].tolist() == want.tolist()
    assert torch.equal(out, O.full(q, K, V, lens))


def test_select_gqa_uses_sum_of_group_logits():
    q, K, V, lens = rand_case(7, B=2, Hq=8, Hkv=2, d=16, N=80, lens=[80, 37])
    out, pos, scores = O.select(q, K, V, lens, 12, return_scores=True)
    s = brute_logits(q, K, lens)
    for b in range(2):
        for g in range(2):
            r = s[b, 4 * g:4 * g + 4, :lens[b]].sum(0)
            np.testing.assert_allclose(scores[b, g, :lens[b]].numpy(), r, atol=1e-5)
            want = np.sort(np.argsort(-r, kind="stable")[:12])
            assert pos[b, g].tolist() == want.tolist()
            # gap at the boundary is far above fp32 noise, so the float64 ranking is decisive
            srt = np.sort(r)[::-1]
            assert srt[11] - srt[12] > 1e-4


def test_select_positions_are_valid_and_padded():
    q, K, V, lens = rand_case(8, B=2, Hq=4, Hkv=2, d=8, N=30, lens=[30, 5])
    _, pos = O.select(q, K, V, lens, 8)
    for g in range(2):
        a = pos[0, g].tolist()
        assert len(set(a)) == 8 and a == sorted(a) and 0 <= a[0] and a[-1] < 30
        assert pos[1, g].tolist() == [0, 1, 2, 3, 4, -1, -1, -1]     # k > N: all tokens, -1 tail
    _, pos = O.select(q, K, V, [30, 30], 30)
    assert all(pos[b, g].tolist() == list(range(30)) for b in range(2) for g in range(2))


def test_select_ties_go_to_smaller_index():
    q, K, V, lens = rand_case(9, B=1, Hq=2, Hkv=1, d=8, N=12)
    K[0, 0, 3] = K[0, 0, 9] = K[0, 0, 6] = q[0, 0] + q[0, 1]       # three identical, dominant rows
    K[0, 0, 3] *= 1.0
    _, pos = O.select(q, K * 1.0, V, lens, 2)
    assert pos[0, 0].tolist() == [3, 6]


def test_select_is_invariant_to_per_head_shifts():
    q, K, V, lens = rand_case(10, B=1, Hq=4, Hkv=1, d=8, N=200)
    w = torch.randn(8, generator=torch.Generator().manual_seed(11)) * 0.5
    _, a, sa = O.select(q, K, V, lens, 16, return_scores=True)
    _, b = O.select(q, K + w, V, lens, 16)
    srt = sa[0, 0].sort(descending=True).values
    assert srt[15] - srt[16] > 1e-4       # boundary not within rounding noise
    assert torch.equal(a, b)


def test_select_finds_planted_heavy_hitters_of_toy_config():
    w = W.workload("c1")
    heavy = W.heavy_positions(w)
    for layer in (1, 2):
        q, K, V = W.make_layer(w, layer, heavy=heavy)
        _, pos = O.select(q, K, V, w.seq_lens, w.k)
        for g in range(w.num_kv_heads):
            assert set(heavy[0, g].tolist()) <= set(pos[0, g].tolist())


@pytest.mark.parametrize("n,k", [(1, 1), (1, 4), (7, 3), (16, 16), (50, 7)])
def test_topk_row_against_sorted(n, k):
    g = torch.Generator().manual_seed(100 + n + k)
    x = torch.randint(0, 6, (n,), generator=g).float()     # many ties
    order = sorted(range(n), key=lambda j: (-float(x[j]), j))[:min(n, k)]
    want = sorted(order) + [-1] * (k - min(n, k))
    assert O.topk_row(x, k).tolist() == want


# ---------------------------------------------------------------- sparse attention

def test_sparse_with_all_positions_reproduces_full_bit_for_bit():
    q, K, V, lens = rand_case(12, B=2, Hq=4, Hkv=2, d=8, N=40, lens=[40, 22], dtype=torch.bfloat16)
    pos = torch.full((2, 2, 40), -1, dtype=torch.int32)
    for b in range(2):
        pos[b, :, :lens[b]] = torch.arange(lens[b], dtype=torch.int32)
    assert torch.equal(O.sparse(q, K, V, lens, pos), O.full(q, K, V, lens))


def test_sparse_matches_brute_force_and_gathered_subcache():
    q, K, V, lens = rand_case(13, B=2, Hq=4, Hkv=2, d=8, N=64)
    g = torch.Generator().manual_seed(14)
    pos = torch.stack([torch.stack([torch.randperm(64, generator=g)[:10].sort().values
                                    for _ in range(2)]) for _ in range(2)]).int()
    pos[1, 0, 7:] = -1
    out = O.sparse(q, K, V, lens, pos)
    ref = brute_attention(q, K, V, lens, rows=pos.numpy())
    assert np.abs(out.numpy() - ref).max() <= 1e-5
    # same thing as full attention over the physically gathered rows
    for b in range(2):
        for gi in range(2):
            idx = pos[b, gi][pos[b, gi] >= 0].long()
            Kg, Vg = K[b:b + 1, gi:gi + 1, idx], V[b:b + 1, gi:gi + 1, idx]
            sub = O.full(q[b:b + 1, 2 * gi:2 * gi + 2], Kg.contiguous(), Vg.contiguous(), [len(idx)])
            assert torch.equal(sub[0], out[b, 2 * gi:2 * gi + 2])
    # order of rho does not matter beyond fp32 reassociation
    perm = pos[:, :, torch.randperm(10, generator=g)]
    assert (O.sparse(q, K, V, lens, perm) - out).abs().max() <= 1e-6


def test_sparse_rejects_positions_beyond_length_and_handles_empty_rho():
    q, K, V, lens = rand_case(15, B=1, Hq=2, Hkv=1, d=8, N=10, lens=[6])
    with pytest.raises(RuntimeError):
        O.sparse(q, K, V, lens, torch.tensor([[[1, 6]]], dtype=torch.int32))
    out = O.sparse(q, K, V, lens, torch.tensor([[[-1, -1]]], dtype=torch.int32))
    assert torch.equal(out, torch.zeros_like(out))


# ---------------------------------------------------------------- the layer loop

def test_step_persists_positions_until_next_selection_layer():
    sched = (W.DENSE, W.SELECT, W.SPARSE, W.SPARSE, W.SELECT, W.SPARSE)
    w = W.workload("c1", context=300, k=20, schedule=sched)
    heavy = W.heavy_positions(w)
    layers = [W.make_layer(w, i, heavy=heavy) for i in range(6)]
    qs, Ks, Vs = zip(*layers)
    outs, pos = O.step(sched, qs, Ks, Vs, w.seq_lens, w.k)
    assert pos.shape == (2, 1, 2, 20)
    for i, slot in ((1, 0), (4, 1)):
        o, p = O.select(qs[i], Ks[i], Vs[i], w.seq_lens, w.k)
        assert torch.equal(p, pos[slot]) and torch.equal(o, outs[i])
    assert torch.equal(outs[0], O.full(qs[0], Ks[0], Vs[0], w.seq_lens))
    for i, slot in ((2, 0), (3, 0), (5, 1)):
        assert torch.equal(outs[i], O.sparse(qs[i], Ks[i], Vs[i], w.seq_lens, pos[slot]))
    assert not torch.equal(pos[0], pos[1])
    with pytest.raises(RuntimeError):
        O.step((W.DENSE, W.SPARSE), qs[:2], Ks[:2], Vs[:2], w.seq_lens, w.k)


def test_paper_constants():
    with open(os.path.join(GOLDEN, "paper_constants.json")) as f:
        c = json.load(f)
    s = W.schedule_for(32)
    counts = [s.count(W.DENSE), s.count(W.SELECT), s.count(W.SPARSE)]
    assert counts == c["layers_32"]["dense_select_sparse"]
    assert [i for i, x in enumerate(s) if x == W.SELECT] == c["selection_layers_llama3_8b"]
    s64 = W.schedule_for(64, select_layers=(2, 31))
    assert [s64.count(W.DENSE), s64.count(W.SELECT), s64.count(W.SPARSE)] == c["layers_64"]["dense_select_sparse"]
    w = W.workload("c3")       # Llama-2-7B shape at 128K tokens: the footnote's 64 GB KV cache
    assert w.num_layers * w.kv_bytes_per_layer() == c["kv_cache_bytes_llama2_7b_128k"] == 64 * 2**30


# ---- paged cache: the mapping (block table, slot) -> logical token, pinned independently


def _toy_pool(num_pages, Hkv, P, d, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn((num_pages, Hkv, P, d), generator=g).to(dtype)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("P", [1, 4, 16])
def test_gather_pages_matches_direct_indexing(dtype, P):
    # the definition written out with plain indexing, no shared code
    Hkv, d, lens = 3, 8, [37, 5, 16]
    N = max(lens)
    pool = _toy_pool(40, Hkv, P, d, dtype, 3)
    g = torch.Generator().manual_seed(4)
    table = torch.stack([torch.randperm(40, generator=g)[: (N + P - 1) // P] for _ in lens]).to(torch.int32)
    got = O.gather_pages(pool, table, lens, N, fill=0.0)
    for b, n in enumerate(lens):
        for j in range(N):
            want = pool[table[b, j // P], :, j % P] if j < n else torch.zeros(Hkv, d, dtype=dtype)
            assert torch.equal(got[b, :, j], want), (b, j)


def test_gather_pages_inverts_the_workload_pagination():
    # the generator's scatter and the oracle's gather are written separately; both layouts
    w = W.workload("c4", seq_lens=(50, 7, 33), k=8)
    q, K, V = W.make_layer(w, 0)
    for P, layout in ((4, "HND"), (16, "NHD"), (1, "HND")):
        table, num_pages = W.page_table(w, P)
        pool, view = W.paginate(K, table, num_pages, P, layout)
        back = O.gather_pages(view, table, w.seq_lens, w.max_seq_len)
        for b, n in enumerate(w.seq_lens):
            assert torch.equal(back[b, :, :n].view(torch.int16), K[b, :, :n].view(torch.int16)), (P, layout, b)
            assert torch.isnan(back[b, :, n:].float()).all()


def test_gather_pages_identity_table_is_a_reshape():
    P, Hkv, d, N = 8, 2, 4, 32
    pool = _toy_pool(N // P, Hkv, P, d, torch.float32, 9)
    table = torch.arange(N // P, dtype=torch.int32)[None]
    got = O.gather_pages(pool, table, [N], N)
    assert torch.equal(got[0], pool.permute(1, 0, 2, 3).reshape(Hkv, N, d))


def test_gather_pages_rejects_a_page_outside_the_pool():
    pool = _toy_pool(4, 1, 4, 4, torch.float32, 1)
    with pytest.raises(RuntimeError):
        O.gather_pages(pool, torch.tensor([[0, 4]], dtype=torch.int32), [8], 8)
    with pytest.raises(RuntimeError):
        O.gather_pages(pool, torch.tensor([[0, -1]], dtype=torch.int32), [8], 8)


def test_paged_full_attention_equals_contiguous_for_any_page_permutation():
    # paging only moves rows: attention over the gathered cache is bit-identical to the original
    w = W.workload("c1", context=200, k=16)
    q, K, V = W.make_layer(w, 1)
    want = O.full(q, K, V, w.seq_lens)
    for seed in (0, 1):
        table, num_pages = W.page_table(w, 16, seed=seed)
        Kp, Kv = W.paginate(K, table, num_pages, 16)
        Vp, Vv = W.paginate(V, table, num_pages, 16)
        got = O.full(q, O.gather_pages(Kv, table, w.seq_lens, w.max_seq_len, fill=0.0),
                          O.gather_pages(Vv, table, w.seq_lens, w.max_seq_len, fill=0.0), w.seq_lens)
        assert torch.equal(got, want)


# ---- other grouped-query selection rules (max over the group, per-head as in Sec. 3.1)


def _small_gqa(seed=5):
    g = torch.Generator().manual_seed(seed)
    B, Hq, Hkv, N, d = 2, 6, 2, 40, 8
    q = torch.randn((B, Hq, d), generator=g)
    K = torch.randn((B, Hkv, N, d), generator=g)
    V = torch.randn((B, Hkv, N, d), generator=g)
    return q, K, V, [40, 23]


def test_per_head_selection_is_the_single_head_rule_applied_to_each_head():
    # repeating each KV head G times turns GQA into MHA, where tdo_select is the paper's per-head rule
    q, K, V, lens = _small_gqa()
    G = q.shape[1] // K.shape[1]
    out, pos, sc = O.select_variant(q, K, V, lens, 7, O.PER_HEAD)
    Kr, Vr = K.repeat_interleave(G, 1), V.repeat_interleave(G, 1)
    out2, pos2, sc2 = O.select(q, Kr, Vr, lens, 7, return_scores=True)
    assert torch.equal(pos, pos2) and torch.equal(out, out2)
    for b, n in enumerate(lens):
        assert torch.equal(sc[b, :, :n], sc2[b, :, :n])
    sp = O.sparse_per_head(q, K, V, lens, pos)
    assert torch.equal(sp, O.sparse(q, Kr, Vr, lens, pos2))


def test_max_reduction_against_float64_ranking():
    q, K, V, lens = _small_gqa(6)
    G = q.shape[1] // K.shape[1]
    out, pos, sc = O.select_variant(q, K, V, lens, 5, O.REDUCE_MAX)
    assert torch.equal(out, O.full(q, K, V, lens))
    for b, n in enumerate(lens):
        for g in range(K.shape[1]):
            s64 = torch.stack([(K[b, g, :n].double() @ q[b, g * G + i].double()) / math.sqrt(q.shape[2])
                               for i in range(G)]).max(0).values
            assert torch.allclose(sc[b, g, :n].double(), s64, atol=1e-5)
            want = sorted(torch.topk(s64, 5).indices.tolist())
            assert pos[b, g].tolist() == want


def test_reductions_coincide_for_a_single_head_per_group():
    g = torch.Generator().manual_seed(7)
    q = torch.randn((1, 3, 8), generator=g)
    K = torch.randn((1, 3, 30, 8), generator=g)
    V = torch.randn((1, 3, 30, 8), generator=g)
    base = O.select(q, K, V, [30], 6)
    for variant in (O.REDUCE_MAX, O.PER_HEAD):
        out, pos, _ = O.select_variant(q, K, V, [30], 6, variant)
        assert torch.equal(pos, base[1]) and torch.equal(out, base[0])


def test_max_and_sum_differ_when_one_head_dominates():
    # token 3 is loved by head 0 and disliked by head 1: the max keeps it, the sum drops it
    d = 4
    q = torch.zeros((1, 2, d)); q[0, 0, 0] = 2.0; q[0, 1, 1] = 2.0
    K = torch.zeros((1, 1, 6, d)); V = torch.zeros((1, 1, 6, d))
    K[0, 0, 3, 0], K[0, 0, 3, 1] = 5.0, -9.0
    K[0, 0, 1, 0], K[0, 0, 1, 1] = 1.0, 1.0
    _, pos_sum = O.select(q, K, V, [6], 1)
    _, pos_max, _ = O.select_variant(q, K, V, [6], 1, O.REDUCE_MAX)
    assert pos_sum[0, 0].tolist() == [1] and pos_max[0, 0].tolist() == [3]


# ---- C.append(k, v) of Alg. 1


def test_append_writes_the_last_row_of_every_sequence_and_nothing_else():
    g = torch.Generator().manual_seed(11)
    B, Hkv, N, d = 3, 2, 20, 8
    lens = [20, 7, 1]
    for dtype in (torch.float32, torch.bfloat16):
        K = torch.randn((B, Hkv, N, d), generator=g).to(dtype)
        V = torch.randn((B, Hkv, N, d), generator=g).to(dtype)
        kn = torch.randn((B, Hkv, d), generator=g).to(dtype)
        vn = torch.randn((B, Hkv, d), generator=g).to(dtype)
        K0, V0 = K.clone(), V.clone()
        O.append(K, V, kn, vn, lens)
        for b, n in enumerate(lens):
            assert torch.equal(K[b, :, n - 1], kn[b]) and torch.equal(V[b, :, n - 1], vn[b])
            keep = [j for j in range(N) if j != n - 1]
            assert torch.equal(K[b, :, keep], K0[b, :, keep]) and torch.equal(V[b, :, keep], V0[b, :, keep])


def test_append_then_attend_equals_attention_over_the_concatenated_cache():
    # Alg. 1 appends first and attends over the whole cache: the new token is visible to itself
    g = torch.Generator().manual_seed(12)
    q = torch.randn((1, 2, 8), generator=g)
    K = torch.randn((1, 2, 10, 8), generator=g)
    V = torch.randn((1, 2, 10, 8), generator=g)
    kn = torch.randn((1, 2, 8), generator=g)
    vn = torch.randn((1, 2, 8), generator=g)
    want = O.full(q, torch.cat([K[:, :, :9], kn[:, :, None]], 2), torch.cat([V[:, :, :9], vn[:, :, None]], 2), [10])
    O.append(K, V, kn, vn, [10])
    assert torch.equal(O.full(q, K, V, [10]), want)


def test_mean_probability_reduction_against_float64_softmax():
    q, K, V, lens = _small_gqa(8)
    G = q.shape[1] // K.shape[1]
    out, pos, sc = O.select_variant(q, K, V, lens, 5, O.REDUCE_MEAN_PROB)
    assert torch.equal(out, O.full(q, K, V, lens))
    for b, n in enumerate(lens):
        for g in range(K.shape[1]):
            p64 = torch.stack([torch.softmax((K[b, g, :n].double() @ q[b, g * G + i].double()) / math.sqrt(q.shape[2]), 0)
                               for i in range(G)]).mean(0)
            assert torch.allclose(sc[b, g, :n].double(), p64, atol=1e-6)
            assert abs(sc[b, g, :n].sum().item() - 1.0) < 1e-5         # a mean of distributions is a distribution
            assert pos[b, g].tolist() == sorted(torch.topk(p64, 5).indices.tolist())


def test_mean_probability_equals_the_logit_rule_for_a_single_head():
    # softmax preserves order (the paper's footnote to Sec. 3.1): same rho as top-k of the logits
    g = torch.Generator().manual_seed(9)
    q = torch.randn((1, 3, 8), generator=g)
    K = torch.randn((1, 3, 30, 8), generator=g)
    V = torch.randn((1, 3, 30, 8), generator=g)
    _, pos, _ = O.select_variant(q, K, V, [30], 6, O.REDUCE_MEAN_PROB)
    assert torch.equal(pos, O.select(q, K, V, [30], 6)[1])


# ---- prefill over the last P tokens (attention of the cache-correction step, Sec. 3.2)


def test_prefill_against_float64_causal_attention():
    g = torch.Generator().manual_seed(21)
    B, P_new, Hq, Hkv, N, d = 2, 5, 4, 2, 19, 8
    lens = [19, 7]
    q = torch.randn((B, P_new, Hq, d), generator=g)
    K = torch.randn((B, Hkv, N, d), generator=g)
    V = torch.randn((B, Hkv, N, d), generator=g)
    out = O.prefill(q, K, V, lens)
    for b, n in enumerate(lens):
        for j in range(P_new):
            vis = n - P_new + j + 1
            for h in range(Hq):
                kv = h // (Hq // Hkv)
                p = torch.softmax((K[b, kv, :vis].double() @ q[b, j, h].double()) / math.sqrt(d), 0)
                assert torch.allclose(out[b, j, h].double(), p @ V[b, kv, :vis].double(), atol=1e-5), (b, j, h)


def test_prefill_is_causal_and_reduces_to_full_attention_for_one_token():
    g = torch.Generator().manual_seed(22)
    q = torch.randn((1, 3, 2, 8), generator=g)
    K = torch.randn((1, 2, 12, 8), generator=g)
    V = torch.randn((1, 2, 12, 8), generator=g)
    base = O.prefill(q, K, V, [12])
    K2, V2 = K.clone(), V.clone()
    K2[0, :, 11] += 3.0
    V2[0, :, 11] -= 2.0                      # only the last token may notice its own row
    moved = O.prefill(q, K2, V2, [12])
    assert torch.equal(moved[0, :2], base[0, :2]) and not torch.equal(moved[0, 2], base[0, 2])
    assert torch.equal(O.prefill(q[:, 2:], K, V, [12])[0, 0], O.full(q[0, 2][None], K, V, [12])[0])
    # token j is the decode step of a sequence that ends at its position
    for j in range(3):
        assert torch.equal(base[0, j], O.full(q[0, j][None], K, V, [12 - 2 + j])[0])
