"""GPU parity for the other grouped-query selection rules (td_shape.selection): the maximum of
the group's logits, and the paper's per-head rule with one rho per query head (Sec. 3.1),
on both attention kernels, contiguous and paged, through the single calls and the step."""
import pytest
import torch

from oracle import tidal_oracle as O
from paper_2410_05076_amd import tidal
import workloads as W
from parity_util import check_output, check_positions, same_positions
from test_gpu_parity import DEV, device_layers, host, say

pytestmark = pytest.mark.gpu
RULES = {"max": (tidal.SELECT_GROUP_MAX, O.REDUCE_MAX), "per_head": (tidal.SELECT_PER_HEAD, O.PER_HEAD),
         "mean_prob": (tidal.SELECT_GROUP_MEAN_PROB, O.REDUCE_MEAN_PROB)}


def run_rule(w, rule, kernel_variant=0, page_size=0):
    sel, o_rule = RULES[rule]
    (q1, K1, V1), (q2, K2, V2) = device_layers(w, range(2))
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    if page_size:
        table, num_pages = W.page_table(w, page_size, device=DEV)
        pools = [W.paginate(x, table, num_pages, page_size) for x in (K1, V1, K2, V2)]
        shape = tidal.make_paged_shape(q1, pools[0][1], table, lens, w.max_seq_len, selection=sel,
                                       total_seq_len=sum(w.seq_lens))
        dK1, dV1, dK2, dV2 = [p for p, _ in pools]
    else:
        shape = tidal.make_shape(q1, K1, lens, selection=sel, total_seq_len=sum(w.seq_lens))
        dK1, dV1, dK2, dV2 = K1, V1, K2, V2
    td = tidal.Tidal(shape, w.k)
    if kernel_variant:
        td.set_tuning(kernel_variant=kernel_variant)
    rows = w.num_q_heads if rule == "per_head" else w.num_kv_heads
    tag = "%s %s v%d page %d" % (w.name, rule, kernel_variant, page_size)
    say("%s: selection layer" % tag)
    out = torch.full_like(q1, float("nan"))
    pos = torch.full((w.batch, rows, w.k), -7, dtype=torch.int32, device=DEV)
    scores = torch.full((w.batch, rows, w.max_seq_len), float("nan"), device=DEV)
    td.select_tokens(shape, q1, dK1, dV1, w.k, out, pos, scores)
    torch.cuda.synchronize()
    o_out, o_pos, o_scores = O.select_variant(host(q1), host(K1), host(V1), w.seq_lens, w.k, o_rule)
    check_output(out, o_out, tag + " select")
    prob = rule == "mean_prob"      # scores are probabilities: compare relative to the row's largest
    for b, n in enumerate(w.seq_lens):
        gs, os_ = host(scores)[b, :, :n], o_scores[b, :, :n]
        if prob:
            d = ((gs - os_).abs().max(dim=-1).values / os_.max(dim=-1).values).max().item()
            assert d <= 1e-4, "%s probabilities off by %g of the row maximum" % (tag, d)
        else:
            d = (gs - os_).abs().max().item()
            assert d <= 1e-4 * max(1.0, os_.abs().max().item()), "%s scores %g" % (tag, d)
        assert torch.isnan(host(scores)[b, :, n:]).all()
    check_positions(pos, o_scores, w.seq_lens, w.k, tag, relative_band=prob)
    say("%s: positions identical to oracle: %s" % (tag, same_positions(pos, o_pos)))
    pos2, out2 = torch.full_like(pos, -7), torch.full_like(q1, float("nan"))
    td.select_tokens(shape, q1, dK1, dV1, w.k, out2, pos2)      # scores in the workspace
    torch.cuda.synchronize()
    assert torch.equal(pos, pos2) and torch.equal(out, out2)
    say("%s: sparse layer" % tag)
    sp = torch.full_like(q2, float("nan"))
    td.sparse_attend(shape, q2, dK2, dV2, pos, w.k, sp)
    torch.cuda.synchronize()
    oracle_sparse = O.sparse_per_head if rule == "per_head" else O.sparse
    check_output(sp, oracle_sparse(host(q2), host(K2), host(V2), w.seq_lens, host(pos)), tag + " sparse")
    td.close()


@pytest.mark.parametrize("rule", ["max", "per_head", "mean_prob"])
@pytest.mark.parametrize("name,over", [
    ("c2", dict(context=4099, k=300)),                                  # G = 4, matrix-core kernel
    ("c6", dict(context=3000, k=200)),                                  # G = 8
    ("c3", dict(context=5000, k=512, tau=512.0)),                       # G = 1: all rules coincide
    ("c4", dict(seq_lens=(777, 64, 1, 2500, 1300), k=256)),             # ragged, k > N for some
    ("c1", dict(context=1500, k=128)),                                  # fp32 d64 G = 4: vector-ALU kernel
    ("c2", dict(context=900, k=100, head_dim=64, num_q_heads=16)),      # bf16 d64, G = 2
])
def test_selection_rules(name, over, rule):
    run_rule(W.workload(name, **over), rule)


@pytest.mark.parametrize("rule", ["max", "per_head", "mean_prob"])
@pytest.mark.parametrize("variant", [2, 3, 4])
def test_selection_rules_on_each_kernel(rule, variant):
    run_rule(W.workload("c2", context=4500, k=300), rule, kernel_variant=variant)


@pytest.mark.parametrize("rule", ["max", "per_head", "mean_prob"])
def test_selection_rules_paged(rule):
    run_rule(W.workload("c2", context=4099, k=300), rule, page_size=16)
    run_rule(W.workload("c1", context=1500, k=128), rule, page_size=8)


def test_per_head_decode_step():
    w = W.workload("c1")
    layers = device_layers(w, range(w.num_layers))
    qs, Ks, Vs = zip(*layers)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(qs[0], Ks[0], lens, selection=tidal.SELECT_PER_HEAD)
    td = tidal.Tidal(shape, w.k)
    outs = [torch.full_like(q, float("nan")) for q in qs]
    pos = torch.full((1, w.batch, w.num_q_heads, w.k), -7, dtype=torch.int32, device=DEV)
    td.decode_step(shape, w.schedule, qs, Ks, Vs, w.k, outs, pos)
    torch.cuda.synchronize()
    # layer by layer with the oracle: full, per-head selection, two sparse layers on that rho
    check_output(outs[0], O.full(host(qs[0]), host(Ks[0]), host(Vs[0]), w.seq_lens), "L0")
    o_out, o_pos, o_scores = O.select_variant(host(qs[1]), host(Ks[1]), host(Vs[1]), w.seq_lens, w.k, O.PER_HEAD)
    check_output(outs[1], o_out, "L1")
    check_positions(pos[0], o_scores, w.seq_lens, w.k, "per-head step")
    for i in (2, 3):
        check_output(outs[i], O.sparse_per_head(host(qs[i]), host(Ks[i]), host(Vs[i]), w.seq_lens, host(pos[0])),
                     "L%d" % i)
    td.close()
