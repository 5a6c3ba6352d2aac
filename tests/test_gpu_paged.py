"""GPU parity for the paged (block-table) KV cache: the same entry points, called through the
C ABI with page pools and a block table, against the oracle run on the logical cache that
the oracle itself gathers from the pools.  Pages are scattered over a pool with spare pages;
spare pages and never-written slots hold NaN, so a read through a wrong page shows up."""
import pytest
import torch

from oracle import tidal_oracle as O
from paper_2410_05076_amd import tidal
import workloads as W
from parity_util import check_output, check_positions, same_positions
from test_gpu_parity import DEV, device_layers, host, say

pytestmark = pytest.mark.gpu
D, S, P = W.DENSE, W.SELECT, W.SPARSE


class PagedCase:
    def __init__(self, w, page_size, layout, layers, kernel_variant=0):
        self.w, self.page_size = w, page_size
        self.table, self.num_pages = W.page_table(w, page_size, device=DEV)
        self.q, self.pools, self.views = [], [], []
        for q, K, V in layers:
            Kp, Kv = W.paginate(K, self.table, self.num_pages, page_size, layout)
            Vp, Vv = W.paginate(V, self.table, self.num_pages, page_size, layout)
            self.q.append(q)
            self.pools.append((Kp, Vp))
            self.views.append((Kv, Vv))
        self.lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
        self.shape = tidal.make_paged_shape(self.q[0], self.views[0][0], self.table, self.lens, w.max_seq_len,
                                            total_seq_len=sum(w.seq_lens))
        self.td = tidal.Tidal(self.shape, w.k)
        if kernel_variant:
            self.td.set_tuning(kernel_variant=kernel_variant)

    def logical(self, i):
        """Layer i's cache as the oracle reads it out of the pools."""
        Kv, Vv = self.views[i]
        t = host(self.table)
        return (O.gather_pages(host(Kv), t, self.w.seq_lens, self.w.max_seq_len),
                O.gather_pages(host(Vv), t, self.w.seq_lens, self.w.max_seq_len))


def run_paged_checks(w, page_size, layout, kinds, tag, kernel_variant=0):
    c = PagedCase(w, page_size, layout, device_layers(w, range(len(kinds))), kernel_variant)
    rho = None
    for i, kind in enumerate(kinds):
        q, (Kp, Vp) = c.q[i], c.pools[i]
        qh = host(q)
        Kh, Vh = c.logical(i)
        out = torch.full_like(q, float("nan"))
        if kind == D:
            say("%s: layer %d full attention, page %d %s" % (tag, i, page_size, layout))
            c.td.full_attend(c.shape, q, Kp, Vp, out)
            torch.cuda.synchronize()
            check_output(out, O.full(qh, Kh, Vh, w.seq_lens), "%s L%d full" % (tag, i))
        elif kind == S:
            say("%s: layer %d selection, page %d %s" % (tag, i, page_size, layout))
            pos = torch.full((w.batch, w.num_kv_heads, w.k), -7, dtype=torch.int32, device=DEV)
            scores = torch.full((w.batch, w.num_kv_heads, w.max_seq_len), float("nan"), device=DEV)
            c.td.select_tokens(c.shape, q, Kp, Vp, w.k, out, pos, scores)
            torch.cuda.synchronize()
            o_out, o_pos, o_scores = O.select(qh, Kh, Vh, w.seq_lens, w.k, return_scores=True)
            check_output(out, o_out, "%s L%d select" % (tag, i))
            for b in range(w.batch):
                n = w.seq_lens[b]
                d = (host(scores)[b, :, :n] - o_scores[b, :, :n]).abs().max().item()
                assert d <= 1e-4 * max(1.0, o_scores[b, :, :n].abs().max().item()), "%s scores %g" % (tag, d)
                assert torch.isnan(host(scores)[b, :, n:]).all(), "scores written beyond the sequence"
            check_positions(pos, o_scores, w.seq_lens, w.k, "%s L%d" % (tag, i))
            say("%s: positions identical to oracle: %s" % (tag, same_positions(pos, o_pos)))
            rho = pos
        else:
            say("%s: layer %d sparse attention, page %d %s" % (tag, i, page_size, layout))
            c.td.sparse_attend(c.shape, q, Kp, Vp, rho, w.k, out)
            torch.cuda.synchronize()
            check_output(out, O.sparse(qh, Kh, Vh, w.seq_lens, host(rho)), "%s L%d sparse" % (tag, i))
    c.td.close()


@pytest.mark.parametrize("name,over,page_size,layout", [
    ("c2", dict(context=4099, k=300), 16, "HND"),                       # G = 4, several chunks, ragged tail
    ("c2", dict(context=4099, k=300), 16, "NHD"),                       # token-major pages
    ("c3", dict(context=8229, k=512, tau=512.0), 64, "NHD"),            # G = 1
    ("c4", dict(seq_lens=(777, 64, 1, 2500, 1300), k=256), 16, "HND"),  # ragged batch, k > N for some
    ("c5", dict(context=6000, batch=2, k=1024), 32, "HND"),             # Zipf mass
    ("c2", dict(context=3001, k=257), 1, "HND"),                        # one token per page
    ("c2", dict(context=5000, k=500), 1024, "HND"),                     # pages longer than a chunk granule
    ("c1", dict(context=1500, k=128), 8, "HND"),                        # fp32, head_dim 64
    ("c1", dict(context=333, k=64, head_dim=128, num_q_heads=16), 4, "NHD"),    # fp32 d128, G = 8
    ("c2", dict(context=900, k=100, head_dim=64, num_q_heads=16), 16, "HND"),   # bf16 d64, G = 2
])
def test_paged_layers(name, over, page_size, layout):
    w = W.workload(name, **over)
    run_paged_checks(w, page_size, layout, (D, S, P), "paged %s%s" % (name, sorted(over.items())))


@pytest.mark.parametrize("variant", [2, 3])
def test_paged_layers_both_workgroup_sizes(variant):
    w = W.workload("c2", context=6200, k=300)
    run_paged_checks(w, 16, "HND", (D, S, P), "paged v%d" % variant, kernel_variant=variant)
    w = W.workload("c3", context=9000, k=512, tau=512.0)
    run_paged_checks(w, 16, "NHD", (D, S, P), "paged v%d" % variant, kernel_variant=variant)


@pytest.mark.parametrize("variant", [0, 4, 5])
def test_paged_layers_matrix_core_kernel(variant):
    # groups of eight query heads run on the matrix-core kernel by default (variant 0)
    w = W.workload("c6", context=5100, k=300)
    run_paged_checks(w, 16, "HND", (D, S, P), "paged mfma v%d" % variant, kernel_variant=variant)
    if variant:
        w = W.workload("c2", context=4099, k=300)
        run_paged_checks(w, 32, "NHD", (D, S, P), "paged mfma v%d" % variant, kernel_variant=variant)


def test_paged_decode_step_matches_oracle_and_contiguous_run():
    w = W.workload("c1")
    layers = device_layers(w, range(w.num_layers))
    c = PagedCase(w, 16, "HND", layers)
    outs = [torch.full_like(q, float("nan")) for q in c.q]
    pos = torch.full((1, w.batch, w.num_kv_heads, w.k), -7, dtype=torch.int32, device=DEV)
    c.td.decode_step(c.shape, w.schedule, c.q, [kp for kp, _ in c.pools], [vp for _, vp in c.pools], w.k, outs, pos)
    torch.cuda.synchronize()
    logical = [c.logical(i) for i in range(w.num_layers)]
    o_outs, o_pos = O.step(w.schedule, [host(q) for q in c.q], [k for k, _ in logical], [v for _, v in logical],
                           w.seq_lens, w.k)
    assert same_positions(pos, o_pos)
    for i in range(w.num_layers):
        check_output(outs[i], o_outs[i], "paged c1 L%d" % i)
    # the contiguous cache holding the same tokens gives the same positions
    qs, Ks, Vs = zip(*layers)
    shape = tidal.make_shape(qs[0], Ks[0], c.lens)
    td = tidal.Tidal(shape, w.k)
    outs2 = [torch.full_like(q, float("nan")) for q in qs]
    pos2 = torch.full_like(pos, -7)
    td.decode_step(shape, w.schedule, qs, Ks, Vs, w.k, outs2, pos2)
    torch.cuda.synchronize()
    assert torch.equal(pos, pos2)
    for a, b in zip(outs, outs2):
        check_output(a, b.float().cpu(), "paged vs contiguous")
    td.close()
    c.td.close()


def test_out_of_range_page_ids_do_not_fault():
    # ids outside the pool are clamped into it: the call completes and other sequences are unaffected
    w = W.workload("c4", seq_lens=(600, 300), k=64)
    layers = device_layers(w, range(1))
    c = PagedCase(w, 16, "HND", layers)
    good = torch.full_like(c.q[0], float("nan"))
    c.td.full_attend(c.shape, c.q[0], *c.pools[0], good)
    torch.cuda.synchronize()
    bad_table = c.table.clone()
    bad_table[1, :5] = torch.tensor([-3, 10 ** 6, c.num_pages, -1, 2 ** 30], dtype=torch.int32, device=DEV)
    shape = tidal.make_paged_shape(c.q[0], c.views[0][0], bad_table, c.lens, w.max_seq_len,
                                   total_seq_len=sum(w.seq_lens))   # same launch plan as above
    out = torch.full_like(c.q[0], float("nan"))
    c.td.full_attend(shape, c.q[0], *c.pools[0], out)
    torch.cuda.synchronize()
    assert torch.equal(out[0], good[0])
    c.td.close()
