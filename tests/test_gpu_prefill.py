"""GPU parity for td_prefill_attend (the attention of the cache-correction step, Sec. 3.2): causal
full attention of the last P tokens of every sequence, against the oracle's tdo_prefill."""
import pytest
import torch

from oracle import tidal_oracle as O
from paper_2410_05076_amd import tidal
import workloads as W
from parity_util import check_output
from test_gpu_parity import DEV, device_layers, host, say

pytestmark = pytest.mark.gpu


def run_prefill(w, num_new, seed=3, chunked=True):
    (_, K, V), = device_layers(w, [0])
    g = torch.Generator(device=DEV).manual_seed(seed)
    q = torch.randn((w.batch, num_new, w.num_q_heads, w.head_dim), generator=g, device=DEV).to(torch.bfloat16)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(q[:, 0].contiguous(), K, lens)
    # chunked: a workspace for every token chunk the plan wants; else none, so one chunk
    td = tidal.Tidal(shape, 0, prefill_new=num_new) if chunked else tidal.Tidal(shape, 0, workspace_bytes=0)
    out = torch.full_like(q, float("nan"))
    say("prefill %s P=%d chunked=%s" % (w.name, num_new, chunked))
    td.prefill_attend(shape, q, K, V, out)
    torch.cuda.synchronize()
    check_output(out, O.prefill(host(q), host(K), host(V), w.seq_lens), "prefill %s P=%d" % (w.name, num_new))
    td.close()


@pytest.mark.parametrize("name,over,num_new", [
    ("c2", dict(context=3000, k=64), 1),                                   # one token: the decode step
    ("c2", dict(context=3000, k=64), 16),                                  # G = 4: exactly one row block
    ("c2", dict(context=3000, k=64), 37),                                  # ragged last row block
    ("c2", dict(context=777, k=64), 300),                                  # many row blocks, short prefix
    ("c3", dict(context=2500, k=64, tau=512.0), 100),                      # G = 1: 64 tokens per block
    ("c6", dict(context=2000, k=64), 21),                                  # G = 8
    ("c2", dict(context=1000, k=64, num_q_heads=16), 50),                  # G = 2
    ("c4", dict(seq_lens=(900, 33, 64, 2048), k=64), 33),                  # ragged batch, P = N for one
    ("c2", dict(context=40, k=8), 40),                                     # the whole sequence is new
])
@pytest.mark.parametrize("chunked", [True, False])
def test_prefill_attend(name, over, num_new, chunked):
    run_prefill(W.workload(name, **over), num_new, chunked=chunked)


def test_prefill_over_many_token_chunks():
    run_prefill(W.workload("c2", context=20000, k=64), 16)            # 39 chunks of 576 tokens


def test_prefill_with_a_workspace_for_some_of_the_chunks():
    w = W.workload("c2", context=6000, k=64)
    (_, K, V), = device_layers(w, [0])
    g = torch.Generator(device=DEV).manual_seed(5)
    q = torch.randn((1, 16, w.num_q_heads, w.head_dim), generator=g, device=DEV).to(torch.bfloat16)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(q[:, 0].contiguous(), K, lens)
    full = tidal.lib().td_prefill_workspace_bytes(shape, 16)
    assert full > 0
    ref = O.prefill(host(q), host(K), host(V), w.seq_lens)
    for ws in (full, full // 2, full // 4):
        td = tidal.Tidal(shape, 0, workspace_bytes=ws)
        out = torch.full_like(q, float("nan"))
        say("prefill with %d workspace bytes" % ws)
        td.prefill_attend(shape, q, K, V, out)
        torch.cuda.synchronize()
        check_output(out, ref, "workspace %d" % ws)
        td.close()


def test_prefill_longer_than_a_sequence_yields_zeros_for_the_missing_tokens():
    w = W.workload("c4", seq_lens=(50, 10), k=8)
    (_, K, V), = device_layers(w, [0])
    g = torch.Generator(device=DEV).manual_seed(1)
    q = torch.randn((2, 16, w.num_q_heads, w.head_dim), generator=g, device=DEV).to(torch.bfloat16)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(q[:, 0].contiguous(), K, lens)
    td = tidal.Tidal(shape, 0)
    out = torch.full_like(q, float("nan"))
    td.prefill_attend(shape, q, K, V, out)
    torch.cuda.synchronize()
    assert (out[1, :6] == 0).all()                     # tokens at positions -6 .. -1 do not exist
    ref = O.prefill(host(q[1:, 6:]).contiguous(), host(K[1:]), host(V[1:]), [10])
    check_output(out[1:, 6:], ref, "tail of the short sequence")
    check_output(out[:1], O.prefill(host(q[:1]), host(K[:1]), host(V[:1]), [50]), "long sequence")
    td.close()


def test_chunked_prefill_of_a_ragged_batch_with_a_sequence_shorter_than_the_new_tokens():
    w = W.workload("c4", seq_lens=(3000, 10, 1700), k=8)    # 5 chunks of 640 tokens; sequence 1 uses none of them
    (_, K, V), = device_layers(w, [0])
    g = torch.Generator(device=DEV).manual_seed(2)
    q = torch.randn((3, 16, w.num_q_heads, w.head_dim), generator=g, device=DEV).to(torch.bfloat16)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(q[:, 0].contiguous(), K, lens)
    assert tidal.lib().td_prefill_workspace_bytes(shape, 16) > 0
    td = tidal.Tidal(shape, 0, prefill_new=16)
    out = torch.full_like(q, float("nan"))
    say("chunked prefill, ragged")
    td.prefill_attend(shape, q, K, V, out)
    torch.cuda.synchronize()
    assert (out[1, :6] == 0).all()                     # tokens at positions -6 .. -1 do not exist
    ref = O.prefill(host(q[1:2, 6:]).contiguous(), host(K[1:2]), host(V[1:2]), [10])
    check_output(out[1:2, 6:], ref, "tail of the short sequence")
    for b in (0, 2):
        check_output(out[b:b + 1], O.prefill(host(q[b:b + 1]), host(K[b:b + 1]), host(V[b:b + 1]), [w.seq_lens[b]]),
                     "sequence %d" % b)
    td.close()


def run_plain_prefill(w, num_new, page_size=0, workspace="whole", seed=9):
    """Shapes outside the matrix-core kernel (fp32, head_dim 64, pages under 16 tokens) take the library's plain
    path; workspace: "whole" = td_prefill_workspace_bytes (one launch for all new tokens), "some" = room for about
    a quarter of them (runs of new tokens, one sequence at a time), or a byte count.  Sequences shorter than num_new are compared
    token by token: zeros before the start of the cache, the oracle on the rest."""
    (_, K, V), = device_layers(w, [0])
    g = torch.Generator(device=DEV).manual_seed(seed)
    q = torch.randn((w.batch, num_new, w.num_q_heads, w.head_dim), generator=g, device=DEV).to(w.torch_dtype)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    Kd, Vd = K, V
    if page_size:
        table, num_pages = W.page_table(w, page_size, device=DEV)
        _, Kd = W.paginate(K, table, num_pages, page_size)
        _, Vd = W.paginate(V, table, num_pages, page_size)
        shape = tidal.make_paged_shape(q[:, 0].contiguous(), Kd, table, lens, w.max_seq_len)
    else:
        shape = tidal.make_shape(q[:, 0].contiguous(), K, lens)
    if workspace == "whole":
        assert tidal.lib().td_prefill_workspace_bytes(shape, num_new) > 0
        td = tidal.Tidal(shape, 0, prefill_new=num_new)
    elif workspace == "some":
        whole = tidal.lib().td_prefill_workspace_bytes(shape, num_new)
        base = tidal.lib().td_prefill_workspace_bytes(shape, 1)
        td = tidal.Tidal(shape, 0, workspace_bytes=base + (whole - base) // 4)
    else:
        td = tidal.Tidal(shape, 0, workspace_bytes=workspace)
    out = torch.full_like(q, float("nan"))
    say("plain prefill %s %s d%d P=%d page %d workspace %s" % (w.name, w.dtype, w.head_dim, num_new, page_size, workspace))
    td.prefill_attend(shape, q, Kd, Vd, out)
    torch.cuda.synchronize()
    for b, n in enumerate(w.seq_lens):
        missing = max(0, num_new - n)
        assert (out[b, :missing] == 0).all(), "tokens before the start of sequence %d" % b
        ref = O.prefill(host(q[b:b + 1, missing:]).contiguous(), host(K[b:b + 1]), host(V[b:b + 1]), [n])
        check_output(out[b:b + 1, missing:], ref, "plain prefill, sequence %d" % b)
    # the ticket counters are back at zero: the context serves a decode call as before (where its workspace
    # has room for one), and the same prefill again gives the same bits
    if workspace == "whole":
        out1 = torch.full_like(q[:, 0], float("nan"))
        td.full_attend(shape, q[:, 0].contiguous(), Kd, Vd, out1)
        torch.cuda.synchronize()
        check_output(out1, O.full(host(q[:, 0]).contiguous(), host(K), host(V), w.seq_lens), "decode call afterwards")
    again = torch.full_like(q, float("nan"))
    td.prefill_attend(shape, q, Kd, Vd, again)
    torch.cuda.synchronize()
    assert torch.equal(again, out)
    td.close()


@pytest.mark.parametrize("name,over,num_new,page_size", [
    ("c1", dict(context=300, k=8), 1, 0),                                          # fp32, head_dim 64: one token
    ("c1", dict(context=300, k=8), 40, 0),
    ("c1", dict(seq_lens=(300, 5, 120), k=8), 16, 0),                              # a sequence shorter than the new tokens
    ("c1", dict(context=700, k=8, dtype="bf16"), 33, 0),                           # bf16, head_dim 64
    ("c2", dict(context=600, k=8, dtype="f32"), 21, 0),                            # fp32, head_dim 128
    ("c3", dict(context=500, k=8, head_dim=64), 9, 0),                             # G = 1
    ("c2", dict(context=500, k=16), 33, 8),                                        # bf16, head_dim 128, pages of 8 tokens
    ("c2", dict(seq_lens=(500, 90), k=16), 12, 4),                                 # pages of 4, two sequences
    ("c1", dict(seq_lens=(3000, 2100), k=8), 24, 1),                               # pages of 1: every token its own page
    ("c1", dict(context=9000, k=8), 3, 0),                                         # few rows: the tokens are cut into chunks
])
@pytest.mark.parametrize("workspace", ["whole", "some"])
def test_plain_prefill_for_shapes_outside_the_matrix_core_kernel(name, over, num_new, page_size, workspace):
    run_plain_prefill(W.workload(name, **over), num_new, page_size=page_size, workspace=workspace)


def test_plain_prefill_with_a_workspace_too_small_for_one_token():
    w = W.workload("c1", context=100, k=8)
    (q1, K, V), = device_layers(w, [0])
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(q1, K, lens)
    td = tidal.Tidal(shape, 0, workspace_bytes=4096)
    q = q1[:, None].contiguous()
    with pytest.raises(tidal.TidalError) as e:
        td.prefill_attend(shape, q, K, V, torch.empty_like(q))
    assert e.value.status == tidal.ERR_WORKSPACE
    td.close()


@pytest.mark.parametrize("num_new", [16, 1024])
def test_prefill_at_the_benchmark_shape_on_sampled_tokens(num_new):
    """c2 at full size, in the launch configuration `bench.py --prefill` times (16 new tokens: token chunks and
    the merge kernel; 1024: one chunk, 64-row blocks).  The oracle takes the new tokens one by one: token j is a
    decode query over the first N - P + j + 1 positions, so a sample of tokens (ends, neighbours across a row
    block boundary, some in between) is compared with tdo_full on those prefixes."""
    w = W.workload("c2")
    (_, K, V), = device_layers(w, [0])
    g = torch.Generator(device=DEV).manual_seed(11)
    q = torch.randn((w.batch, num_new, w.num_q_heads, w.head_dim), generator=g, device=DEV).to(torch.bfloat16)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(q[:, 0].contiguous(), K, lens)
    td = tidal.Tidal(shape, 0, prefill_new=num_new)
    out = torch.full_like(q, float("nan"))
    say("prefill c2 full size P=%d" % num_new)
    td.prefill_attend(shape, q, K, V, out)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    Kh, Vh = host(K), host(V)
    n = w.seq_lens[0]
    G = w.num_q_heads // w.num_kv_heads
    per_block = 64 // G                                 # tokens per 64-row block
    sample = sorted({0, 1, num_new // 2, num_new - 2, num_new - 1, min(per_block - 1, num_new - 1),
                     min(per_block, num_new - 1), min(5 * per_block + 3, num_new - 1)})
    for j in sample:
        ref = O.full(host(q[:, j]).contiguous(), Kh, Vh, [n - num_new + j + 1])
        check_output(out[:, j], ref, "c2 P=%d token %d" % (num_new, j))
    td.close()


@pytest.mark.parametrize("num_new", [24, 200])
def test_prefill_with_a_token_major_cache_layout(num_new):
    # K, V stored [B][N][Hkv][d] and passed through the strides; 200 new tokens use the 64-row blocks
    w = W.workload("c2", context=2100, k=64)
    (_, K, V), = device_layers(w, [0])
    Kt = K.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    Vt = V.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    g = torch.Generator(device=DEV).manual_seed(8)
    q = torch.randn((w.batch, num_new, w.num_q_heads, w.head_dim), generator=g, device=DEV).to(torch.bfloat16)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(q[:, 0].contiguous(), Kt, lens)
    assert shape.kv_stride_tok == w.num_kv_heads * w.head_dim
    td = tidal.Tidal(shape, 0, prefill_new=num_new)
    out = torch.full_like(q, float("nan"))
    say("prefill token-major P=%d" % num_new)
    td.prefill_attend(shape, q, Kt, Vt, out)
    torch.cuda.synchronize()
    check_output(out, O.prefill(host(q), host(K), host(V), w.seq_lens), "token-major prefill")
    td.close()


def test_prefill_results_are_deterministic():
    w = W.workload("c2", context=3000, k=64)
    (_, K, V), = device_layers(w, [0])
    g = torch.Generator(device=DEV).manual_seed(9)
    q = torch.randn((w.batch, 40, w.num_q_heads, w.head_dim), generator=g, device=DEV).to(torch.bfloat16)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(q[:, 0].contiguous(), K, lens)
    td = tidal.Tidal(shape, 0, prefill_new=40)
    outs = []
    for _ in range(3):
        out = torch.full_like(q, float("nan"))
        td.prefill_attend(shape, q, K, V, out)
        torch.cuda.synchronize()
        outs.append(out)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    td.close()


def test_chunked_prefill_as_a_hip_graph():
    # two kernels (chunks, merge) and no memset: replays, with eager work in between, reproduce the eager result
    w = W.workload("c2", context=5000, k=64)
    (_, K, V), = device_layers(w, [0])
    g = torch.Generator(device=DEV).manual_seed(13)
    q = torch.randn((w.batch, 16, w.num_q_heads, w.head_dim), generator=g, device=DEV).to(torch.bfloat16)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(q[:, 0].contiguous(), K, lens)
    td = tidal.Tidal(shape, 0, prefill_new=16)
    out = torch.full_like(q, float("nan"))
    td.prefill_attend(shape, q, K, V, out)
    torch.cuda.synchronize()
    eager = out.clone()
    check_output(eager, O.prefill(host(q), host(K), host(V), w.seq_lens), "eager")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        td.prefill_attend(shape, q, K, V, out)
    for rep in range(3):
        out.fill_(float("nan"))
        scratch = torch.randn(1 << 20, device=DEV).sum()     # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "replay %d" % rep
    td.close()


@pytest.mark.parametrize("name,over,num_new,page_size,layout", [
    ("c2", dict(context=3000, k=64), 16, 16, "HND"),                      # two pages per tile, token chunks
    ("c2", dict(context=3000, k=64), 37, 64, "NHD"),                      # token-major pool, ragged last row block
    ("c2", dict(context=2100, k=64), 200, 32, "HND"),                     # 64-row blocks, one page per tile
    ("c6", dict(context=2000, k=64), 21, 128, "NHD"),                     # G = 8, pages longer than a tile
    ("c3", dict(context=2500, k=64, tau=512.0), 100, 16, "HND"),          # G = 1
    ("c4", dict(seq_lens=(900, 33, 64, 2048), k=64), 33, 16, "HND"),      # ragged batch, P = N for one
])
def test_prefill_over_a_paged_cache(name, over, num_new, page_size, layout):
    """Pages scattered over a pool with spare pages; spare pages and never-written slots hold NaN."""
    w = W.workload(name, **over)
    (_, K, V), = device_layers(w, [0])
    table, num_pages = W.page_table(w, page_size, device=DEV)
    Kp, Kv = W.paginate(K, table, num_pages, page_size, layout)
    Vp, Vv = W.paginate(V, table, num_pages, page_size, layout)
    g = torch.Generator(device=DEV).manual_seed(17)
    q = torch.randn((w.batch, num_new, w.num_q_heads, w.head_dim), generator=g, device=DEV).to(torch.bfloat16)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    shape = tidal.make_paged_shape(q[:, 0].contiguous(), Kv, table, lens, w.max_seq_len)
    td = tidal.Tidal(shape, 0, prefill_new=num_new)
    out = torch.full_like(q, float("nan"))
    say("paged prefill %s P=%d page %d %s" % (w.name, num_new, page_size, layout))
    td.prefill_attend(shape, q, Kv, Vv, out)
    torch.cuda.synchronize()
    t = host(table)
    Kl = O.gather_pages(host(Kv), t, w.seq_lens, w.max_seq_len)
    Vl = O.gather_pages(host(Vv), t, w.seq_lens, w.max_seq_len)
    check_output(out, O.prefill(host(q), Kl, Vl, w.seq_lens), "paged prefill")
    td.close()


def _random_prefill_case(seed):
    """A small random prefill: shape, lengths around tile and chunk boundaries, cache kind and workspace by seed."""
    r = torch.Generator().manual_seed(1000 + seed)
    pick = lambda xs: xs[int(torch.randint(len(xs), (1,), generator=r))]
    G, Hkv, B = pick([1, 2, 4, 8]), pick([1, 2]), pick([1, 2, 3])
    n_max = pick([40, 130, 257, 600, 1100])
    lens = [int(torch.randint(1, n_max + 1, (1,), generator=r)) for _ in range(B)]
    lens[int(torch.randint(B, (1,), generator=r))] = n_max
    P = min(pick([1, 3, 17, 40, 90]), n_max)
    page = pick([0, 0, 16, 32])
    chunked = pick([True, False])
    return G, Hkv, B, lens, n_max, P, page, chunked


@pytest.mark.parametrize("seed", range(40))
def test_random_small_prefills(seed):
    G, Hkv, B, lens, n_max, P, page, chunked = _random_prefill_case(seed)
    g = torch.Generator(device=DEV).manual_seed(seed)
    d = 128
    q = torch.randn((B, P, G * Hkv, d), generator=g, device=DEV).to(torch.bfloat16)
    K = torch.randn((B, Hkv, n_max, d), generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn((B, Hkv, n_max, d), generator=g, device=DEV).to(torch.bfloat16)
    lens_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    Kc, Vc = K, V
    if page:
        w = W.workload("c4", seq_lens=tuple(lens), k=8, num_q_heads=G * Hkv, num_kv_heads=Hkv)
        table, num_pages = W.page_table(w, page, device=DEV)
        _, Kc = W.paginate(K, table, num_pages, page)
        _, Vc = W.paginate(V, table, num_pages, page)
        shape = tidal.make_paged_shape(q[:, 0].contiguous(), Kc, table, lens_d, n_max)
    else:
        shape = tidal.make_shape(q[:, 0].contiguous(), K, lens_d)
    td = tidal.Tidal(shape, 0, prefill_new=P) if chunked else tidal.Tidal(shape, 0, workspace_bytes=0)
    out = torch.full_like(q, float("nan"))
    say("random prefill %d: G%d Hkv%d lens %s P%d page %d chunked %s" % (seed, G, Hkv, lens, P, page, chunked))
    td.prefill_attend(shape, q, Kc, Vc, out)
    torch.cuda.synchronize()
    for b, n in enumerate(lens):        # new tokens that would sit before the start of the cache yield zeros
        m = min(P, n)
        assert (out[b, :P - m] == 0).all()
        ref = O.prefill(host(q[b:b + 1, P - m:]).contiguous(), host(K[b:b + 1]), host(V[b:b + 1]), [n])
        check_output(out[b:b + 1, P - m:], ref, "random prefill %d, sequence %d" % (seed, b))
    td.close()


def test_prefill_whose_row_maxima_keep_rising():
    """Keys grow along the sequence, so every later tile raises the rows' reference maxima by far more than the
    lazy margin: the rescale path and the reload after it run throughout, also across token chunks."""
    n, P, Hq, Hkv, d = 3000, 20, 8, 2, 128
    g = torch.Generator(device=DEV).manual_seed(4)
    q = torch.randn((1, P, Hq, d), generator=g, device=DEV).abs().to(torch.bfloat16)
    ramp = torch.linspace(0.05, 3.0, n, device=DEV)[None, None, :, None]
    K = (torch.randn((1, Hkv, n, d), generator=g, device=DEV).abs() * ramp).to(torch.bfloat16)
    V = torch.randn((1, Hkv, n, d), generator=g, device=DEV).to(torch.bfloat16)
    lens = torch.tensor([n], dtype=torch.int32, device=DEV)
    shape = tidal.make_shape(q[:, 0].contiguous(), K, lens)
    for chunked in (True, False):
        td = tidal.Tidal(shape, 0, prefill_new=P) if chunked else tidal.Tidal(shape, 0, workspace_bytes=0)
        out = torch.full_like(q, float("nan"))
        say("rising maxima, chunked %s" % chunked)
        td.prefill_attend(shape, q, K, V, out)
        torch.cuda.synchronize()
        check_output(out, O.prefill(host(q), host(K), host(V), [n]), "rising maxima")
        td.close()
