"""Decode-step attention benchmark (one MI355X).

A "step" is one pass of the whole hot path - every layer of the schedule: full attention,
token selection (attention + fused score write + top-k) and position persistent sparse
attention - over one batch of synthetic, HBM-resident inputs, enqueued through
td_decode_step.  Timed iterations rotate over independent copies of the inputs so that
a small working set is not served from the 256 MB Infinity Cache.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

DESCRIPTIONS = {
    "c1": "c1 toy: 4 layers (full, selection, 2 sparse), batch 1, 8 q / 2 KV heads, d 64, context 2048, k 128, fp32",
    "c2": "c2 Llama-3-8B shape: 32 layers (2 full, selection at 2 and 13, 28 sparse), batch 1, 32 q / 8 KV heads, "
          "d 128, context 32768, k 2048, bf16 KV",
    "c3": "c3 Llama-2-7B MHA shape: 32 layers, batch 1, 32 q / 32 KV heads, d 128, context 131072, k 4096, bf16 KV",
    "c4": "c4 batched Llama-3-8B shape: 32 layers, batch 16, ragged contexts 8192..65536, k 2048, bf16 KV",
    "c5": "c5 Llama-3-8B shape: 32 layers, batch 4, context 131072, k sweep, bf16 KV, Zipf(1.1) mass",
    "c6": "c6 64-layer model with the 70B head shape: 64 layers (2 full, selection at 2 and 31, 60 sparse), batch 1, "
          "64 q / 8 KV heads, d 128, context 32768, k 2048, bf16 KV",
}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--workload", default="c2", choices=sorted(DESCRIPTIONS))
    ap.add_argument("--k", type=int, default=0, help="token budget override (c5 sweep)")
    ap.add_argument("--num-q-heads", type=int, default=0, help="override the workload's query head count")
    ap.add_argument("--num-kv-heads", type=int, default=0, help="override the workload's KV head count")
    ap.add_argument("--context", type=int, default=0, help="override the context length of every sequence")
    ap.add_argument("--copies", type=int, default=0, help="independent input copies to rotate over")
    ap.add_argument("--no-graph", action="store_true", help="enqueue eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-reps", type=int, default=24)
    ap.add_argument("--probe-only", action="store_true",
                    help="run only the plain streaming kernels (1 GiB read, 1 GiB copy): counter calibration")
    ap.add_argument("--page-size", type=int, default=0,
                    help="hold the cache in pages of this many tokens behind a shuffled block table (0: contiguous)")
    ap.add_argument("--page-layout", default="HND", choices=["HND", "NHD"],
                    help="inside a page: [KV head][slot][d] or [slot][KV head][d]")
    ap.add_argument("--prefill", type=int, default=0,
                    help="instead of the decode step, time td_prefill_attend over this many new tokens per sequence "
                         "(the attention of the cache-correction step) on one layer of the workload")
    ap.add_argument("--append", action="store_true",
                    help="time td_decode_step_append: every layer also appends the current token's k, v to its cache")
    ap.add_argument("--selection", default="sum", choices=["sum", "max", "per_head", "mean_prob"],
                    help="grouped-query selection rule (td_shape.selection)")
    ap.add_argument("--tune", default="", help="target_workgroups,min_chunk_dense,min_chunk_sparse,max_splits,kernel_variant (0 = default)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported "
              "(no collectives or sharding are part of it)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2410_05076_amd import tidal, workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    tidal.lib()                      # fail loudly if the HIP library is missing
    dev = "cuda:0"
    if args.probe_only:
        print(json.dumps({"hbm_probe": hbm_probe(torch, tidal, dev)}), flush=True)
        return
    if args.prefill:
        print(json.dumps(prefill_bench(args, torch, tidal, W, dev)), flush=True)
        return
    over = {"k": args.k} if args.k else {}
    if args.num_q_heads:
        over["num_q_heads"] = args.num_q_heads
    if args.num_kv_heads:
        over["num_kv_heads"] = args.num_kv_heads
    if args.context:
        over["context"] = args.context
    w = W.workload(args.workload, **over)
    step_bytes = w.algorithmic_bytes_per_step()
    cache_bytes = w.num_layers * 2 * w.batch * w.num_kv_heads * w.max_seq_len * w.head_dim * w.elem_bytes
    copies = args.copies or (3 if cache_bytes <= 8 * 2**30 else 1)
    log("%s: cache %.1f GiB per copy, %d cop%s, %.1f MB algorithmic bytes per step"
        % (w.name, cache_bytes / 2**30, copies, "y" if copies == 1 else "ies", step_bytes / 1e6))

    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=dev)
    n_sel = sum(1 for x in w.schedule if x == W.SELECT)
    selection = {"sum": tidal.SELECT_GROUP_SUM, "max": tidal.SELECT_GROUP_MAX, "per_head": tidal.SELECT_PER_HEAD,
                 "mean_prob": tidal.SELECT_GROUP_MEAN_PROB}[args.selection]
    sel_rows = w.num_q_heads if args.selection == "per_head" else w.num_kv_heads
    sets, all_news = [], []
    for c in range(copies):
        wc = W.workload(args.workload, seed=w.seed + 7919 * c, **over)
        heavy = W.heavy_positions(wc)
        ranks = W.zipf_ranks(wc) if wc.structure == "zipf" else None
        layers = [W.make_layer(wc, i, dev, heavy=heavy, ranks=ranks) for i in range(wc.num_layers)]
        if args.page_size:      # the same tokens, scattered over a page pool; all copies share the table
            if c == 0:
                table, num_pages = W.page_table(w, args.page_size, device=dev)
            paged = []
            for q, K, V in layers:
                Kp, Kv = W.paginate(K, table, num_pages, args.page_size, args.page_layout)
                Vp, _ = W.paginate(V, table, num_pages, args.page_size, args.page_layout)
                paged.append((q, Kp, Vp))
                pool_view = Kv
            layers = paged
        if args.append and not args.page_size:   # the current token's rows, handed over separately
            news = [(torch.stack([K[b, :, n - 1] for b, n in enumerate(w.seq_lens)]).contiguous(),
                     torch.stack([V[b, :, n - 1] for b, n in enumerate(w.seq_lens)]).contiguous()) for _, K, V in layers]
        elif args.append:
            news = [(torch.randn((w.batch, w.num_kv_heads, w.head_dim), device=dev).to(w.torch_dtype),
                     torch.randn((w.batch, w.num_kv_heads, w.head_dim), device=dev).to(w.torch_dtype)) for _ in layers]
        else:
            news = None
        qs, Ks, Vs = zip(*layers)
        outs = [torch.zeros_like(q) for q in qs]
        pos = torch.full((n_sel, w.batch, sel_rows, w.k), -1, dtype=torch.int32, device=dev)
        sets.append((qs, Ks, Vs, outs, pos))
        all_news.append(news)
        log("generated copy %d" % c)
    if args.page_size:
        shape = tidal.make_paged_shape(sets[0][0][0], pool_view, table, lens, w.max_seq_len,
                                       total_seq_len=sum(w.seq_lens), selection=selection)
    else:
        shape = tidal.make_shape(sets[0][0][0], sets[0][1][0], lens, total_seq_len=sum(w.seq_lens),
                                 selection=selection)
    td = tidal.Tidal(shape, w.k)
    if args.tune:
        td.set_tuning(*[int(x) for x in args.tune.split(",")])

    def enqueue(c):
        qs, Ks, Vs, outs, pos = sets[c]
        if args.append:
            td.decode_step_append(shape, w.schedule, qs, [a for a, _ in all_news[c]], [b for _, b in all_news[c]],
                                  Ks, Vs, w.k, outs, pos)
        else:
            td.decode_step(shape, w.schedule, qs, Ks, Vs, w.k, outs, pos)

    for c in range(copies):
        enqueue(c)
    torch.cuda.synchronize()

    use_graph = not args.no_graph
    graphs = []
    if use_graph:
        for c in range(copies):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                enqueue(c)
            graphs.append(g)
        torch.cuda.synchronize()

    def step(i):
        c = i % copies
        if use_graph:
            graphs[c].replay()
        else:
            enqueue(c)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) / args.steps * 1e3
    us_per_step = ms_per_step * 1e3
    log("%.1f us per decode step (%s)" % (us_per_step, "graph replay" if use_graph else "eager"))

    # Per-launch duration of each layer kind: `reps` launches of that kind (rotating over input
    # copies and layers, so each launch streams data that is not in cache) are captured into one
    # HIP graph; HIP events on the launch stream bracket each replay.  Back-to-back kernels in a
    # graph leave gaps well under a microsecond, so time / reps is the kernel's own duration.
    def time_kind(kind, reps):
        idx = [i for i, x in enumerate(w.schedule) if x == kind]
        if not idx:
            return None

        def launches():
            for r in range(reps):
                qs, Ks, Vs, outs, pos = sets[r % copies]
                i = idx[(r // copies) % len(idx)]
                if kind == W.DENSE:
                    td.full_attend(shape, qs[i], Ks[i], Vs[i], outs[i])
                elif kind == W.SELECT:
                    td.select_tokens(shape, qs[i], Ks[i], Vs[i], w.k, outs[i], pos[0])
                else:
                    td.sparse_attend(shape, qs[i], Ks[i], Vs[i], pos[0], w.k, outs[i])

        if use_graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                launches()
            run = g.replay
        else:
            run = launches
        run()
        torch.cuda.synchronize()
        evs = []
        for _ in range(5):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            run()
            b.record()
            evs.append((a, b))
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) * 1e3 / reps for a, b in evs)
        return sum(ts) / len(ts), ts[len(ts) // 2]

    per_kind = {}
    for name, kind in (("full", W.DENSE), ("select", W.SELECT), ("sparse", W.SPARSE)):
        r = time_kind(kind, args.kernel_reps)
        if r:
            per_kind[name] = {"avg_us": round(r[0], 2), "median_us": round(r[1], 2)}
    dense_bytes = w.kv_bytes_per_layer()
    dense_us = per_kind["full"]["avg_us"]
    achieved = dense_bytes / (dense_us * 1e-6) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "attend_dense_%s_traffic.json" % w.name)
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")
    roofline = {"kernel": "full-attention layer launch (attend_mfma_kernel for bf16 head_dim 128, else attend_split_kernel): K and V of one layer streamed once",
                "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "algorithmic_bytes_per_launch": dense_bytes, "avg_launch_us": dense_us}
    for name, nbytes in (("select", dense_bytes), ("sparse", w.sparse_bytes_per_layer())):
        if name in per_kind:
            per_kind[name]["GBps"] = round(nbytes / (per_kind[name]["avg_us"] * 1e-6) / 1e9, 1)
    per_kind["full"]["GBps"] = round(achieved, 1)

    probe = hbm_probe(torch, tidal, dev, td)
    log("plain streaming kernels: read %.0f GB/s, copy %.0f GB/s (read + write bytes)"
        % (probe["read_GBps"], probe["copy_GBps"]))
    cpu = None
    if not args.no_cpu_baseline and not args.page_size and args.selection == "sum":
        cpu = cpu_baseline(w, sets[0], torch)

    out = {
        "metric": "decode_step_attention_us", "value": round(us_per_step, 2), "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": DESCRIPTIONS[w.name] + ("".join(", %s overridden to %s" % (a, b) for a, b in sorted(over.items()) if a != "k")) + (", cache in pages of %d tokens (%s) behind a shuffled block table"
                                                       % (args.page_size, args.page_layout) if args.page_size else ""),
                   "k": w.k, "selection": args.selection, "input_copies_rotated": copies,
                   "launch": ("hip graph replay of " if use_graph else "eager ") +
                             ("td_decode_step_append" if args.append else "td_decode_step")},
        "step_hbm": {"algorithmic_bytes": step_bytes,
                     "achieved_GBps": round(step_bytes / (us_per_step * 1e-6) / 1e9, 1),
                     "frac_of_peak": round(step_bytes / (us_per_step * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)},
        "per_layer_kind": per_kind,
        "hbm_probe": probe,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    td.close()
    print(json.dumps(out), flush=True)


def prefill_bench(args, torch, tidal, W, dev):
    """Time of td_prefill_attend for P new tokens per sequence on one layer's cache, against the higher of its two
    floors: the stream of the cache from HBM (few new tokens) or the dense MFMA peak (many).

    flop = 4 * d * sum over tokens and heads of the positions each token sees (two products, multiply-add);
    bytes = the keys and values of all positions, once."""
    over = {}
    if args.num_q_heads:
        over["num_q_heads"] = args.num_q_heads
    if args.num_kv_heads:
        over["num_kv_heads"] = args.num_kv_heads
    if args.context:
        over["context"] = args.context
    w = W.workload(args.workload, **over)
    P = args.prefill
    q1, K, V = W.make_layer(w, 0, dev, heavy=W.heavy_positions(w), ranks=W.zipf_ranks(w) if w.structure == "zipf" else None)
    q = torch.randn((w.batch, P, w.num_q_heads, w.head_dim), device=dev).to(w.torch_dtype)
    out = torch.empty_like(q)
    lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=dev)
    if args.page_size:      # the same tokens, scattered over a page pool
        table, num_pages = W.page_table(w, args.page_size, device=dev)
        _, K = W.paginate(K, table, num_pages, args.page_size, args.page_layout)
        _, V = W.paginate(V, table, num_pages, args.page_size, args.page_layout)
        shape = tidal.make_paged_shape(q1, K, table, lens, w.max_seq_len)
    else:
        shape = tidal.make_shape(q1, K, lens)
    td = tidal.Tidal(shape, 0, prefill_new=P)
    for _ in range(max(1, args.warmup)):
        td.prefill_attend(shape, q, K, V, out)
    torch.cuda.synchronize()
    evs = []
    for _ in range(args.steps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        td.prefill_attend(shape, q, K, V, out)
        b.record()
        evs.append((a, b))
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
    us = sum(ts) / len(ts)
    seen = sum(sum(max(n - P + j + 1, 0) for j in range(P)) for n in w.seq_lens)
    flop = 4.0 * w.head_dim * w.num_q_heads * seen
    # the keys and values of every position some new token sees, once
    esize = 2 if w.dtype == "bf16" else 4
    kv_bytes = 2.0 * w.num_kv_heads * w.head_dim * esize * sum(w.seq_lens)
    td.close()
    # whichever of the two floors is higher for this P names the bound
    if kv_bytes / 8.0e12 > flop / 2.5e15:
        rate = kv_bytes / (us * 1e-6) / 1e9
        roof = {"kernel": "prefill_mfma_kernel + prefill_merge_kernel", "bound": "hbm", "achieved": round(rate, 1),
                "peak": 8000.0, "unit": "GB/s", "frac": round(rate / 8000.0, 4), "traffic": None,
                "bytes_per_launch": kv_bytes, "flop_per_launch": flop}
    else:
        tflops = flop / (us * 1e-6) / 1e12
        roof = {"kernel": "prefill_mfma_kernel", "bound": "mfma", "achieved": round(tflops, 1), "peak": 2500.0,
                "unit": "TFLOP/s", "frac": round(tflops / 2500.0, 4), "traffic": None, "flop_per_launch": flop,
                "bytes_per_launch": kv_bytes}
    return {"metric": "prefill_attention_us", "value": round(us, 2), "unit": "us", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(us / 1e3, 5), "higher_is_better": False, "scaling": "weak",
            "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
            "config": {"workload": DESCRIPTIONS[w.name] + ", one layer, prefill attention over the last %d tokens" % P
                       + (", paged cache, page size %d (%s)" % (args.page_size, args.page_layout) if args.page_size else "")},
            "median_us": round(ts[len(ts) // 2], 2), "roofline": roof}


def hbm_probe(torch, tidal, dev, td=None, nbytes=2**30, reps=6):
    """Measured rate of a plain streaming read and a plain copy of 1 GiB (cold: larger than every cache)."""
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(3)
    dst = torch.empty_like(src)
    own = td is None
    if own:
        lens = torch.ones(1, dtype=torch.int32, device=dev)
        q = torch.zeros((1, 1, 64), dtype=torch.float32, device=dev)
        K = torch.zeros((1, 1, 8, 64), dtype=torch.float32, device=dev)
        td = tidal.Tidal(tidal.make_shape(q, K, lens), 1)
    out = {"bytes": nbytes}
    for name, d, moved in (("read_GBps", None, nbytes), ("copy_GBps", dst, 2 * nbytes)):
        evs = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            td.probe_stream(src, d)
            b.record()
            evs.append((a, b))
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in evs[1:])
        out[name] = round(moved / (ts[len(ts) // 2] * 1e-3) / 1e9, 1)
    if own:
        td.close()
    return out


def cpu_baseline(w, inputs, torch):
    """The CPU oracle on the host cores, one layer at a time (one layer's K, V on the host at once).

    Small caches: every layer of one decode step.  Large caches: one layer of each kind,
    scaled by the number of layers of that kind (stated in `sample`)."""
    from oracle import tidal_oracle as O
    from paper_2410_05076_amd import workloads as W
    qs, Ks, Vs, _, _ = inputs
    layer_bytes = 2 * Ks[0].numel() * Ks[0].element_size()
    whole = layer_bytes * w.num_layers <= 6 * 2**30
    kinds = list(w.schedule)
    if whole:
        todo = list(range(w.num_layers))
    else:
        todo = [kinds.index(W.DENSE), kinds.index(W.SELECT), kinds.index(W.SPARSE)]
    t_kind = {W.DENSE: [], W.SELECT: [], W.SPARSE: []}
    rho = None
    for i in sorted(todo):
        q, K, V = qs[i].cpu(), Ks[i].cpu(), Vs[i].cpu()
        t0 = time.perf_counter()
        if kinds[i] == W.DENSE:
            O.full(q, K, V, w.seq_lens)
        elif kinds[i] == W.SELECT:
            _, rho = O.select(q, K, V, w.seq_lens, w.k)
        else:
            O.sparse(q, K, V, w.seq_lens, rho)
        t_kind[kinds[i]].append(time.perf_counter() - t0)
        log("oracle layer %d: %.3f s" % (i, t_kind[kinds[i]][-1]))
    total = 0.0
    for kind, ts in t_kind.items():
        if ts:
            total += sum(ts) if whole else sum(ts) / len(ts) * kinds.count(kind)
    sample = ("all %d layers of one %s decode step, one layer at a time" % (w.num_layers, w.name) if whole else
              "one full, one selection and one sparse layer of %s, each scaled by its layer count" % w.name)
    return {"value": round(total * 1e6, 1), "unit": "us", "cores": O.num_threads(), "kind": "oracle",
            "sample": sample}


if __name__ == "__main__":
    main()
