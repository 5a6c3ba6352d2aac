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


HEADLINE = "c3"
# the other configurations, reported in `configs` next to the headline (c5 is the budget sweep)
OTHERS = (("c2", (0,)), ("c4", (0,)), ("c5", (256, 1024, 4096, 16384)))
KIND_NAMES = ("full", "select", "sparse")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="", choices=[""] + sorted(DESCRIPTIONS),
                    help="time this workload only (default: the headline %s as `value`, and c2, c4 and the c5 "
                         "budget sweep in `configs`)" % HEADLINE)
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
    from paper_2410_05076_amd import tidal
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    tidal.lib()                      # fail loudly if the HIP library is missing
    dev = "cuda:0"
    if args.probe_only:
        print(json.dumps({"hbm_probe": hbm_probe(torch, tidal, dev)}), flush=True)
        return
    if args.prefill:
        args.workload = args.workload or "c2"
        print(json.dumps(prefill_bench(args, torch, tidal, W, dev)), flush=True)
        return
    over = {}
    if args.num_q_heads:
        over["num_q_heads"] = args.num_q_heads
    if args.num_kv_heads:
        over["num_kv_heads"] = args.num_kv_heads
    if args.context:
        over["context"] = args.context
    probe = hbm_probe(torch, tidal, dev)
    log("plain streaming kernels: read %.0f GB/s, copy %.0f GB/s (read + write bytes)"
        % (probe["read_GBps"], probe["copy_GBps"]))
    single = bool(args.workload)
    head_name = args.workload or HEADLINE
    want_cpu = not args.no_cpu_baseline and not args.page_size and args.selection == "sum"
    head = measure(args, torch, tidal, W, dev, head_name, over, (args.k,), probe, want_cpu)[0]
    configs = []
    if not single:
        for name, ks in OTHERS:
            configs += measure(args, torch, tidal, W, dev, name, {}, ks, probe, False)

    out = {
        "metric": "decode_step_attention_us", "value": head["us_per_step"], "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(head["us_per_step"] / 1e3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": head["config"],
        "step_hbm": head["step_hbm"],
        "per_layer_kind": head["per_layer_kind"],
        "hbm_probe": probe,
        "roofline": head["roofline"],
        "cpu_baseline": head["cpu_baseline"],
    }
    if not single:
        out["configs"] = [{x: c[x] for x in ("config", "us_per_step", "step_hbm", "per_layer_kind", "roofline")}
                          for c in configs]
    print(json.dumps(out), flush=True)


def kernel_name(tidal, W, shape, kind, k, w):
    """The attention kernel that a layer of this kind launches, from the library's own launch plan."""
    plan = tidal.plan_launch(shape, kind, k)
    mode = {W.DENSE: "dense", W.SELECT: "select", W.SPARSE: "sparse"}[kind]
    if plan.matrix_core:
        return "attend_mfma_kernel<G=%d, %s, %d waves>" % (w.group, mode, plan.waves_per_workgroup)
    return "attend_split_kernel<%s, d=%d, G=%d, %s, %d waves>" % (w.dtype, w.head_dim, w.group, mode,
                                                                  plan.waves_per_workgroup)


def measure(args, torch, tidal, W, dev, name, over, ks, probe, want_cpu):
    """Times one workload (inputs generated once) for every budget in ks (0: the workload's own).
    Returns one record per budget."""
    w0 = W.workload(name, **over)
    cache_bytes = w0.num_layers * 2 * w0.batch * w0.num_kv_heads * w0.max_seq_len * w0.head_dim * w0.elem_bytes
    copies = args.copies or (3 if cache_bytes <= 8 * 2**30 else 1)
    log("%s: cache %.1f GiB per copy, %d cop%s" % (w0.name, cache_bytes / 2**30, copies, "y" if copies == 1 else "ies"))
    lens = torch.tensor(w0.seq_lens, dtype=torch.int32, device=dev)
    n_sel = sum(1 for x in w0.schedule if x == W.SELECT)
    selection = {"sum": tidal.SELECT_GROUP_SUM, "max": tidal.SELECT_GROUP_MAX, "per_head": tidal.SELECT_PER_HEAD,
                 "mean_prob": tidal.SELECT_GROUP_MEAN_PROB}[args.selection]
    sel_rows = w0.num_q_heads if args.selection == "per_head" else w0.num_kv_heads
    inputs, all_news = [], []
    for c in range(copies):
        wc = W.workload(name, seed=w0.seed + 7919 * c, **over)
        heavy = W.heavy_positions(wc)
        ranks = W.zipf_ranks(wc) if wc.structure == "zipf" else None
        layers = [W.make_layer(wc, i, dev, heavy=heavy, ranks=ranks) for i in range(wc.num_layers)]
        if args.page_size:      # the same tokens, scattered over a page pool; all copies share the table
            if c == 0:
                table, num_pages = W.page_table(w0, args.page_size, device=dev)
            paged = []
            for q, K, V in layers:
                Kp, Kv = W.paginate(K, table, num_pages, args.page_size, args.page_layout)
                Vp, _ = W.paginate(V, table, num_pages, args.page_size, args.page_layout)
                paged.append((q, Kp, Vp))
                pool_view = Kv
            layers = paged
        if args.append and not args.page_size:   # the current token's rows, handed over separately
            news = [(torch.stack([K[b, :, n - 1] for b, n in enumerate(w0.seq_lens)]).contiguous(),
                     torch.stack([V[b, :, n - 1] for b, n in enumerate(w0.seq_lens)]).contiguous()) for _, K, V in layers]
        elif args.append:
            news = [(torch.randn((w0.batch, w0.num_kv_heads, w0.head_dim), device=dev).to(w0.torch_dtype),
                     torch.randn((w0.batch, w0.num_kv_heads, w0.head_dim), device=dev).to(w0.torch_dtype)) for _ in layers]
        else:
            news = None
        qs, Ks, Vs = zip(*layers)
        outs = [torch.zeros_like(q) for q in qs]
        inputs.append((qs, Ks, Vs, outs))
        all_news.append(news)
        log("generated copy %d" % c)
    if args.page_size:
        shape = tidal.make_paged_shape(inputs[0][0][0], pool_view, table, lens, w0.max_seq_len,
                                       total_seq_len=sum(w0.seq_lens), selection=selection)
    else:
        shape = tidal.make_shape(inputs[0][0][0], inputs[0][1][0], lens, total_seq_len=sum(w0.seq_lens),
                                 selection=selection)

    records = []
    for k_over in ks:
        w = W.workload(name, **dict(over, k=k_over)) if k_over else w0
        sets = [(qs, Ks, Vs, outs, torch.full((n_sel, w.batch, sel_rows, w.k), -1, dtype=torch.int32, device=dev))
                for qs, Ks, Vs, outs in inputs]
        rec = measure_budget(args, torch, tidal, W, dev, w, over, shape, lens, sets, all_news, copies, sel_rows, probe)
        rec["cpu_baseline"] = cpu_baseline(w, sets[0], torch) if want_cpu else None
        records.append(rec)
    del inputs, all_news, sets
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return records


def measure_budget(args, torch, tidal, W, dev, w, over, shape, lens, sets, all_news, copies, sel_rows, probe):
    step_bytes = w.algorithmic_bytes_per_step()
    td = tidal.Tidal(shape, w.k, topk_rows=w.batch * sel_rows, topk_max_len=w.max_seq_len)
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
    us_per_step = (t1 - t0) / args.steps * 1e6
    log("%s k=%d: %.1f us per decode step (%s)" % (w.name, w.k, us_per_step, "graph replay" if use_graph else "eager"))

    # Per-launch duration of each layer kind: `reps` launches of that kind (rotating over input
    # copies and layers, so each launch streams data that is not in cache) are captured into one
    # HIP graph; HIP events on the launch stream bracket each replay.  Back-to-back kernels in a
    # graph leave gaps well under a microsecond, so time / reps is the kernel's own duration.
    scores = torch.zeros((w.batch, sel_rows, w.max_seq_len), dtype=torch.float32, device=dev)

    def time_launches(launch_one, reps):
        def launches():
            for r in range(reps):
                launch_one(r)

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

    def time_kind(kind, reps):
        idx = [i for i, x in enumerate(w.schedule) if x == kind]
        if not idx:
            return None

        def one(r):
            qs, Ks, Vs, outs, pos = sets[r % copies]
            i = idx[(r // copies) % len(idx)]
            if kind == W.DENSE:
                td.full_attend(shape, qs[i], Ks[i], Vs[i], outs[i])
            elif kind == W.SELECT:
                td.select_tokens(shape, qs[i], Ks[i], Vs[i], w.k, outs[i], pos[0], scores)
            else:
                td.sparse_attend(shape, qs[i], Ks[i], Vs[i], pos[0], w.k, outs[i])

        return time_launches(one, reps)

    kv_bytes = w.kv_bytes_per_layer()
    score_bytes = sum(w.seq_lens) * sel_rows * 4
    pos_bytes = w.batch * sel_rows * w.k * 4
    read_peak = probe["read_GBps"]
    per_kind = {}
    for kname, kind in zip(KIND_NAMES, (W.DENSE, W.SELECT, W.SPARSE)):
        r = time_kind(kind, args.kernel_reps)
        if r:
            per_kind[kname] = {"layers": sum(1 for x in w.schedule if x == kind),
                               "avg_us": round(r[0], 2), "median_us": round(r[1], 2)}
    if "select" in per_kind:
        # the selection layer's attention launch alone (fused score write and score histogram): the same calls
        # with the library's timing switch that stops a selection call after its attention launch
        tune = [int(x) for x in args.tune.split(",")] if args.tune else [0, 0, 0, 0, 0]
        td.set_tuning(*(tune[:4] + [tune[4] | 32]))
        td.reset()          # the switch marks the rows' state for clearing: do it here, not inside the timed graph
        r = time_kind(W.SELECT, args.kernel_reps)
        td.set_tuning(*tune)
        td.reset()
        per_kind["select"]["attention_us"] = round(r[0], 2)
        per_kind["select"]["topk_us"] = round(per_kind["select"]["avg_us"] - r[0], 2)
    # algorithmic bytes per layer of each kind: K and V once; a selection layer also writes the fp32
    # scores and reads them back for the top-k, and writes rho; a sparse layer reads rho and its rows
    layer_bytes = {"full": kv_bytes, "select": kv_bytes + 2 * score_bytes + pos_bytes,
                   "sparse": w.sparse_bytes_per_layer() * (w.group if args.selection == "per_head" else 1) + pos_bytes}
    for kname, d in per_kind.items():
        gbps = layer_bytes[kname] / (d["avg_us"] * 1e-6) / 1e9
        d.update({"algorithmic_bytes": layer_bytes[kname], "GBps": round(gbps, 1),
                  "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4), "frac_of_measured_read": round(gbps / read_peak, 4),
                  "share_of_step": round(d["layers"] * d["avg_us"] / us_per_step, 4)})

    # Roofline of the dominant kernel: the attention launch of the layer kind with the largest
    # share of this run's step time (a selection layer's attention launch is timed with its top-k switched off).
    launch_us = {kname: d.get("attention_us", d["avg_us"]) for kname, d in per_kind.items()}
    dominant = max(per_kind, key=lambda n: per_kind[n]["layers"] * launch_us[n])
    launch_bytes = {"full": kv_bytes, "select": kv_bytes + score_bytes, "sparse": layer_bytes["sparse"]}[dominant]
    kind_code = {"full": W.DENSE, "select": W.SELECT, "sparse": W.SPARSE}[dominant]
    achieved = launch_bytes / (launch_us[dominant] * 1e-6) / 1e9
    traffic, traffic_source = None, None
    tpath = os.path.join("profiles", "attend_%s_%s_traffic.json" % (dominant, w.name))
    if os.path.exists(os.path.join(ROOT, tpath)) and not over and not args.page_size:
        with open(os.path.join(ROOT, tpath)) as f:
            t = json.load(f)
        if t.get("k", w.k) == w.k:
            traffic = t.get("hbm_bytes_per_launch")
            traffic_source = tpath + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this kernel on this workload, not of this run)"
    roofline = {"kernel": kernel_name(tidal, W, shape, kind_code, w.k, w) + ": the %s-layer attention launch, %d per step, "
                          "the launch with the largest share of this run's step time (%.0f %%)"
                          % (dominant, per_kind[dominant]["layers"],
                             100.0 * per_kind[dominant]["layers"] * launch_us[dominant] / us_per_step),
                "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_source,
                "algorithmic_bytes_per_launch": launch_bytes, "avg_launch_us": round(launch_us[dominant], 2),
                "frac_of_measured_read": round(achieved / read_peak, 4),
                "per_kind_frac": {n: per_kind[n]["frac_of_peak"] for n in per_kind}}

    desc = DESCRIPTIONS[w.name] + "".join(", %s overridden to %s" % (a, b) for a, b in sorted(over.items()))
    if args.page_size:
        desc += ", cache in pages of %d tokens (%s) behind a shuffled block table" % (args.page_size, args.page_layout)
    step_gbps = step_bytes / (us_per_step * 1e-6) / 1e9
    rec = {
        "us_per_step": round(us_per_step, 2), "dtype": w.dtype,
        "config": {"workload": desc, "k": w.k, "selection": args.selection, "input_copies_rotated": copies,
                   "launch": ("hip graph replay of " if use_graph else "eager ") +
                             ("td_decode_step_append" if args.append else "td_decode_step")},
        "step_hbm": {"algorithmic_bytes": step_bytes, "achieved_GBps": round(step_gbps, 1),
                     "frac_of_peak": round(step_gbps / HBM_PEAK_GBPS, 4),
                     "frac_of_measured_read": round(step_gbps / read_peak, 4)},
        "per_layer_kind": per_kind,
        "roofline": roofline,
    }
    del graphs
    td.close()
    return rec


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
    cpu = None
    if not args.no_cpu_baseline and not args.page_size:
        # the oracle's causal attention for a bounded sample of the new tokens (the last ones, which see the
        # most positions), scaled to all of them by the positions they see
        from oracle import tidal_oracle as O
        sample = min(P, 8)
        qh, Kh, Vh = q[:, P - sample:].cpu().contiguous(), K.cpu(), V.cpu()
        t0 = time.perf_counter()
        O.prefill(qh, Kh, Vh, w.seq_lens)
        dt = time.perf_counter() - t0
        seen_sample = sum(sum(max(n - sample + j + 1, 0) for j in range(sample)) for n in w.seq_lens)
        seen_all = sum(sum(max(n - P + j + 1, 0) for j in range(P)) for n in w.seq_lens)
        cpu = {"value": round(dt * 1e6 * seen_all / max(seen_sample, 1), 1), "unit": "us", "cores": O.num_threads(),
               "kind": "oracle",
               "sample": "the last %d of the %d new tokens of every sequence, scaled by the positions attended" % (sample, P)}
    seen = sum(sum(max(n - P + j + 1, 0) for j in range(P)) for n in w.seq_lens)
    flop = 4.0 * w.head_dim * w.num_q_heads * seen
    # the keys and values of every position some new token sees, once
    esize = 2 if w.dtype == "bf16" else 4
    kv_bytes = 2.0 * w.num_kv_heads * w.head_dim * esize * sum(w.seq_lens)
    td.close()
    # shapes outside the matrix-core kernel take the library's plain path: the vector-ALU full-attention kernel,
    # one grid row block per new token, which streams the cache once per new token
    plain = w.dtype != "bf16" or w.head_dim != 128 or (args.page_size and args.page_size < 16)
    if plain:
        rate = kv_bytes / (us * 1e-6) / 1e9
        roof = {"kernel": "attend_split_kernel (plain path: the cache is read once per new token, %d times here)" % P,
                "bound": "hbm", "achieved": round(rate, 1), "peak": 8000.0, "unit": "GB/s", "frac": round(rate / 8000.0, 4),
                "traffic": None, "bytes_per_launch": kv_bytes, "flop_per_launch": flop}
    # whichever of the two floors is higher for this P names the bound
    elif kv_bytes / 8.0e12 > flop / 2.5e15:
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
            "median_us": round(ts[len(ts) // 2], 2), "roofline": roof, "cpu_baseline": cpu}


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

    Small caches: every layer of one decode step.  Large caches: every full and selection layer and
    the first four sparse layers, the sparse time scaled to the number of sparse layers (stated in `sample`)."""
    from oracle import tidal_oracle as O
    import workloads as W
    qs, Ks, Vs, _, _ = inputs
    layer_bytes = 2 * Ks[0].numel() * Ks[0].element_size()
    whole = layer_bytes * w.num_layers <= 6 * 2**30
    kinds = list(w.schedule)
    if whole:
        todo = list(range(w.num_layers))
    else:
        todo = [i for i, x in enumerate(kinds) if x != W.SPARSE] + [i for i, x in enumerate(kinds) if x == W.SPARSE][:4]
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
              "every full and selection layer and the first four sparse layers of one %s decode step, one layer at a "
              "time, the sparse time scaled to its %d sparse layers" % (w.name, kinds.count(W.SPARSE)))
    return {"value": round(total * 1e6, 1), "unit": "us", "cores": O.num_threads(), "kind": "oracle",
            "sample": sample}


if __name__ == "__main__":
    main()
