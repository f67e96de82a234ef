#!/usr/bin/env python3
"""Benchmark of the KV-Compress hot path on one MI355X.

A step = one pass of the path over the batch: append the new token's k, v for
every (sequence, layer, KV head), then one paged decode over all layers with
metric accumulation; every --evict-every steps a compression round (block keys
-> selection -> compaction) returns as many blocks as were appended since the
last round, so the cache stays at its compression rate.

Workload at N = 1: the Llama-3.1-8B-shaped decode (32 layers, 32 q / 8 KV
heads, d = 128, bf16, b = 16, 64 sequences of 8192 prompt tokens, per-head
retention log-uniform with mean 8x), synthetic data, inputs resident in HBM.

Prints ONE JSON line.  value = algorithmic decode bytes moved per second over
the whole timed region (append and compression rounds included in the time).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def algorithmic_bytes_per_kv(shape):
    """K row + V row read, metric read + write (f32), one table entry per b KVs."""
    return 2 * shape.head_dim * shape.kv_bytes + 8 + 4.0 / shape.block_size


def read_traffic_note(name):
    """HBM bytes per launch measured with rocprofv3 --pmc, kept as text under profiles/."""
    p = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(p):
        return None
    for line in open(p):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


def cpu_baseline(sess, q, shape, n_heads, seed, budget_s=12.0):
    """Times the CPU oracle, as it stands, on a sample of head instances."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_limits
    from oracle import kvc_oracle as O
    from paper_2410_00161_amd import workloads as W
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import oracle_state
    g = torch.Generator().manual_seed(seed)
    heads = torch.randperm(shape.G, generator=g)[:n_heads].tolist()
    small, q_small = W.gather_heads(sess.cache, heads, q)
    st = oracle_state(small)
    kvs = int(st.lens().sum())
    reps, dt = 0, 0.0
    with threadpool_limits(limits=1):
        while dt < budget_s:                      # whole decode steps until the time budget is used
            t0 = time.perf_counter()
            O.paged_decode(st, q_small.double().numpy())
            key, _ = O.block_keys(st)
            dt += time.perf_counter() - t0
            reps += 1
    gbs = reps * kvs * algorithmic_bytes_per_kv(shape) / dt / 1e9
    return {"value": gbs, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{n_heads} of {shape.G} head instances ({kvs} KVs) x {reps} decode steps with "
                      f"metric accumulation + block keys, {dt:.1f} s, numpy fp64 oracle, BLAS limited to 1 thread"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--evict-every", type=int, default=16)
    ap.add_argument("--num-seqs", type=int, default=64)
    ap.add_argument("--prompt", type=int, default=8192)
    ap.add_argument("--rho", type=float, default=8.0, help="mean compression rate")
    ap.add_argument("--placement", default="fresh", choices=["fresh", "fragmented"])
    ap.add_argument("--chunk", type=int, default=0, help="decode chunk tokens (0 = library default)")
    ap.add_argument("--cpu-heads", type=int, default=1024, help="head instances timed on the CPU oracle (0 = skip)")
    ap.add_argument("--workload", default="llama8b", choices=["llama8b", "llama70b"])
    ap.add_argument("--block-size", type=int, default=16, choices=[16, 32, 64],
                    help="variant (llama8b workload): tokens per cache block")
    ap.add_argument("--kv-dtype", default="bf16", choices=["bf16", "fp8"],
                    help="variant: K and V stored as OCP e4m3 bytes (queries stay bf16)")
    ap.add_argument("--evict-mode", default="block", choices=["block", "rank"],
                    help="block: physical blocks by summed metric; rank: the paper's rank-block schedule")
    ap.add_argument("--uniform", action="store_true", help="diagnostic: every head holds prompt/rho KVs")
    ap.add_argument("--no-metric", action="store_true", help="diagnostic: decode without metric accumulation")
    ap.add_argument("--per-layer-steps", type=int, default=4,
                    help="extra untimed-region steps that call the decode once per layer (0 = skip)")
    ap.add_argument("--all-queries-block", type=int, default=1024, choices=[32, 64, 256, 1024],
                    help="queries per call when the prefill-end probe gathers the metric over all prompt queries")
    ap.add_argument("--window-probe", type=int, default=1,
                    help="also time the observation-window metric and a rank-block eviction to 8x on a "
                         "Mistral-7B-shaped 16384-token prompt (0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known traffic, for scaling rocprofv3 counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(every step is independent per head instance and would shard without communication).",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2410_00161_amd import binding as B, workloads as W
    from paper_2410_00161_amd.session import KvcSession
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    total_steps = args.steps + args.warmup
    extra = total_steps + 2 * args.evict_every + 16
    if args.workload == "llama8b":
        shape, ctx, seed = W.llama8b_decode(num_seqs=args.num_seqs, prompt=args.prompt, rho=args.rho,
                                            extra_tokens=extra, block_size=args.block_size)
        name = (f"Llama-3.1-8B-shaped decode: 32 layers, 32q/8kv heads, d=128, {args.kv_dtype} KV, b={args.block_size}, "
                f"{args.num_seqs} seqs x {args.prompt} prompt tokens, per-head retention log-uniform mean {args.rho:g}x")
    else:
        shape, ctx, seed = W.llama70b_decode(num_seqs=args.num_seqs, prompt=args.prompt, rho=args.rho,
                                             extra_tokens=extra)
        name = (f"Llama-3.1-70B-shaped decode: 80 layers, 64q/8kv heads, d=128, {args.kv_dtype} KV, b=16, "
                f"{args.num_seqs} seqs x {args.prompt} prompt tokens, per-head retention log-uniform mean {args.rho:g}x")
    if args.kv_dtype != "bf16":
        import dataclasses
        shape = dataclasses.replace(shape, kv_dtype=args.kv_dtype)
    if args.uniform:
        ctx = W.uniform_lengths(shape.G, int(args.prompt / args.rho))
        name += " [diagnostic: uniform lengths]"
    t_setup = time.perf_counter()
    cache = W.make_cache(shape, ctx, seed, device=dev, placement=args.placement, init_metric="prefill")
    sess = KvcSession(cache, device=dev)
    del cache
    B.kvc_set_decode_chunk(args.chunk)
    bytes_kv = algorithmic_bytes_per_kv(shape)
    G = shape.G
    per_seq = shape.num_layers * shape.num_kv_heads
    print(f"[bench] {name}", file=sys.stderr)
    print(f"[bench] G={G} head instances, {int(ctx.sum())} KVs, {shape.num_blocks} blocks in the pool, "
          f"realised compression {args.prompt * G / float(ctx.sum()):.2f}x, "
          f"setup {time.perf_counter() - t_setup:.1f}s", file=sys.stderr, flush=True)

    # pre-generated inputs for a few steps, reused round-robin (they stay in HBM)
    n_in = 4
    qs = [W.make_query(shape, seed, i, dev) for i in range(n_in)]
    kvs_new = [W.make_new_kv(shape, seed, i, dev) for i in range(n_in)]
    snaps = {}   # step -> context lengths the decode of that step saw
    snap_every = args.evict_every if args.evict_every > 0 else 16
    prof_every = 4
    budget = torch.full((shape.num_seqs,), per_seq * args.evict_every // shape.block_size,
                        dtype=torch.int32, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    evict_events = []

    def step(i, timed):
        k, v = kvs_new[i % n_in]
        sess.append(k, v, flags=B.KVC_ASYNC)
        if timed:
            B.kvc_profile_enable((i - args.warmup) % prof_every == 0)
        sess.paged_decode(qs[i % n_in], accumulate_metric=not args.no_metric)
        if i % snap_every == 0 or i == args.warmup:
            snaps[i] = sess.cache.ctx_len.reshape(-1).clone()
        if args.evict_every > 0 and (i + 1) % args.evict_every == 0:
            e = [ev() for _ in range(4)]
            e[0].record()
            if args.evict_mode == "block":
                sess.metric_reduce()
                e[1].record()
                sess.evict_select(budget, flags=B.KVC_ASYNC)
                e[2].record()
                sess.compact(flags=B.KVC_ASYNC)
            else:
                e[1].record()
                sess.evict_rank_select(budget, flags=B.KVC_ASYNC)
                e[2].record()
                sess.compact_rank(flags=B.KVC_ASYNC)
            e[3].record()
            if timed:
                evict_events.append(e)

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    assert B.kvc_poll_status(sess.cfg, sess.ws) == B.KVC_OK
    B.kvc_profile_begin((args.steps + prof_every - 1) // prof_every)
    t0, t1 = ev(), ev()
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    t0.record()
    for i in range(args.warmup, total_steps):
        step(i, True)
    t1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    status = B.kvc_poll_status(sess.cfg, sess.ws)
    if status != B.KVC_OK:
        print(f"bench.py: device-side error {status} ({B.status_string(status)})", file=sys.stderr)
        sys.exit(1)
    ms_total = t0.elapsed_time(t1)
    chunk_ms, short_ms, combine_ms = B.kvc_profile_collect(4096)
    B.kvc_profile_begin(0)

    # Between two compression rounds every head grows by exactly one KV per step, so the
    # lengths each decode saw follow from the snapshot taken at the start of the period.
    # A head of C tokens is cut into chunks of chunk_T; a last chunk (or whole head) of at most
    # short_T tokens runs in the short-item launch, everything else in the long-item launch.  A
    # head of one chunk gets its metric from the launch that streams it, others from the combine.
    chunk_T = B.kvc_get_decode_chunk(sess.cfg)
    short_T = B.kvc_get_decode_short(sess.cfg)
    kv_per_step, long_kv, long_single, short_single = [], [], [], []
    keys = sorted(snaps)
    for i in range(args.warmup, total_steps):
        s0 = max(k for k in keys if k <= i)
        c = snaps[s0].to(torch.int64) + (i - s0)
        rem = c % chunk_T
        in_short = rem * ((rem > 0) & (rem <= short_T))
        kv_per_step.append(float(c.sum()))
        long_kv.append(float((c - in_short).sum()))
        long_single.append(float((c * ((c <= chunk_T) & (c > short_T))).sum()))
        short_single.append(float((c * (c <= min(short_T, chunk_T))).sum()))
    kv_per_step, long_kv = np.array(kv_per_step), np.array(long_kv)
    long_single, short_single = np.array(long_single), np.array(short_single)
    total_bytes = float(kv_per_step.sum()) * bytes_kv
    value = total_bytes / (ms_total * 1e-3) / 1e9
    ms_step = ms_total / args.steps

    # dominant kernel: decode_chunk_kernel over the long items (four wavefronts per item): streams
    # their K and V once, metric RMW for heads of one chunk
    per_kv = 2 * shape.head_dim * shape.kv_bytes + 4.0 / shape.block_size
    chunk_alg = long_kv * per_kv + 8.0 * long_single
    short_alg = (kv_per_step - long_kv) * per_kv + 8.0 * short_single
    chunk_ms = np.array(chunk_ms, dtype=np.float64)
    short_ms = np.array(short_ms, dtype=np.float64)
    combine_ms = np.array(combine_ms, dtype=np.float64)
    chunk_alg_s = chunk_alg[::prof_every][:len(chunk_ms)]          # the steps that were timed
    short_alg_s = short_alg[::prof_every][:len(chunk_ms)]
    ach = float(chunk_alg_s.mean() / (chunk_ms.mean() * 1e-3) / 1e9)
    traffic = read_traffic_note("decode_chunk_kernel_llama8b_pmc.txt") if args.workload == "llama8b" else None
    roofline = {"bound": "hbm", "kernel": "decode_chunk_kernel<%d,128,%d,b16,4> (long items)" % (shape.kv_bytes, shape.group_size),
                "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                "traffic": traffic, "avg_kernel_ms": float(chunk_ms.mean()),
                "algorithmic_bytes_per_launch": float(chunk_alg_s.mean()),
                "timed_launches": int(len(chunk_ms)),
                "short_items_kernel_ms": float(short_ms.mean()),
                "short_items_GBps": float(short_alg_s.mean() / (short_ms.mean() * 1e-3) / 1e9),
                "short_items_max_tokens": short_T,
                "decode_call_GBps": float((kv_per_step[::prof_every][:len(chunk_ms)] * bytes_kv).mean() /
                                          ((chunk_ms + short_ms + combine_ms).mean() * 1e-3) / 1e9),
                "combine_kernel_ms": float(combine_ms.mean())}

    # measured streaming-read ceiling of this GPU: the K cache read once with plain 16-byte loads
    nbytes = sess.cache.k_cache.numel() * sess.cache.k_cache.element_size()
    nbytes -= nbytes % 16
    sink = torch.zeros(65536, dtype=torch.int32, device=dev)
    best = 0.0
    for wgs in (2048, 4096, 8192, 16384):
        for _ in range(3):
            a, b_ = ev(), ev()
            a.record()
            B.kvc_stream_read_probe(sess.cache.k_cache, nbytes, sink, wgs)
            b_.record()
            torch.cuda.synchronize()
            best = max(best, nbytes / (a.elapsed_time(b_) * 1e-3) / 1e9)
    roofline["measured_stream_read_GBps"] = best
    roofline["frac_of_measured_stream_read"] = ach / best

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # the same decode issued the way a model runs it: one call per layer (no append, no metric
    # writes skipped), a few steps, reported beside the all-layers launch
    per_layer_ms = per_layer_graph_ms = None
    if args.per_layer_steps > 0:
        a, b_ = ev(), ev()
        torch.cuda.synchronize()
        a.record()
        for i in range(args.per_layer_steps):
            for l in range(shape.num_layers):
                sess.paged_decode(qs[i % n_in], accumulate_metric=not args.no_metric, layer_begin=l, layer_end=l + 1)
        b_.record()
        torch.cuda.synchronize()
        per_layer_ms = a.elapsed_time(b_) / args.per_layer_steps
        # the same 32 calls captured once into a HIP graph and replayed
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            for l in range(shape.num_layers):
                sess.paged_decode(qs[0], accumulate_metric=not args.no_metric, layer_begin=l, layer_end=l + 1)
        torch.cuda.synchronize()
        a, b_ = ev(), ev()
        a.record()
        for i in range(args.per_layer_steps):
            graph.replay()
        b_.record()
        torch.cuda.synchronize()
        per_layer_graph_ms = a.elapsed_time(b_) / args.per_layer_steps
        del graph

    # prefill-end compression, Mistral-7B shape: one 16384-token prompt, metric from the last 32
    # prompt queries on the matrix cores, then rank-block eviction to 8x
    prefill_end = None
    if args.window_probe:
        Lp, wq = 16384, 32
        shp = W.Shape(1, 32, 8, 4, 128, 16, 256 * (Lp // 16) + 512, Lp // 16 + 2, "bf16")
        c4 = W.make_cache(shp, W.uniform_lengths(shp.G, Lp), 1004, device=dev)
        s4 = KvcSession(c4, device=dev)
        del c4
        g4 = torch.Generator(device=dev).manual_seed(1004)
        qw = torch.randn((1, 32, 32, wq, 128), generator=g4, device=dev, dtype=torch.float32).to(torch.bfloat16)
        # the metric over ALL prompt queries (every query attends to the keys at least 10
        # positions before it), gathered one block of 1024 queries at a time; the same random
        # block of queries stands in for every block of the prompt
        wb, excl = args.all_queries_block, 10
        qb = torch.randn((1, 32, 32, wb, 128), generator=g4, device=dev, dtype=torch.float32).to(torch.bfloat16)
        s4.cache.metric.zero_()
        a, b_ = ev(), ev()
        a.record()
        for start in range(0, Lp, wb):
            s4.query_block_metric(qb, wb, start, excl)
        b_.record()
        torch.cuda.synchronize()
        all_queries_ms = a.elapsed_time(b_)
        del qb
        best = 1e9
        for _ in range(4):
            a, b_ = ev(), ev()
            a.record()
            s4.window_metric(qw, wq, 7)
            b_.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b_))
        kvs4 = shp.G * Lp
        bud4 = torch.tensor([shp.G * (Lp // 16) * 7 // 8], dtype=torch.int32, device=dev)
        s4.evict_rank_select(bud4, flags=B.KVC_ASYNC)   # untimed first call (selection changes no cache state)
        torch.cuda.synchronize()
        a, b_, c_ = ev(), ev(), ev()
        a.record()
        s4.evict_rank_select(bud4, flags=B.KVC_ASYNC)
        b_.record()
        s4.compact_rank(flags=B.KVC_ASYNC)
        c_.record()
        torch.cuda.synchronize()
        assert B.kvc_poll_status(s4.cfg, s4.ws) == B.KVC_OK
        kvs_after = int(s4.cache.ctx_len.sum().item())
        select_ms, compact_ms = a.elapsed_time(b_), b_.elapsed_time(c_)
        # then 256 decode steps on what is left (append + decode + metric)
        q4 = [W.make_query(shp, 1004, i, dev) for i in range(2)]
        kv4 = [W.make_new_kv(shp, 1004, i, dev) for i in range(2)]
        nd = 256
        a, b_ = ev(), ev()
        a.record()
        for i in range(nd):
            s4.append(*kv4[i % 2], flags=B.KVC_ASYNC)
            s4.paged_decode(q4[i % 2])
        b_.record()
        torch.cuda.synchronize()
        assert B.kvc_poll_status(s4.cfg, s4.ws) == B.KVC_OK
        decode_ms = a.elapsed_time(b_) / nd
        prefill_end = {"workload": "Mistral-7B-shaped: 32 layers, 32q/8kv heads, d=128, bf16, one 16384-token prompt",
                       "window_queries": wq, "pool": 7, "window_metric_ms": best,
                       "window_metric_K_GBps": 2 * 256 * kvs4 / (best * 1e-3) / 1e9,
                       "window_metric_TFLOPs": 2 * 2 * (wq * 4) * 128 * kvs4 / (best * 1e-3) / 1e12,
                       "rank_select_to_8x_ms": select_ms, "rank_compact_ms": compact_ms,
                       "kvs_after": kvs_after, "kvs_before": kvs4,
                       "all_queries_metric_ms": all_queries_ms, "all_queries_block": wb, "all_queries_exclude": excl,
                       "all_queries_TFLOPs": 2 * 2 * (4 * 128) * shp.G * (Lp * (Lp + min(wb, 64)) / 2) / (all_queries_ms * 1e-3) / 1e12,
                       "decode_steps_after": nd, "decode_ms_per_step_after": decode_ms,
                       "decode_GBps_after": (kvs_after + shp.G * nd / 2) * algorithmic_bytes_per_kv(shp) / (decode_ms * 1e-3) / 1e9}
        del s4, qw, q4, kv4

    evict = None
    if evict_events:
        r = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(3)] for e in evict_events])
        evict = {"mode": args.evict_mode, "rounds": len(evict_events), "reduce_ms": float(r[:, 0].mean()),
                 "select_ms": float(r[:, 1].mean()), "compact_ms": float(r[:, 2].mean()),
                 "total_ms": float(r.sum(1).mean()), "blocks_per_round": int(budget.sum().item())}

    cpu = None
    if args.cpu_heads > 0:
        cpu = cpu_baseline(sess, qs[0], shape, args.cpu_heads, seed)

    out = {
        "metric": "decode-attn HBM GB/s (% of peak) at 8x compression; eviction+compaction ms",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if args.kv_dtype == "bf16" else "fp8 K/V (e4m3), bf16 q, f32 accumulation", "data": "synthetic",
        "config": {"workload": name, "placement": args.placement, "evict_every": args.evict_every,
                   "evict_mode": args.evict_mode,
                   "chunk_tokens": chunk_T, "head_instances": G,
                   "mean_kvs_per_step": float(kv_per_step.mean())},
        "frac_of_hbm_peak": value / HBM_PEAK_GBS,
        "kv_only_GBps": float(kv_per_step.sum()) * 2 * shape.head_dim * shape.kv_bytes / (ms_total * 1e-3) / 1e9,
        "decode_steps_per_s": 1e3 / ms_step,
        "decode_only_ms_per_step_one_call_per_layer": per_layer_ms,
        "decode_only_ms_per_step_one_call_per_layer_hip_graph": per_layer_graph_ms,
        "wall_s": wall,
        "eviction": evict,
        "prefill_end": prefill_end,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "gpu": torch.cuda.get_device_name(0), "host_cpus": os.cpu_count(),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
