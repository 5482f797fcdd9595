#!/usr/bin/env python3
"""Benchmark of the GNS hot path on one MI355X.

A step is one mini-batch through the whole path: (periodic cache draw) ->
gns_sample_blocks -> gns_gather_features (input nodes) -> gns_aggregate (input
layer).  The workload is the medium power-law graph (1M nodes, ~20M undirected
edges, 128-dim fp32 features in HBM, 1% degree-proportional cache redrawn every
20 mini-batches, fan-outs 15/10/5, batch 1024), seeded and synthetic.

Prints one JSON line: whole-job mini-batches/s with inputs resident in HBM, the
roofline figures of the dominant kernel (HIP-event timed inside the timed
region), and the CPU oracle's rate on a bounded sample of the same batches.
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", type=int, default=2, help="workload id (see synth.CONFIGS)")
    ap.add_argument("--cpu-batches", type=int, default=32, help="mini-batches the CPU oracle is timed on (0: skip)")
    ap.add_argument("--stages", action="store_true", help="add an untimed pass that times every stage")
    ap.add_argument("--threads", type=int, default=0, help="1: one host thread per slot")
    ap.add_argument("--flag-mode", type=int, default=0,
                    help="0: membership flags per mini-batch (CSR-segment scan); 1: once per cache draw")
    ap.add_argument("--slots", type=int, default=4,
                    help="mini-batches kept in flight (one context + stream each; they share the cache)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2106_06150_amd import binding as B
    from paper_2106_06150_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg_id = args.config
    c = synth.CONFIGS[cfg_id]
    sd = synth.config_seeds(cfg_id)
    n, F, batch = c["n"], c["feat"], c["batch"]
    fanouts = list(c["fanouts"])
    L = len(fanouts)
    policies = [B.GNS_UNIFORM] * (L - 1) + [B.GNS_CACHE_ONLY]
    cache_size = int(n * c["cache_frac"])
    refresh = c.get("refresh_every", 20)

    # ---- inputs (generated on the device, resident in HBM before timing starts)
    g = synth.make_config_graph(cfg_id, device=dev)
    feat = synth.node_features(n, F, sd["feat"], device=dev)
    total = args.warmup + args.steps
    seeds = [synth.uniform_seed_batch(n, batch, sd["batch"] + b, device=dev) for b in range(total)]
    deg = (g.indptr[1:] - g.indptr[:-1]).to(torch.int64)

    graph = B.make_graph(g.indptr, g.indices, feat_dev=feat)
    config = B.make_config(fanouts, policies, cache_size, batch, flag_mode=args.flag_mode)
    ws = B.alloc_workspace(graph, config, dev)
    ctx = B.gns_create(graph, config, ws)
    last = L - 1
    # one slot = context + stream + output buffers; slot 0 is the created context, the others are forks
    S = max(1, args.slots)
    ctxs, fork_ws = [ctx], []
    for _ in range(S - 1):
        w = torch.empty(B.gns_fork_workspace_bytes(ctx), dtype=torch.uint8, device=dev)
        fork_ws.append(w)
        ctxs.append(B.gns_fork(ctx, w))
    streams = [torch.cuda.Stream() for _ in range(S)]
    bufs = [B.BlockBuffers(graph, config, dev) for _ in range(S)]
    x_in = [torch.empty((bufs[i].array[last].cap_src, F), dtype=torch.float32, device=dev) for i in range(S)]
    h_out = [torch.empty((bufs[i].array[last].cap_dst, F), dtype=torch.float32, device=dev) for i in range(S)]
    blocks = bufs[0]

    def step(b):
        """One mini-batch, enqueued on its slot's stream without any host synchronisation."""
        if b % refresh == 0:
            torch.cuda.synchronize()                      # no batch may be in flight while the cache changes
            B.gns_sample_cache(ctx, sd["cache"], b // refresh, streams[0])
        i = b % S
        st = streams[i]
        B.gns_sample_blocks_async(ctxs[i], sd["batch"] + b, seeds[b], bufs[i].array, st)
        B.gns_gather_features(ctxs[i], bufs[i].tensors[last]["src_nodes"], -1, x_in[i], st)
        B.gns_aggregate(ctxs[i], bufs[i].array[last], x_in[i], F, h_out[i], st)

    def step_sync(b):
        """The same mini-batch on slot 0 with host-visible counts (used for the byte accounting)."""
        if b % refresh == 0:
            torch.cuda.synchronize()
            B.gns_sample_cache(ctx, sd["cache"], b // refresh, streams[0])
        B.gns_sample_blocks(ctx, sd["batch"] + b, seeds[b], blocks.array, streams[0])
        blk = blocks.array[last]
        B.gns_gather_features(ctx, blocks.tensors[last]["src_nodes"], blk.num_src, x_in[0], streams[0])
        B.gns_aggregate(ctx, blk, x_in[0], F, h_out[0], streams[0])

    torch.cuda.synchronize()
    for b in range(args.warmup):
        step(b)
    torch.cuda.synchronize()

    def run_range(lo, hi):
        """Steps lo..hi-1.  With --threads, each slot is driven by its own host thread (kernel
        launches are host-bound); the threads meet at every cache refresh."""
        if not args.threads or S == 1:
            for b in range(lo, hi):
                step(b)
            return
        import threading
        barrier = threading.Barrier(S)

        def worker(i):
            for b in range(lo, hi):
                if b % refresh == 0:
                    barrier.wait()
                    if i == 0:
                        torch.cuda.synchronize()
                        B.gns_sample_cache(ctx, sd["cache"], b // refresh, streams[0])
                    barrier.wait()
                if b % S != i:
                    continue
                st = streams[i]
                B.gns_sample_blocks_async(ctxs[i], sd["batch"] + b, seeds[b], bufs[i].array, st)
                B.gns_gather_features(ctxs[i], bufs[i].tensors[last]["src_nodes"], -1, x_in[i], st)
                B.gns_aggregate(ctxs[i], bufs[i].array[last], x_in[i], F, h_out[i], st)

        ths = [threading.Thread(target=worker, args=(i,)) for i in range(S)]
        for t in ths:
            t.start()
        for t in ths:
            t.join()

    # ---- timed region: on slot 0 the input-layer sampler is bracketed by HIP events
    dom_stage = B.GNS_STAGE_SAMPLE + last
    B.gns_profile_begin(ctx, 1 << dom_stage, args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_range(args.warmup, total)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_ms, dom_launches = B.gns_profile_collect(ctx, dom_stage)
    B.gns_profile_begin(ctx, 0, 0)
    elapsed = t1 - t0
    ms_per_step = 1e3 * elapsed / args.steps

    # ---- untimed replay of the same steps: algorithmic bytes of the dominant kernel, shape statistics
    off_bytes = 8 if g.indptr.dtype == torch.int64 else 4
    alg_bytes = 0.0
    alg_bytes_subgraph = 0.0
    stats = dict(rows=0, scanned_entries=0, edges=0, input_nodes=0, cached_input=0, eligible=0)
    stage_ms = {}
    if args.stages:
        mask = 0
        for i in range(L):
            mask |= (1 << (B.GNS_STAGE_SAMPLE + i)) | (1 << (B.GNS_STAGE_FINISH + i))
        mask |= (1 << B.GNS_STAGE_GATHER) | (1 << B.GNS_STAGE_AGGREGATE)
        B.gns_profile_begin(ctx, mask, args.steps * (2 * L + 2))
    for b in range(args.warmup, total):
        step_sync(b)
        torch.cuda.synchronize()
        blk = blocks.array[last]
        v = blocks.views(last)
        rows = blk.num_dst
        dst_nodes = v["src_nodes"][:rows].to(torch.int64)
        scanned = int(deg[dst_nodes].sum())
        elig = int(v["row_eligible"].sum())
        # CSR segments streamed + per-row dst id and two offsets + per-row count/eligible out
        # + 8 B per emitted edge (id + weight) + the membership bitmap once
        alg_bytes += scanned * 4 + rows * (4 + 2 * off_bytes + 8) + blk.num_edges * 8 + (n + 7) // 8
        alg_bytes_subgraph += elig * 4 + rows * (4 + 2 * off_bytes + 8) + blk.num_edges * 8
        stats["rows"] += rows
        stats["scanned_entries"] += scanned
        stats["edges"] += blk.num_edges
        stats["input_nodes"] += blk.num_src
        stats["cached_input"] += blk.num_src - rows
        stats["eligible"] += elig
    torch.cuda.synchronize()
    if args.stages:
        for i in range(L):
            for name, base in (("sample", B.GNS_STAGE_SAMPLE), ("finish", B.GNS_STAGE_FINISH)):
                ms, cnt = B.gns_profile_collect(ctx, base + i)
                stage_ms["%s_layer_index_%d" % (name, i)] = round(1e3 * ms / max(cnt, 1), 2)
        for name, st in (("gather", B.GNS_STAGE_GATHER), ("aggregate", B.GNS_STAGE_AGGREGATE)):
            ms, cnt = B.gns_profile_collect(ctx, st)
            stage_ms[name] = round(1e3 * ms / max(cnt, 1), 2)
        B.gns_profile_begin(ctx, 0, 0)

    for c_ in ctxs[1:]:
        B.gns_destroy(c_)
    achieved = (alg_bytes / args.steps) / (1e6 * dom_ms / max(dom_launches, 1))   # GB/s
    roofline = {
        "kernel": "k_sample_cache_only (input-layer sampler)",
        "bound": "hbm",
        "achieved": round(achieved, 2),
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 5),
        "traffic": None,
        "avg_launch_us": round(1e3 * dom_ms / max(dom_launches, 1), 2),
        "launches": dom_launches,
        "algorithmic_bytes_per_launch": int(alg_bytes / args.steps),
        "induced_subgraph_bytes_per_launch": int(alg_bytes_subgraph / args.steps),
    }

    # ---- CPU oracle on a bounded sample of the same batches
    cpu = None
    if args.cpu_batches > 0:
        import oracle
        ip = g.indptr.cpu().numpy()
        ix = g.indices.cpu().numpy()
        xf = feat.cpu().numpy()
        nb = min(args.cpu_batches, args.steps)
        ids = list(range(args.warmup, args.warmup + nb))
        seeds_cpu = {b: seeds[b].cpu().numpy() for b in ids}
        _, bitmap, _ = oracle.sample_cache(ip, sd["cache"], 0, cache_size)

        def cpu_batch(b):
            blks = oracle.sample_blocks(ip, ix, bitmap, cache_size, sd["batch"] + b, seeds_cpu[b], fanouts, policies)
            x = oracle.gather(xf, blks[-1].src_nodes)
            return oracle.aggregate(blks[-1].indptr, blks[-1].indices, blks[-1].weights, x).shape

        t = time.perf_counter()
        cpu_batch(ids[0])
        single = 1.0 / (time.perf_counter() - t)
        threads = max(1, min(16, os.cpu_count() or 1))
        t = time.perf_counter()
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(cpu_batch, ids))
        multi = nb / (time.perf_counter() - t)
        cpu = {"value": round(multi, 3), "unit": "mini-batches/s", "cores": threads, "kind": "oracle",
               "sample": "%d of the timed mini-batches (sample+gather+aggregate, cache draw excluded), one batch per "
                         "thread; single-thread rate %.3f mini-batches/s" % (nb, single)}

    out = {
        "metric": "sampled mini-batches/sec (fanout %s, batch %d) + gather/aggregate HBM GB/s"
                  % ("/".join(map(str, fanouts)), batch),
        "value": round(args.steps / elapsed, 2),
        "unit": "mini-batches/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "i32+f32",
        "data": "synthetic",
        "config": {"workload": "config %d: Chung-Lu graph n=%d nnz=%d gamma=%.1f, F=%d fp32 in HBM, cache %d nodes "
                               "redrawn every %d mini-batches, fanouts %s, batch %d"
                               % (cfg_id, n, g.nnz, c["gamma"], F, cache_size, refresh, fanouts, batch),
                   "max_degree": g.max_degree, "batches_in_flight": S,
                   "avg_per_batch": {k: round(v / args.steps, 1) for k, v in stats.items()}},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if stage_ms:
        out["stage_us"] = stage_ms
    B.gns_destroy(ctx)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
