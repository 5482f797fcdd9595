#!/usr/bin/env python3
"""Benchmark of the GNS hot path on one MI355X.

A step is one mini-batch through the whole path: (periodic cache draw) ->
gns_sample_blocks -> gns_gather_features (input nodes) -> gns_aggregate (input
layer).  Default workload: the medium power-law graph (1M nodes, ~20M undirected
edges, 128-dim fp32 features in HBM, 1% degree-proportional cache redrawn every
20 mini-batches, fan-outs 15/10/5, batch 1024), seeded and synthetic.

Two passes over the same K steps:
  A  the timed region of the contract: K steps spread over --slots contexts
     (one stream each, sharing the cache), no host synchronisation inside a
     step -> `value`, `ms_per_step`;
  B  the same K steps on one stream with every kernel stage bracketed by HIP
     events -> per-stage times and the `roofline` object of the kernel that
     takes the most time (one stream, so that its launch duration is the same
     quantity rocprofv3 --kernel-trace reports).
Then an untimed replay counts algorithmic bytes, and the CPU oracle is timed on
a bounded sample of the same mini-batches.  Prints one JSON line.
"""
import argparse
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def profile_traffic(kernel, cfg_id):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by the copy-kernel factors stated there), or None."""
    path = os.path.join(ROOT, "profiles", "pmc_config%d_hbm_traffic.txt" % cfg_id)
    if not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"\s*(\S+)\s+.*traffic_bytes_per_launch=(\d+)", line)
        if m and m.group(1) == kernel:
            return int(m.group(2))
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", type=int, default=2, help="workload id (see synth.CONFIGS)")
    ap.add_argument("--cpu-batches", type=int, default=32, help="mini-batches the CPU oracle is timed on (0: skip)")
    ap.add_argument("--slots", type=int, default=4,
                    help="mini-batches kept in flight in pass A (one context + stream each; they share the cache)")
    ap.add_argument("--flag-mode", type=int, default=1,
                    help="cache-membership flags of the CSR entries: 1 (default) once per cache draw, inside the timed "
                         "region like the draw itself; 0 per mini-batch, for the dst rows' CSR segments only")
    ap.add_argument("--upper-policy", choices=["uniform", "cache_first"], default="uniform",
                    help="policy of the layers above the input layer: uniform node-wise sampling (the workload the "
                         "metric is quoted on) or the paper's cache-first-then-fill (its Section 4.1 setting)")
    ap.add_argument("--cache-probability", choices=["degree", "walk"], default="degree",
                    help="degree: Eq. (1), the workload the metric is quoted on; walk: Section 3.2's random-walk "
                         "probability from the workload's training split (computed once, outside the timed region, "
                         "and reported on its own)")
    ap.add_argument("--dense-hidden", type=int, default=0,
                    help="if > 0 every step also runs the input layer's update step h = relu(W.(h_self, h_neigh)+b) "
                         "with this many output features (synthetic W; outside the metric's path, reported on its own)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference point for rocprofv3 byte counters)")
    ap.add_argument("--skip-pass-a", action="store_true", help="profiling aid: only the single-stream pass")
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
    last = L - 1
    upper = B.GNS_UNIFORM if args.upper_policy == "uniform" else B.GNS_CACHE_FIRST
    policies = [upper] * (L - 1) + [B.GNS_CACHE_ONLY]
    cache_size = int(n * c["cache_frac"])
    refresh = c.get("refresh_every", 20)
    K, W = args.steps, args.warmup
    total = W + K

    # ---- inputs: generated on the device, resident in HBM (or pinned host memory for the feature-heavy
    #      workloads) before any timing starts
    g = synth.make_config_graph(cfg_id, device=dev)
    on_host = bool(c.get("feat_on_host"))
    feat = synth.node_features(n, F, sd["feat"], device=dev, pin=on_host)
    seeds = [synth.uniform_seed_batch(n, batch, sd["batch"] + b, device=dev) for b in range(total)]
    off_bytes = 8 if g.indptr.dtype == torch.int64 else 4

    graph = B.make_graph(g.indptr, g.indices, feat_dev=None if on_host else feat,
                         feat_host_pinned=feat if on_host else None)
    walk = args.cache_probability == "walk"
    config = B.make_config(fanouts, policies, cache_size, batch, flag_mode=args.flag_mode,
                           cache_probability=B.GNS_PROB_WALK if walk else B.GNS_PROB_DEGREE)
    ws = B.alloc_workspace(graph, config, dev)
    ctx = B.gns_create(graph, config, ws)
    walk_info = None
    if walk:
        # the training split of the workload (a seeded 10 % of the nodes where the workload names none)
        split = synth.training_split(n, c.get("split", max(batch, n // 10)), sd["split"]).to(dev)
        scale = 24
        B.gns_cache_walk_probability(ctx, split, scale)                 # warm-up (also validates)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.gns_cache_walk_probability(ctx, split, scale)                 # synchronises before it returns
        dt = time.perf_counter() - t0
        _, _, total_mass, support = B.gns_cache_probability_view(ctx)
        # per step: every CSR entry (4 B) and the 8-B weight it points to, per node two offsets, one weight read
        # and one written; then the prefix scan reads the weights twice and writes the prefix
        step_bytes = g.nnz * (4 + 8) + n * (2 * off_bytes + 16)
        walk_bytes = L * step_bytes + n * 24
        walk_info = {"ms": round(1e3 * dt, 3), "steps": L, "training_nodes": int(split.numel()),
                     "nodes_reached": int(support), "scale_log2": scale,
                     "algorithmic_GBps": round(walk_bytes / dt / 1e9, 1)}
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

    H = args.dense_hidden
    if H > 0:
        gen = torch.Generator(device=dev).manual_seed(sd["feat"] + 17)
        w_dense = torch.randn((2 * F, H), device=dev, generator=gen) / (2 * F) ** 0.5
        b_dense = torch.randn(H, device=dev, generator=gen)
        z_out = [torch.empty((bufs[i].array[last].cap_dst, H), dtype=torch.float32, device=dev) for i in range(S)]

    def refresh_cache(b):
        # The draw fills the copy of the cache structures that is not in use: the batches the other slots have in
        # flight keep reading the old cache, the batches enqueued from here on read the new one.  It runs on slot
        # 0's stream (measured: a stream of its own makes it compete with slot 0's batch and costs 4 %).
        B.gns_sample_cache(ctx, sd["cache"], b // refresh, streams[0])

    def step(b, i):
        """One mini-batch enqueued on slot i's stream; counts stay on the device, nothing synchronises."""
        if b % refresh == 0:
            refresh_cache(b)
        st = streams[i]
        B.gns_sample_blocks_async(ctxs[i], sd["batch"] + b, seeds[b], bufs[i].array, st)
        B.gns_gather_features(ctxs[i], bufs[i].tensors[last]["src_nodes"], -1, x_in[i], st)
        B.gns_aggregate(ctxs[i], bufs[i].array[last], x_in[i], F, h_out[i], st)
        if H > 0:   # the dst nodes are the first rows of the gathered input features
            B.gns_sage_dense(ctxs[i], x_in[i], h_out[i], w_dense, b_dense, True, z_out[i], -1 - last, st)

    torch.cuda.synchronize()
    if args.calib_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)     # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for b in range(W):
        step(b, b % S)
    torch.cuda.synchronize()

    # ---- pass A: the timed region
    if args.skip_pass_a:
        elapsed = float("nan")
    else:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for b in range(W, total):
            step(b, b % S)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0

    # ---- pass B: one stream, every stage bracketed by HIP events on that stream
    stages = {"sample_layer_%d" % (L - i): B.GNS_STAGE_SAMPLE + i for i in range(L)}
    stages.update({"finish_layer_%d" % (L - i): B.GNS_STAGE_FINISH + i for i in range(L)})
    stages.update({"plan": B.GNS_STAGE_PLAN, "flag": B.GNS_STAGE_FLAG, "select": B.GNS_STAGE_SELECT,
                   "gather": B.GNS_STAGE_GATHER, "aggregate": B.GNS_STAGE_AGGREGATE, "dense": B.GNS_STAGE_DENSE})
    mask = 0
    for sid in stages.values():
        mask |= 1 << sid
    B.gns_profile_begin(ctx, mask, K * (2 * L + 7))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for b in range(W, total):
        step(b, 0)
    torch.cuda.synchronize()
    elapsed_b = time.perf_counter() - t0
    stage_us, stage_launches = {}, {}
    for name, sid in stages.items():
        ms, cnt = B.gns_profile_collect(ctx, sid)
        if cnt:
            stage_us[name] = round(1e3 * ms / cnt, 2)
            stage_launches[name] = cnt
    B.gns_profile_begin(ctx, 0, 0)

    # ---- untimed replay with host-visible counts: algorithmic bytes per launch, shape statistics
    start_all = g.indptr[:-1].to(torch.int64)
    end_all = g.indptr[1:].to(torch.int64)
    acc = dict(rows=0, scanned_entries=0, chunks=0, edges=0, input_nodes=0, cached_input=0, eligible=0, read_rows=0)
    blocks = bufs[0]
    for b in range(W, total):
        if b % refresh == 0:
            refresh_cache(b)
        B.gns_sample_blocks(ctx, sd["batch"] + b, seeds[b], blocks.array, streams[0])
        torch.cuda.synchronize()
        blk = blocks.array[last]
        v = blocks.views(last)
        rows = blk.num_dst
        dst_nodes = v["src_nodes"][:rows].to(torch.int64)
        st_, en_ = start_all[dst_nodes], end_all[dst_nodes]
        deg_ = en_ - st_
        acc["rows"] += rows
        acc["scanned_entries"] += int(deg_.sum())
        acc["chunks"] += int(torch.where(deg_ > 0, ((en_ - 1) >> 6) - (st_ >> 6) + 1, torch.zeros_like(deg_)).sum())
        acc["edges"] += blk.num_edges
        acc["input_nodes"] += blk.num_src
        acc["cached_input"] += blk.num_src - rows
        acc["eligible"] += int(v["row_eligible"].sum())
        acc["read_rows"] += int(torch.unique(v["indices"][:blk.num_edges]).numel())    # distinct source rows of the layer
    torch.cuda.synchronize()
    avg = {k: v / K for k, v in acc.items()}
    # algorithmic bytes per launch of each single-kernel stage (averages over the K steps)
    alg = {
        # CSR segments streamed once + the work list read + one flag word written per chunk + the bitmap once
        "flag": avg["scanned_entries"] * 4 + avg["chunks"] * (4 + 8) + (n + 7) // 8,
        # per row: dst id, its CSR extent, count + eligible out; the row's flag words; per edge: index read,
        # 1/p^C of the sampled node, id + weight written
        "select": avg["rows"] * (4 + 16 + 8) + avg["chunks"] * 8 + avg["edges"] * (4 + 4 + 8),
        "gather": avg["input_nodes"] * (F * 4 * 2 + 4),
        # every distinct source row read once, every dst row written once, offsets, and index + weight per edge
        "aggregate": avg["read_rows"] * F * 4 + avg["rows"] * (F * 4 + 4) + avg["edges"] * 8,
    }
    kernel_of = {"flag": "k_flag_chunks", "select": "k_select_rows", "gather": "k_gather", "aggregate": "k_aggregate"}
    candidates = [s_ for s_ in alg if s_ in stage_us]
    dom = max(candidates, key=lambda s_: stage_us[s_])
    achieved = alg[dom] / (1e3 * stage_us[dom])               # bytes / us / 1e3 = GB/s
    roofline = {
        "kernel": kernel_of[dom],
        "stage": dom,
        "bound": "hbm",
        "achieved": round(achieved, 2),
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 5),
        "traffic": profile_traffic(kernel_of[dom], cfg_id),
        "avg_launch_us": stage_us[dom],
        "launches": stage_launches[dom],
        "algorithmic_bytes_per_launch": int(alg[dom]),
        "timed_in": "pass B (same K steps, one stream, HIP events on that stream)",
        "other_kernels_GBps": {kernel_of[s_]: round(alg[s_] / (1e3 * stage_us[s_]), 1) for s_ in candidates if s_ != dom},
    }
    if dom == "aggregate":
        # its edge rows come from a few thousand distinct source rows that stay in L2: the HBM side is the
        # output stream, the kernel itself is bound by L2 reads
        roofline["note"] = ("%d edge rows of %d B are read from %d distinct L2-resident source rows: L2-read bound, "
                            "HBM sees the output rows" % (avg["edges"], F * 4, avg["read_rows"]))
    if dom == "flag":
        # what a layout that stores only the cached neighbors (Section 3.3's induced subgraph) would read
        roofline["induced_subgraph_bytes_per_launch"] = int(avg["eligible"] * 4 + avg["chunks"] * 8)

    # ---- CPU oracle on a bounded sample of the same mini-batches
    cpu = None
    if args.cpu_batches > 0:
        import oracle
        ip = g.indptr.cpu().numpy()
        ix = g.indices.cpu().numpy()
        xf = feat.numpy() if on_host else feat.cpu().numpy()
        nb = min(args.cpu_batches, K)
        ids = list(range(W, W + nb))
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

    for c_ in ctxs[1:]:
        B.gns_destroy(c_)
    B.gns_destroy(ctx)
    out = {
        "metric": "sampled mini-batches/sec (fanout %s, batch %d) + gather/aggregate HBM GB/s"
                  % ("/".join(map(str, fanouts)), batch),
        "value": round(K / elapsed, 2),
        "unit": "mini-batches/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(1e3 * elapsed / K, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "i32+f32",
        "data": "synthetic",
        "config": {"workload": "config %d: Chung-Lu graph n=%d nnz=%d gamma=%.1f, F=%d fp32 in %s, cache %d nodes "
                               "redrawn every %d mini-batches, fanouts %s, batch %d"
                               % (cfg_id, n, g.nnz, c["gamma"], F,
                                  "pinned host memory (cached rows in HBM)" if on_host else "HBM",
                                  cache_size, refresh, fanouts, batch),
                   "max_degree": g.max_degree, "batches_in_flight": S,
                   "cache_flags": "per mini-batch (CSR-segment scan)" if args.flag_mode == 0 else "per cache draw",
                   "upper_layers": args.upper_policy, "cache_probability": args.cache_probability,
                   "avg_per_batch": {k: round(v, 1) for k, v in avg.items()}},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "walk_probability": walk_info,
        "dense_update": None if H == 0 or "dense" not in stage_us else {
            "hidden": H, "avg_launch_us": stage_us["dense"], "bound": "mfma", "dtype": "f32",
            "achieved": round(2.0 * avg["rows"] * 2 * F * H / (stage_us["dense"] * 1e-6) / 1e12, 2),
            "peak": 157.3, "unit": "TFLOP/s",
            "frac": round(2.0 * avg["rows"] * 2 * F * H / (stage_us["dense"] * 1e-6) / 1e12 / 157.3, 4)},
        "single_stream": {"value": round(K / elapsed_b, 2), "ms_per_step": round(1e3 * elapsed_b / K, 4),
                          "stage_us": stage_us},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
