#!/usr/bin/env python3
"""Benchmark of the GNS hot path on one MI355X.

A step is one mini-batch through the whole path: (periodic cache draw) ->
gns_sample_blocks -> gns_gather_features (input nodes) -> gns_aggregate (input
layer).  Default workload: the medium power-law graph (1M nodes, ~20M undirected
edges, 128-dim fp32 features in HBM, 1% degree-proportional cache redrawn every
20 mini-batches, fan-outs 15/10/5, batch 1024), seeded and synthetic.

Mini-batches are independent given the cache, so the loop enqueues them in groups
(gns_*_group: every kernel serves --group mini-batches), the groups alternating
between --slots streams; counts stay on the device and nothing synchronises inside
the timed region except the cache draw's own read-back.

Passes over the same workload:
  A  the timed region of the contract: K steps, repeated --repeats times back to
     back (each window bracketed by a device synchronisation); `value` is K over
     the median window.  Warm-up runs at least --warmup steps and always a whole
     number of cache periods, so that every launch sequence has been captured and
     both copies of the cache structures have been drawn before the first window.
  C  the same windows without the aggregation: the sampler + gather pipeline alone
     (`roofline.sampler_gather`).
  B  K steps on one stream, kernels launched one by one with every stage
     bracketed by HIP events on that stream -> per-stage times and the `roofline`
     object of the single kernel that takes the most time.
Then an untimed replay counts algorithmic bytes, and the CPU oracle is timed on a
bounded sample of the same mini-batches.  The default run repeats passes A-C
(fewer steps, no oracle) on the products-shaped and the giant workload, on the
giant workload with its features in HBM, and on two variants of the headline
workload (upper layers sampled cache first as in the paper's runs; cache flags
found per mini-batch by a CSR-segment scan), all under `per_config`; it also counts
the input nodes of plain node-wise sampling against GNS (`input_nodes`).
Prints one JSON line.
"""
import argparse
import json
import os
import re
import statistics
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def progress(msg):
    """One line on stderr per phase when GNS_BENCH_PROGRESS is set (a long or stuck run then says where it is)."""
    if os.environ.get("GNS_BENCH_PROGRESS"):
        print("bench: " + msg, file=sys.stderr, flush=True)


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


def measured_copy_gbps(torch, dev):
    """Read + written bytes per second of a plain 1 GiB device copy (the ceiling this box gives a stream)."""
    src = torch.ones(256 * 1024 * 1024, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 5
    del src, dst
    torch.cuda.empty_cache()
    return 2 * (1 << 30) / (ms * 1e-3) / 1e9


class Workload:
    """One config: graph, features, contexts, buffers; the passes of the benchmark."""

    def __init__(self, torch, B, synth, cfg_id, args, total_batches, feat_in_hbm=False, upper_policy=None, refresh_every=None):
        self.torch, self.B, self.synth, self.args = torch, B, synth, args
        dev = self.dev = torch.device("cuda:0")
        c = self.c = synth.CONFIGS[cfg_id]
        sd = self.sd = synth.config_seeds(cfg_id)
        self.cfg_id = cfg_id
        self.n, self.F, self.batch = c["n"], c["feat"], c["batch"]
        self.fanouts = list(c["fanouts"])
        L = self.L = len(self.fanouts)
        self.last = L - 1
        self.upper_policy = upper_policy or args.upper_policy
        upper = B.GNS_UNIFORM if self.upper_policy == "uniform" else B.GNS_CACHE_FIRST
        self.policies = [upper] * (L - 1) + [B.GNS_CACHE_ONLY]
        self.cache_size = int(self.n * c["cache_frac"])
        self.refresh = refresh_every or c.get("refresh_every", 20)
        self.g = synth.make_config_graph(cfg_id, device=dev)
        self.on_host = bool(c.get("feat_on_host")) and not feat_in_hbm
        self.feat = synth.node_features(self.n, self.F, sd["feat"], device=dev, pin=self.on_host)
        self.seeds = [synth.uniform_seed_batch(self.n, self.batch, sd["batch"] + b, device=dev)
                      for b in range(total_batches)]
        self.graph = B.make_graph(self.g.indptr, self.g.indices, feat_dev=None if self.on_host else self.feat,
                                  feat_host_pinned=self.feat if self.on_host else None)
        self.walk = args.cache_probability == "walk"
        self.config = B.make_config(self.fanouts, self.policies, self.cache_size, self.batch, flag_mode=args.flag_mode,
                                    cache_probability=B.GNS_PROB_WALK if self.walk else B.GNS_PROB_DEGREE)
        self.ws = B.alloc_workspace(self.graph, self.config, dev)
        self.ctx = B.gns_create(self.graph, self.config, self.ws)
        # measured: groups of 5 on two streams are best when the features live in HBM; with the PCIe-bound gather
        # of a host feature store larger groups are
        group = args.group if args.group > 0 else (10 if self.on_host else 5)
        self.G = max(1, min(group, B.GNS_MAX_GROUP, self.refresh))
        self.S = max(1, args.slots)
        nctx = self.G * self.S
        self.ctxs, self.fork_ws = [self.ctx], []
        for _ in range(nctx - 1):
            w = torch.empty(B.gns_fork_workspace_bytes(self.ctx), dtype=torch.uint8, device=dev)
            self.fork_ws.append(w)
            self.ctxs.append(B.gns_fork(self.ctx, w))
        self.streams = [torch.cuda.Stream() for _ in range(self.S)]
        self.bufs = [B.BlockBuffers(self.graph, self.config, dev) for _ in range(nctx)]
        last = self.last
        self.x_in = [torch.empty((self.bufs[i].array[last].cap_src, self.F), dtype=torch.float32, device=dev)
                     for i in range(nctx)]
        self.h_out = [torch.empty((self.bufs[i].array[last].cap_dst, self.F), dtype=torch.float32, device=dev)
                      for i in range(nctx)]
        self.src_nodes = [self.bufs[i].tensors[last]["src_nodes"] for i in range(nctx)]
        self.calls = {}
        self.H = args.dense_hidden
        if self.H > 0:
            gen = torch.Generator(device=dev).manual_seed(sd["feat"] + 17)
            self.w_dense = torch.randn((2 * self.F, self.H), device=dev, generator=gen) / (2 * self.F) ** 0.5
            self.b_dense = torch.randn(self.H, device=dev, generator=gen)
            self.z_out = [torch.empty((self.bufs[i].array[last].cap_dst, self.H), dtype=torch.float32, device=dev)
                          for i in range(nctx)]
        self.walk_info = None
        self.draw_stream = torch.cuda.Stream()
        self.pending_epoch = None          # cache period whose draw has been enqueued ahead of time
        self.draw_ms = None                # the first (synchronous) draw, host clock
        # A long draw (a flag pass over billions of CSR entries) keeps the L2 request queues full and slows the
        # mini-batches it overlaps by more than it saves (measured: -24 % on the 111 M-node graph, +6 % on the 1 M- and
        # 2.4 M-node graphs): by default the cache is drawn ahead of time only on graphs of under 2^29 entries.
        self.async_draw = args.async_refresh > 0 or (args.async_refresh < 0 and self.g.nnz < (1 << 29))

    def close(self):
        for c_ in self.ctxs[1:]:
            self.B.gns_destroy(c_)
        self.B.gns_destroy(self.ctx)

    # ---- the loop ---------------------------------------------------------------------------------------------
    def call(self, slot, size):
        key = (slot, size)
        if key not in self.calls:
            lo = slot * self.G
            self.calls[key] = self.B.GroupCall(self.ctxs[lo:lo + size], [b.array for b in self.bufs[lo:lo + size]])
        return self.calls[key]

    def groups(self, b0, b1):
        """Mini-batches b0..b1-1 as (slot, [ids]) groups of at most G that do not straddle a cache refresh;
        the slot follows from the group's position in its cache period, so every window reuses the same
        (slot, size) launch sequences."""
        out = []
        b = b0
        while b < b1:
            period_end = (b // self.refresh + 1) * self.refresh
            e = min(b + self.G, period_end, b1)
            out.append((((b % self.refresh) // self.G) % self.S, list(range(b, e))))
            b = e
        return out

    def refresh_cache(self, b):
        # The draw fills the copy of the cache structures that is not in use: the batches in flight keep reading
        # the old cache, the batches enqueued from here on read the new one.
        epoch = b // self.refresh
        if self.pending_epoch == epoch:
            self.B.gns_activate_cache(self.ctx)           # drawn ahead of time on the draw stream: switch over
        else:
            t0 = time.perf_counter()
            self.B.gns_sample_cache(self.ctx, self.sd["cache"], epoch, self.streams[0])     # returns when the draw is done
            if self.draw_ms is None and b == 0:
                self.torch.cuda.synchronize()
                self.draw_ms = 1e3 * (time.perf_counter() - t0)
        self.pending_epoch = None

    def prepare_next_cache(self, b):
        # Half a period ahead, on a stream of its own and without any host synchronisation: the next period's
        # cache only depends on (seed, epoch), so its draw overlaps the current period's mini-batches.
        if self.async_draw and self.pending_epoch is None:
            self.B.gns_sample_cache_async(self.ctx, self.sd["cache"], b // self.refresh + 1, self.draw_stream)
            self.pending_epoch = b // self.refresh + 1

    def run(self, b0, b1, aggregate=True, one_stream=False):
        B, last, F = self.B, self.last, self.F
        groups = self.groups(b0, b1)
        i = 0
        while i < len(groups):
            # The groups that are in flight together (one per stream) are enqueued side by side: first the sampling
            # sequence of each, then the feature kernels of each, so that no stream waits for the host to finish
            # with another one's calls.  A group that starts a cache period starts such a set.
            n = 1
            while (not one_stream and n < self.S and i + n < len(groups)
                   and groups[i + n][1][0] % self.refresh != 0):
                n += 1
            chunk = groups[i:i + n]
            i += n
            work = []
            for slot, ids in chunk:
                if ids[0] % self.refresh == 0:
                    self.refresh_cache(ids[0])
                elif not one_stream and ids[0] % self.refresh >= self.refresh // 2:
                    self.prepare_next_cache(ids[0])
                if one_stream:
                    slot = 0
                st = self.streams[slot]
                call = self.call(slot, len(ids))
                call.sample([self.sd["batch"] + b for b in ids], [self.seeds[b] for b in ids], st)
                work.append((slot, ids, st, call))
            for slot, ids, st, call in work:
                lo = slot * self.G
                hi = lo + len(ids)
                call.gather(self.src_nodes[lo:hi], [-1] * len(ids), self.x_in[lo:hi], st)
                if aggregate:
                    call.aggregate(last, self.x_in[lo:hi], F, self.h_out[lo:hi], st)
                    if self.H > 0:   # the dst nodes are the first rows of the gathered input features
                        for k_ in range(lo, hi):
                            B.gns_sage_dense(self.ctxs[k_], self.x_in[k_], self.h_out[k_], self.w_dense, self.b_dense, True,
                                             self.z_out[k_], -1 - last, st)

    def windows(self, b0, K, repeats, aggregate=True):
        """`repeats` windows of K steps back to back; seconds per window (host clock between device
        synchronisations) and, from HIP events on the streams, the device-side span of each window."""
        torch = self.torch
        host, devs = [], []
        for r in range(repeats):
            torch.cuda.synchronize()
            start = torch.cuda.Event(enable_timing=True)
            ends = [torch.cuda.Event(enable_timing=True) for _ in self.streams]
            start.record(self.streams[0])
            t0 = time.perf_counter()
            self.run(b0 + r * K, b0 + (r + 1) * K, aggregate=aggregate)
            for e, s in zip(ends, self.streams):
                e.record(s)
            torch.cuda.synchronize()
            host.append(time.perf_counter() - t0)
            devs.append(max(start.elapsed_time(e) for e in ends) * 1e-3)
        return host, devs

    def walk_probability(self):
        torch, B = self.torch, self.B
        split = self.synth.training_split(self.n, self.c.get("split", max(self.batch, self.n // 10)),
                                          self.sd["split"]).to(self.dev)
        scale = 24
        B.gns_cache_walk_probability(self.ctx, split, scale)                 # warm-up (also validates)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.gns_cache_walk_probability(self.ctx, split, scale)                 # synchronises before it returns
        dt = time.perf_counter() - t0
        _, _, total_mass, support = B.gns_cache_probability_view(self.ctx)
        off_bytes = 8 if self.g.indptr.dtype == torch.int64 else 4
        step_bytes = self.g.nnz * (4 + 8) + self.n * (2 * off_bytes + 16)
        walk_bytes = self.L * step_bytes + self.n * 24
        self.walk_info = {"ms": round(1e3 * dt, 3), "steps": self.L, "training_nodes": int(split.numel()),
                          "nodes_reached": int(support), "scale_log2": scale,
                          "algorithmic_GBps": round(walk_bytes / dt / 1e9, 1)}

    # ---- per-stage times: one stream, kernels launched one by one, HIP events around every stage --------------
    def stage_times(self, b0, K):
        B, L, torch = self.B, self.L, self.torch
        stages = {"sample_layer_%d" % (L - i): B.GNS_STAGE_SAMPLE + i for i in range(L)}
        stages.update({"finish_layer_%d" % (L - i): B.GNS_STAGE_FINISH + i for i in range(L)})
        stages.update({"plan": B.GNS_STAGE_PLAN, "flag": B.GNS_STAGE_FLAG, "select": B.GNS_STAGE_SELECT,
                       "gather": B.GNS_STAGE_GATHER, "aggregate": B.GNS_STAGE_AGGREGATE, "dense": B.GNS_STAGE_DENSE})
        mask = 0
        for sid in stages.values():
            mask |= 1 << sid
        B.gns_profile_begin(self.ctx, mask, (K + self.G) * (2 * L + 7))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.run(b0, b0 + K, one_stream=True)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        launch_us, launches = {}, {}
        for name, sid in stages.items():
            ms, cnt = B.gns_profile_collect(self.ctx, sid)
            if cnt:
                launch_us[name] = 1e3 * ms / cnt
                launches[name] = cnt
        B.gns_profile_begin(self.ctx, 0, 0)
        groups = self.groups(b0, b0 + K)
        per_launch = K / len(groups)                  # mini-batches one launch serves, on average
        return launch_us, launches, per_launch, elapsed

    # ---- untimed replay with host-visible counts: algorithmic bytes per mini-batch, shape statistics ----------
    def shape_stats(self, b0, count):
        torch, B, g, last = self.torch, self.B, self.g, self.last
        start_all = g.indptr[:-1].to(torch.int64)
        end_all = g.indptr[1:].to(torch.int64)
        acc = dict(rows=0, scanned_entries=0, chunks=0, edges=0, input_nodes=0, cached_input=0, eligible=0,
                   read_rows=0, upper_rows=0, upper_edges=0, all_rows=0, all_edges=0, new_nodes=0, host_rows=0)
        blocks = self.bufs[0]
        for b in range(b0, b0 + count):
            if b % self.refresh == 0 or b == b0:
                self.B.gns_sample_cache(self.ctx, self.sd["cache"], b // self.refresh, self.streams[0])
                nodes_ptr, csize, _, _ = B.gns_cache_view(self.ctx)
                cache_nodes = B.device_view_i32(nodes_ptr, csize, self.dev).to(torch.int64)
                is_cached = torch.zeros(self.n, dtype=torch.bool, device=self.dev)
                is_cached[cache_nodes] = True
            B.gns_sample_blocks(self.ctx, self.sd["batch"] + b, self.seeds[b], blocks.array, self.streams[0])
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
            acc["cached_input"] += int(is_cached[v["src_nodes"].to(torch.int64)].sum())
            acc["host_rows"] += blk.num_src - int(is_cached[v["src_nodes"].to(torch.int64)].sum())
            acc["eligible"] += int(v["row_eligible"].sum())
            acc["read_rows"] += int(torch.unique(v["indices"][:blk.num_edges]).numel())    # distinct source rows of the layer
            for i in range(self.L):
                bi = blocks.array[i]
                acc["all_rows"] += bi.num_dst
                acc["all_edges"] += bi.num_edges
                acc["new_nodes"] += bi.num_src - bi.num_dst
                if i < last:
                    acc["upper_rows"] += bi.num_dst
                    acc["upper_edges"] += bi.num_edges
        torch.cuda.synchronize()
        return {k: v / count for k, v in acc.items()}


    # ---- input nodes per mini-batch of plain node-wise sampling against GNS (the comparison of the paper's Table 3) ----
    def input_node_shapes(self, b0, count):
        torch, B = self.torch, self.B
        U, CF, C = B.GNS_UNIFORM, B.GNS_CACHE_FIRST, B.GNS_CACHE_ONLY
        settings = {"ns_all_layers_uniform": [U] * self.L,
                    "gns_upper_layers_uniform": [U] * (self.L - 1) + [C],
                    "gns_upper_layers_cache_first": [CF] * (self.L - 1) + [C]}
        out = {}
        B.gns_sample_cache(self.ctx, self.sd["cache"], b0 // self.refresh)
        nodes_ptr, csize, _, _ = B.gns_cache_view(self.ctx)
        is_cached = torch.zeros(self.n, dtype=torch.bool, device=self.dev)
        is_cached[B.device_view_i32(nodes_ptr, csize, self.dev).to(torch.int64)] = True
        for name, pol in settings.items():
            cfg = B.make_config(self.fanouts, pol, self.cache_size, self.batch, flag_mode=self.args.flag_mode)
            ws = B.alloc_workspace(self.graph, cfg, self.dev)
            ctx = B.gns_create(self.graph, cfg, ws)
            bufs = B.BlockBuffers(self.graph, cfg, self.dev)
            if any(p != U for p in pol):
                B.gns_sample_cache(ctx, self.sd["cache"], b0 // self.refresh)       # the same cache: (seed, epoch) fix it
            total = cached = 0
            for b in range(b0, b0 + count):
                B.gns_sample_blocks(ctx, self.sd["batch"] + b, self.seeds[b], bufs.array)
                total += bufs.array[self.last].num_src
                cached += int(is_cached[bufs.views(self.last)["src_nodes"].to(torch.int64)].sum())
            out[name] = {"input_nodes": round(total / count, 1), "of_them_cached": round(cached / count, 1)}
            B.gns_destroy(ctx)
            del ws, bufs
        ns = out["ns_all_layers_uniform"]["input_nodes"]
        out["ns_over_gns"] = {k_: round(ns / v["input_nodes"], 2) for k_, v in out.items() if k_.startswith("gns_")}
        out["note"] = ("averages over %d mini-batches with one cache; the paper's Table 3 reports the same comparison on "
                       "its datasets (its GNS also samples the upper layers cache first)" % count)
        return out


def algorithmic_bytes(w, avg, flag_mode):
    """Bytes each stage has to move per mini-batch (averages over the replayed batches)."""
    n, F, C = w.n, w.F, w.cache_size
    nnz = w.g.nnz
    off_bytes = 8 if w.g.indptr.dtype == w.torch.int64 else 4
    alg = {
        # CSR segments streamed once + the work list read + one flag word written per chunk + the bitmap once
        "flag": avg["scanned_entries"] * 4 + avg["chunks"] * (4 + 8) + (n + 7) // 8,
        # per row: dst id, its CSR extent, count + eligible out; the row's flag words; per edge: index read,
        # 1/p^C of the sampled node, id + weight written
        "select": avg["rows"] * (4 + 16 + 8) + avg["chunks"] * 8 + avg["edges"] * (4 + 4 + 8),
        # uniform layers: per row dst id, extent, count + eligible; per edge one index read, id + weight written
        "uniform": avg["upper_rows"] * (4 + 16 + 8) + avg["upper_edges"] * (4 + 8),
        # union + relabel, all layers: per row dst copy + offset; per edge scratch read (8), local id + weight
        # written (8), one hash probe (8); per new node id written, extent (2 offsets read, 16 written), hash slot (8)
        "frontier": avg["all_rows"] * 8 + avg["all_edges"] * 24 + avg["new_nodes"] * (4 + 2 * off_bytes + 16 + 8),
        "gather": avg["input_nodes"] * (F * 4 * 2 + 4),
        # every distinct source row read once, every dst row written once, offsets, and index + weight per edge
        "aggregate": avg["read_rows"] * F * 4 + avg["rows"] * (F * 4 + 4) + avg["edges"] * 8,
    }
    # one cache draw: the stream's draws (8 B each, about 1.1 |C|), bitmap + prefix + list, the cached rows copied
    # into the table, and with flags per cache draw one pass over the CSR (entries read, one bit each written)
    draw = 1.1 * C * (8 + 2 * off_bytes * 20) + n / 8 * 3 + C * (4 + 4 + 2 * off_bytes) + C * F * 4 * 2
    if flag_mode == 1:
        draw += nnz * 4 + nnz / 8
    alg["cache_draw"] = draw
    return alg


def bench_config(torch, B, synth, cfg_id, args, K, W, repeats, with_oracle, feat_in_hbm=False, upper_policy=None,
                 refresh_every=None):
    c = synth.CONFIGS[cfg_id]
    refresh = refresh_every or c.get("refresh_every", 20)
    warm = max(W, refresh)
    warm = (warm + refresh - 1) // refresh * refresh          # whole cache periods: the windows start at a refresh
    if warm // refresh < 2:
        warm = 2 * refresh                                     # both copies of the cache structures get drawn
    total = warm + (2 * repeats + 1) * K
    t_setup = time.perf_counter()
    progress("config %d: building graph, features and contexts" % cfg_id)
    w = Workload(torch, B, synth, cfg_id, args, total, feat_in_hbm=feat_in_hbm, upper_policy=upper_policy,
                 refresh_every=refresh_every)
    if w.walk:
        w.walk_probability()
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup
    if args.calib_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=w.dev)     # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # warm-up: whole cache periods, and one window's worth of the exact group pattern the windows use
    progress("config %d: set up in %.1f s, warm-up of %d steps" % (cfg_id, setup_s, warm))
    w.run(0, warm)
    torch.cuda.synchronize()
    b0 = warm
    progress("pass A")
    # ---- pass A
    if args.skip_pass_a:
        host, devs = [float("nan")], [float("nan")]
    else:
        host, devs = w.windows(b0, K, repeats)
    elapsed = statistics.median(host)
    b1 = b0 + repeats * K
    progress("pass C")
    # ---- pass C: sampler + gather only
    host_c, devs_c = ([float("nan")], [float("nan")]) if args.skip_pass_a else w.windows(b1, K, repeats, aggregate=False)
    elapsed_c = statistics.median(host_c)
    b2 = b1 + repeats * K
    progress("cache draws alone")
    # ---- refresh alone (host clock around the synchronising call, the streams idle)
    refresh_ms = []
    for r in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        w.refresh_cache((b2 // refresh + r) * refresh)
        torch.cuda.synchronize()
        refresh_ms.append(1e3 * (time.perf_counter() - t0))
    progress("pass B")
    # ---- pass B
    launch_us, launches, per_launch, elapsed_b = w.stage_times(b2, K)
    progress("replay for byte counts")
    # ---- shapes and algorithmic bytes
    avg = w.shape_stats(b2, min(K, args.shape_batches))
    alg = algorithmic_bytes(w, avg, args.flag_mode)
    F = w.F
    # the input layer's CACHE_ONLY sampler: one row per lane on the induced subgraph when there is one, else flag words
    select_kernel = "k_sample_lane" if (args.flag_mode == 1 and w.fanouts[-1] <= 16) else "k_select_rows"
    kernel_of = {"flag": "k_flag_chunks", "select": select_kernel, "gather": "k_gather", "aggregate": "k_aggregate"}
    candidates = [s_ for s_ in kernel_of if s_ in launch_us]
    dom = max(candidates, key=lambda s_: launch_us[s_])
    bytes_per_launch = alg[dom] * per_launch
    achieved = bytes_per_launch / (1e3 * launch_us[dom])               # bytes / us / 1e3 = GB/s
    traffic = profile_traffic(kernel_of[dom], cfg_id)
    roofline = {
        "kernel": kernel_of[dom],
        "stage": dom,
        "bound": "hbm",
        "achieved": round(achieved, 2),
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 5),
        "traffic": traffic,
        "avg_launch_us": round(launch_us[dom], 2),
        "launches": launches[dom],
        "mini_batches_per_launch": round(per_launch, 3),
        "algorithmic_bytes_per_launch": int(bytes_per_launch),
        "timed_in": "pass B (K steps, one stream, kernels launched one by one, HIP events on that stream)",
        "other_kernels_GBps": {kernel_of[s_]: round(alg[s_] * per_launch / (1e3 * launch_us[s_]), 1)
                               for s_ in candidates if s_ != dom},
    }
    # the union + relabel stage (several small kernels per layer): bytes it has to move over the time of its launches
    fr_us = sum(v for k_, v in launch_us.items() if k_.startswith("finish_layer_"))
    # the relabel of every layer but the last rides in the next layer's sampler launch, so this is a lower bound on time
    roofline["frontier"] = {"stage": "union + relabel (a4), all layers", "bytes_per_mini_batch": int(alg["frontier"]),
                            "us_per_mini_batch": round(fr_us / per_launch, 2),
                            "achieved": round(alg["frontier"] * per_launch / (1e3 * fr_us), 1) if fr_us else None,
                            "frac": round(alg["frontier"] * per_launch / (1e3 * fr_us) / HBM_PEAK_GBS, 5) if fr_us else None,
                            "unit": "GB/s"}
    # sampler + gather together: cache draw (amortised over its period), all sampler layers, union + relabel, gather
    sg_bytes = alg["uniform"] + alg["select"] + alg["frontier"] + alg["gather"] + alg["cache_draw"] / w.refresh
    if args.flag_mode == 0:
        sg_bytes += alg["flag"]
    sg_us_b = sum(v for k_, v in launch_us.items() if k_.startswith(("sample_layer_", "finish_layer_")) or k_ == "gather")
    roofline["sampler_gather"] = {
        "bytes_per_mini_batch": int(sg_bytes),
        "achieved": round(sg_bytes * K / elapsed_c / 1e9, 1),
        "frac": round(sg_bytes * K / elapsed_c / 1e9 / HBM_PEAK_GBS, 5),
        "unit": "GB/s",
        "ms_per_step": round(1e3 * elapsed_c / K, 4),
        "timed_in": "pass C (the timed loop without the aggregation, median of %d windows of %d steps)" % (repeats, K),
        "one_stream_us_per_mini_batch": round(sg_us_b / per_launch + 1e3 * statistics.median(refresh_ms) / w.refresh, 2),
        "one_stream_frac": round(sg_bytes / (1e3 * (sg_us_b / per_launch + 1e3 * statistics.median(refresh_ms) / w.refresh))
                                 / HBM_PEAK_GBS, 5),
    }
    if dom == "aggregate":
        roofline["note"] = ("%d edge rows of %d B are read from %d distinct L2-resident source rows per mini-batch: "
                            "L2-read bound, HBM sees the output rows" % (avg["edges"], F * 4, avg["read_rows"]))
    if "flag" in launch_us:
        # what a layout that stores only the cached neighbors (Section 3.3's induced subgraph) would read
        roofline["induced_subgraph_bytes_per_mini_batch"] = int(avg["eligible"] * 4 + avg["chunks"] * 8)
    pcie = None
    if w.on_host and "gather" in launch_us:
        # rows that are not in the cache table come from pinned host memory over PCIe; the gather's time is theirs
        pcie = {"host_rows_per_mini_batch": round(avg["host_rows"], 1),
                "GBps": round(avg["host_rows"] * F * 4 * per_launch / (1e3 * launch_us["gather"]), 2),
                "note": "miss path of the gather (pinned host rows over PCIe), never part of an HBM figure; a cache "
                        "draw also uploads %d cached rows (%.0f MB)" % (w.cache_size, w.cache_size * F * 4 / 1e6)}

    res = {
        "value": round(K / elapsed, 2),
        "ms_per_step": round(1e3 * elapsed / K, 4),
        "windows_ms": [round(1e3 * h, 3) for h in host],
        "device_windows_ms": [round(1e3 * d, 3) for d in devs],
        "roofline": roofline,
        "pcie": pcie,
        "cache_refresh_ms": round(statistics.median(refresh_ms), 3),
        "stage_us_per_mini_batch": {k_: round(v / per_launch, 2) for k_, v in launch_us.items()},
        "one_stream": {"value": round(K / elapsed_b, 2), "ms_per_step": round(1e3 * elapsed_b / K, 4)},
        "avg_per_batch": {k_: round(v, 1) for k_, v in avg.items()},
        "workload": "config %d: Chung-Lu graph n=%d nnz=%d gamma=%.1f, F=%d fp32 in %s, cache %d nodes redrawn every %d "
                    "mini-batches, fanouts %s, batch %d"
                    % (cfg_id, w.n, w.g.nnz, c["gamma"], F,
                       "pinned host memory (cached rows in HBM)" if w.on_host else "HBM",
                       w.cache_size, w.refresh, w.fanouts, w.batch),
        "max_degree": w.g.max_degree,
        "group": w.G, "slots": w.S, "warmup_steps_run": warm, "setup_s": round(setup_s, 1),
        "cache_draw_ahead_of_time": bool(w.async_draw), "first_cache_draw_ms": round(w.draw_ms or 0.0, 3),
        "walk_probability": w.walk_info,
    }
    if args.input_node_batches > 0 and not w.walk and not feat_in_hbm and upper_policy is None:
        res["input_nodes"] = w.input_node_shapes(b2, min(K, args.input_node_batches))
    if w.H > 0 and "dense" in launch_us:
        fl = 2.0 * avg["rows"] * 2 * F * w.H
        res["dense_update"] = {"hidden": w.H, "avg_launch_us": round(launch_us["dense"], 2), "bound": "mfma", "dtype": "f32",
                               "achieved": round(fl / (launch_us["dense"] * 1e-6) / 1e12, 2), "peak": 157.3,
                               "unit": "TFLOP/s", "frac": round(fl / (launch_us["dense"] * 1e-6) / 1e12 / 157.3, 4)}

    progress("stages done")
    # ---- CPU oracle on a bounded sample of the same mini-batches
    if with_oracle and args.cpu_batches > 0:
        import oracle
        g = w.g
        ip = g.indptr.cpu().numpy()
        ix = g.indices.cpu().numpy()
        xf = w.feat.numpy() if w.on_host else w.feat.cpu().numpy()
        nproc = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
        share = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
        threads = max(1, min(nproc, share) if share > 0 else nproc)
        nb = min(max(args.cpu_batches, 2 * threads), K)
        ids = list(range(b0, b0 + nb))
        seeds_cpu = {b: w.seeds[b].cpu().numpy() for b in ids}
        _, bitmap, _ = oracle.sample_cache(ip, w.sd["cache"], b0 // w.refresh, w.cache_size)

        def cpu_batch(b):
            blks = oracle.sample_blocks(ip, ix, bitmap, w.cache_size, w.sd["batch"] + b, seeds_cpu[b], w.fanouts, w.policies)
            x = oracle.gather(xf, blks[-1].src_nodes)
            return oracle.aggregate(blks[-1].indptr, blks[-1].indices, blks[-1].weights, x).shape

        t = time.perf_counter()
        cpu_batch(ids[0])
        single = 1.0 / (time.perf_counter() - t)
        t = time.perf_counter()
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(cpu_batch, ids))
        multi = nb / (time.perf_counter() - t)
        res["cpu_baseline"] = {
            "value": round(multi, 3), "unit": "mini-batches/s", "cores": threads, "kind": "oracle",
            "sample": "%d of the timed mini-batches (sample + gather + aggregate, cache draw excluded), one batch per "
                      "thread on all %d host cores this process may use (nproc %d, CPU share of the box %s); "
                      "single-thread rate %.3f mini-batches/s" % (nb, threads, nproc, share or "not set", single)}
    w.close()
    del w
    import gc
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--repeats", type=int, default=5, help="timed windows of --steps steps each; the median counts")
    ap.add_argument("--config", type=int, default=2, help="workload id (see synth.CONFIGS)")
    ap.add_argument("--per-config", type=str, default="3,5",
                    help="workloads measured besides --config with fewer steps and no oracle ('' for none)")
    ap.add_argument("--per-config-steps", type=int, default=100)
    ap.add_argument("--hbm-variant", type=int, default=1,
                    help="1: the giant workload is also measured with its features resident in HBM (they fit a 288 GB "
                         "GPU), reported as a variant next to the configured pinned-host store")
    ap.add_argument("--cpu-batches", type=int, default=32, help="mini-batches the CPU oracle is timed on (0: skip)")
    ap.add_argument("--shape-batches", type=int, default=40, help="mini-batches replayed for the byte counts")
    ap.add_argument("--paper-upper-layers", type=int, default=1,
                    help="1: also measure --config with the upper layers sampled cache first (reported under per_config)")
    ap.add_argument("--epoch-period", type=int, default=1,
                    help="1: also measure the giant workload (features in HBM) with one cache draw per epoch")
    ap.add_argument("--scan-variant", type=int, default=1,
                    help="1: also measure --config with GNS_FLAGS_PER_BATCH (reported under per_config)")
    ap.add_argument("--input-node-batches", type=int, default=5,
                    help="mini-batches for the input-node comparison of plain node-wise sampling and GNS (0: skip)")
    ap.add_argument("--group", type=int, default=0,
                    help="mini-batches per launch sequence (gns_*_group); 0: 5, or 10 with a host feature store")
    ap.add_argument("--slots", type=int, default=2, help="groups kept in flight (one stream each; they share the cache)")
    ap.add_argument("--async-refresh", type=int, default=-1,
                    help="1: the next period's cache is drawn half a period ahead on its own stream "
                         "(gns_sample_cache_async / gns_activate_cache); 0: a synchronous draw at every period start; "
                         "-1: ahead of time on graphs of under 2^29 CSR entries")
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
    K, W = args.steps, args.warmup
    progress("start")
    copy_gbps = measured_copy_gbps(torch, dev)
    progress("copy rate measured")
    main_res = bench_config(torch, B, synth, args.config, args, K, W, args.repeats, with_oracle=True)
    per_config = {}
    for tok in [t for t in args.per_config.split(",") if t.strip()]:
        cid = int(tok)
        if cid == args.config:
            continue
        r = bench_config(torch, B, synth, cid, args, args.per_config_steps, 0, 3, with_oracle=False)
        per_config["config_%d" % cid] = r
        if synth.CONFIGS[cid].get("feat_on_host") and args.hbm_variant and cid == 5:
            r2 = bench_config(torch, B, synth, cid, args, args.per_config_steps, 0, 3, with_oracle=False, feat_in_hbm=True)
            r2["variant"] = "the same graph and batches with the full feature matrix resident in HBM instead of pinned host memory"
            per_config["config_%d_features_in_hbm" % cid] = r2
            if args.epoch_period and "split" in synth.CONFIGS[cid]:
                # the paper redraws the cache every P >= 1 epochs (Section 4.3), not every 100 mini-batches: the same
                # variant with one draw per epoch over the training split, timed over whole periods
                period = synth.CONFIGS[cid]["split"] // synth.CONFIGS[cid]["batch"]
                r5 = bench_config(torch, B, synth, cid, args, period, 0, 3, with_oracle=False, feat_in_hbm=True,
                                  refresh_every=period)
                r5["variant"] = ("features in HBM and the cache redrawn once per epoch over the training split (%d mini-batches), "
                                 "the paper's update period, instead of every %d" % (period, synth.CONFIGS[cid].get("refresh_every", 20)))
                per_config["config_%d_features_in_hbm_cache_per_epoch" % cid] = r5

    if args.paper_upper_layers and args.upper_policy == "uniform":
        # the same workload with the upper layers sampled cache first, as the paper's own runs do (Section 4.1)
        r3 = bench_config(torch, B, synth, args.config, args, args.per_config_steps, 0, 3, with_oracle=False,
                          upper_policy="cache_first")
        r3["variant"] = "the headline workload with the upper layers sampled cache first (the paper's setting) instead of uniformly"
        per_config["config_%d_upper_layers_cache_first" % args.config] = r3

    if args.scan_variant and args.flag_mode == 1:
        # the same workload with the cache membership of the input layer's rows found per mini-batch, by scanning their
        # CSR segments against the cache bitmap, instead of once per cache draw
        args0 = argparse.Namespace(**{**vars(args), "flag_mode": 0})
        r4 = bench_config(torch, B, synth, args.config, args0, args.per_config_steps, 0, 3, with_oracle=False)
        r4["variant"] = "the headline workload with the CSR-segment scan per mini-batch (GNS_FLAGS_PER_BATCH) instead of flags per cache draw"
        per_config["config_%d_flags_per_batch" % args.config] = r4

    c = synth.CONFIGS[args.config]
    roofline = main_res.pop("roofline")
    roofline["measured_copy_GBps"] = round(copy_gbps, 1)
    out = {
        "metric": "sampled mini-batches/sec (fanout %s, batch %d) + gather/aggregate HBM GB/s"
                  % ("/".join(map(str, c["fanouts"])), c["batch"]),
        "value": main_res["value"],
        "unit": "mini-batches/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "i32+f32",
        "data": "synthetic",
        "config": {"workload": main_res.pop("workload"), "max_degree": main_res.pop("max_degree"),
                   "mini_batches_per_launch": main_res["group"], "groups_in_flight": main_res["slots"],
                   "cache_draw_ahead_of_time": main_res["cache_draw_ahead_of_time"],
                   "cache_flags": "per mini-batch (CSR-segment scan)" if args.flag_mode == 0 else "per cache draw",
                   "upper_layers": args.upper_policy, "cache_probability": args.cache_probability,
                   "timing": "median of %d windows of %d steps, host clock between device synchronisations"
                             % (args.repeats, K),
                   "warmup_steps_run": main_res["warmup_steps_run"],
                   "avg_per_batch": main_res.pop("avg_per_batch")},
        "roofline": roofline,
        "cpu_baseline": main_res.pop("cpu_baseline", None),
        "pcie": main_res.pop("pcie"),
        "measured_copy_GBps": round(copy_gbps, 1),
        "windows_ms": main_res["windows_ms"],
        "device_windows_ms": main_res["device_windows_ms"],
        "cache_refresh_ms": main_res["cache_refresh_ms"],
        "stage_us_per_mini_batch": main_res["stage_us_per_mini_batch"],
        "one_stream": main_res["one_stream"],
        "walk_probability": main_res["walk_probability"],
        "dense_update": main_res.get("dense_update"),
        "input_nodes": main_res.get("input_nodes"),
        "per_config": per_config,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
