"""Shared plumbing of the GPU parity tests: upload a graph, drive the C ABI
through the Python binding, and compare every output with the CPU oracle."""
import numpy as np
import torch

import oracle
from paper_2106_06150_amd import binding as B

WEIGHT_RTOL = 1e-5     # fp32 weights: |gpu - ref| <= 1e-5 * |ref|
AGG_RTOL = 1e-5        # aggregates: error relative to (1/n_v) * sum |w_e x_e| per element


class GpuGns:
    def __init__(self, indptr, indices, feat=None, *, fanouts, policies, cache_size, max_seeds,
                 wmode=B.GNS_W_PRINTED, feat_on_host=False, device="cuda:0", flag_mode=0, cache_probability=0):
        self.device = torch.device(device)
        self.indptr_cpu = indptr
        self.indices_cpu = indices
        self.feat_cpu = feat
        self.indptr = indptr.to(self.device)
        self.indices = indices.to(self.device)
        self.feat_dev = None
        self.feat_host = None
        if feat is not None:
            if feat_on_host:
                self.feat_host = feat if feat.is_pinned() else feat.pin_memory()
            else:
                self.feat_dev = feat.to(self.device)
        self.graph = B.make_graph(self.indptr, self.indices, self.feat_dev, self.feat_host)
        self.config = B.make_config(fanouts, policies, cache_size, max_seeds, wmode, flag_mode, cache_probability)
        self.prob_prefix = None          # oracle-side prefix of the cache probability (None: the CSR offsets)
        self.fanouts, self.policies, self.cache_size, self.wmode = list(fanouts), list(policies), cache_size, wmode
        self.workspace = B.alloc_workspace(self.graph, self.config, self.device)
        self.ctx = B.gns_create(self.graph, self.config, self.workspace)
        self.blocks = B.BlockBuffers(self.graph, self.config, self.device)

    def close(self):
        if self.ctx is not None:
            B.gns_destroy(self.ctx)
            self.ctx = None

    # -- cache ---------------------------------------------------------------
    def walk_probability(self, train_nodes, scale_log2):
        """Random-walk cache probability on the GPU; returns (weights u64[n], prefix i64[n+1], total, support)."""
        B.gns_cache_walk_probability(self.ctx, train_nodes.to(self.device).contiguous(), scale_log2)
        w_ptr, pre_ptr, total, support = B.gns_cache_probability_view(self.ctx)
        n = self.indptr.numel() - 1
        w = B.device_view_u64(w_ptr, n, self.device).cpu().numpy().view(np.uint64)
        pre = B.device_view_u64(pre_ptr, n + 1, self.device).cpu().numpy().view(np.int64)
        return w, pre, total, support

    def sample_cache(self, seed, epoch):
        B.gns_sample_cache(self.ctx, seed, epoch)
        nodes_ptr, size, bitmap_ptr, draws = B.gns_cache_view(self.ctx)
        n = self.indptr.numel() - 1
        nodes = B.device_view_i32(nodes_ptr, size, self.device).cpu().numpy()
        bitmap = B.device_view_u64(bitmap_ptr, (n + 63) // 64, self.device).cpu().numpy().view(np.uint64)
        return nodes, bitmap, draws

    # -- blocks --------------------------------------------------------------
    def sample_blocks(self, seed, seeds):
        seeds_dev = seeds.to(self.device).contiguous()
        B.gns_sample_blocks(self.ctx, seed, seeds_dev, self.blocks.array)
        return [self.blocks.views(i) for i in range(len(self.fanouts))]

    def gather(self, nodes_dev, num):
        F = self.graph.feat_dim
        out = torch.empty((num, F), dtype=torch.float32, device=self.device)
        B.gns_gather_features(self.ctx, nodes_dev, num, out)
        torch.cuda.synchronize()
        return out

    def aggregate(self, layer_index, x_src):
        b = self.blocks.array[layer_index]
        F = x_src.shape[1]
        out = torch.empty((b.num_dst, F), dtype=torch.float32, device=self.device)
        B.gns_aggregate(self.ctx, b, x_src, F, out)
        torch.cuda.synchronize()
        return out


def oracle_cache(indptr, seed, epoch, cache_size):
    return oracle.sample_cache(indptr.numpy(), seed, epoch, cache_size)


def compare_cache(gpu, ref):
    g_nodes, g_bitmap, g_draws = gpu
    r_nodes, r_bitmap, r_draws = ref
    assert g_draws == r_draws, (g_draws, r_draws)
    assert np.array_equal(g_nodes, r_nodes)
    assert np.array_equal(g_bitmap, r_bitmap)


def compare_blocks(gpu_views, ref_blocks):
    assert len(gpu_views) == len(ref_blocks)
    for i, (g, r) in enumerate(zip(gpu_views, ref_blocks)):
        assert (g["num_dst"], g["num_src"], g["num_edges"]) == (r.num_dst, r.num_src, r.num_edges), \
            (i, g["num_dst"], g["num_src"], g["num_edges"], r.num_dst, r.num_src, r.num_edges)
        for name, ref in [("indptr", r.indptr), ("indices", r.indices), ("src_nodes", r.src_nodes),
                          ("row_eligible", r.row_eligible)]:
            got = g[name].cpu().numpy()
            assert got.tobytes() == np.ascontiguousarray(ref, dtype=np.int32).tobytes(), (i, name)
        gw = g["weights"].cpu().numpy().astype(np.float64)
        rw = r.weights.astype(np.float64)
        assert np.all(np.abs(gw - rw) <= WEIGHT_RTOL * np.abs(rw)), (i, float(np.max(np.abs(gw - rw) / np.abs(rw))))


def aggregate_scale(blk, x_src):
    """(1/n_v) * sum_e |w_e * x_e| per output element, fp64 (the error yardstick)."""
    import scipy.sparse as sp
    A = sp.csr_matrix((np.abs(blk.weights.astype(np.float64)), blk.indices, blk.indptr),
                      shape=(blk.num_dst, blk.num_src))
    n_v = np.maximum(np.diff(blk.indptr), 1).astype(np.float64)
    return (A @ np.abs(x_src.astype(np.float64))) / n_v[:, None]


def compare_aggregate(gpu_out, ref_out, scale):
    err = np.abs(gpu_out.astype(np.float64) - ref_out.astype(np.float64))
    assert np.all(err <= AGG_RTOL * scale + 1e-30), float(np.max(err / (scale + 1e-30)))


def full_parity(gns, *, cache_seed, epoch, batch_seed, seeds, check_gather=True, check_aggregate=True):
    """Cache + blocks + gather + aggregate of one mini-batch against the oracle."""
    ip = gns.indptr_cpu.numpy()
    ix = gns.indices_cpu.numpy()
    bitmap = None
    if any(p != B.GNS_UNIFORM for p in gns.policies):
        ref_cache = oracle.sample_cache(ip if gns.prob_prefix is None else gns.prob_prefix, cache_seed, epoch, gns.cache_size)
        compare_cache(gns.sample_cache(cache_seed, epoch), ref_cache)
        bitmap = ref_cache[1]
    ref_blocks = oracle.sample_blocks(ip, ix, bitmap, gns.cache_size, batch_seed, seeds.numpy(), gns.fanouts,
                                      gns.policies, gns.wmode, prob_prefix=gns.prob_prefix)
    views = gns.sample_blocks(batch_seed, seeds)
    compare_blocks(views, ref_blocks)
    if gns.feat_cpu is None:
        return views, ref_blocks
    last = len(ref_blocks) - 1
    x_ref = oracle.gather(gns.feat_cpu.numpy(), ref_blocks[last].src_nodes)
    if check_gather:
        x_gpu = gns.gather(gns.blocks.tensors[last]["src_nodes"], views[last]["num_src"])
        assert x_gpu.cpu().numpy().tobytes() == x_ref.tobytes()
    else:
        x_gpu = torch.from_numpy(x_ref).to(gns.device)
    if check_aggregate:
        out_gpu = gns.aggregate(last, x_gpu).cpu().numpy()
        out_ref = oracle.aggregate(ref_blocks[last].indptr, ref_blocks[last].indices, ref_blocks[last].weights, x_ref)
        compare_aggregate(out_gpu, out_ref, aggregate_scale(ref_blocks[last], x_ref))
    return views, ref_blocks
