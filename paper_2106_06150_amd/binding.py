"""Thin ctypes binding of libgns.so: argument marshalling only.

Every step of the hot path runs in the library's HIP kernels; torch is used for
device memory and streams.  There is no CPU fallback: if the library is not
built, importing this module raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgns.so")

GNS_OK, GNS_EINVAL, GNS_ECAPACITY, GNS_ESTATE, GNS_EHIP, GNS_ENOMEM, GNS_ENOTIMPL = range(7)
GNS_UNIFORM, GNS_CACHE_ONLY, GNS_CACHE_FIRST = 0, 1, 2
GNS_W_PRINTED, GNS_W_UNBIASED = 0, 1
GNS_FLAGS_PER_BATCH, GNS_FLAGS_PER_CACHE = 0, 1
GNS_PROB_DEGREE, GNS_PROB_WALK = 0, 1
GNS_MAX_LAYERS = 8
GNS_MAX_FANOUT = 64
GNS_MAX_GROUP = 16

STATUS_NAMES = ["GNS_OK", "GNS_EINVAL", "GNS_ECAPACITY", "GNS_ESTATE", "GNS_EHIP", "GNS_ENOMEM", "GNS_ENOTIMPL"]


class gns_graph(ctypes.Structure):
    _fields_ = [("num_nodes", ctypes.c_int64), ("num_entries", ctypes.c_int64),
                ("indptr", ctypes.c_void_p), ("indptr_is_i64", ctypes.c_int32),
                ("indices", ctypes.c_void_p), ("feat_dim", ctypes.c_int32),
                ("feat_dev", ctypes.c_void_p), ("feat_host_pinned", ctypes.c_void_p)]


class gns_config(ctypes.Structure):
    _fields_ = [("num_layers", ctypes.c_int32), ("fanout", ctypes.c_int32 * GNS_MAX_LAYERS),
                ("policy", ctypes.c_int32 * GNS_MAX_LAYERS), ("cache_size", ctypes.c_int64),
                ("wmode", ctypes.c_int32), ("max_seeds", ctypes.c_int32),
                ("flag_mode", ctypes.c_int32), ("cache_probability", ctypes.c_int32)]


class gns_block(ctypes.Structure):
    _fields_ = [("num_dst", ctypes.c_int32), ("num_src", ctypes.c_int32), ("num_edges", ctypes.c_int32),
                ("indptr", ctypes.c_void_p), ("indices", ctypes.c_void_p), ("src_nodes", ctypes.c_void_p),
                ("row_eligible", ctypes.c_void_p), ("weights", ctypes.c_void_p),
                ("cap_dst", ctypes.c_int32), ("cap_src", ctypes.c_int32), ("cap_edges", ctypes.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libgns.so is not built: run `python -m paper_2106_06150_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64
    P = ctypes.POINTER
    lib.gns_workspace_bytes.argtypes = [P(gns_graph), P(gns_config)]
    lib.gns_workspace_bytes.restype = ctypes.c_size_t
    lib.gns_block_capacity.argtypes = [P(gns_graph), P(gns_config), i32, P(i32), P(i32), P(i32)]
    lib.gns_block_capacity.restype = ctypes.c_int
    lib.gns_create.argtypes = [P(vp), P(gns_graph), P(gns_config), vp, ctypes.c_size_t, vp]
    lib.gns_create.restype = ctypes.c_int
    lib.gns_fork_workspace_bytes.argtypes = [vp]
    lib.gns_fork_workspace_bytes.restype = ctypes.c_size_t
    lib.gns_fork.argtypes = [vp, vp, ctypes.c_size_t, vp, P(vp)]
    lib.gns_fork.restype = ctypes.c_int
    lib.gns_destroy.argtypes = [vp]
    lib.gns_destroy.restype = ctypes.c_int
    lib.gns_sample_cache.argtypes = [vp, u64, u64, vp]
    lib.gns_sample_cache.restype = ctypes.c_int
    lib.gns_sample_cache_async.argtypes = [vp, u64, u64, vp]
    lib.gns_sample_cache_async.restype = ctypes.c_int
    lib.gns_activate_cache.argtypes = [vp]
    lib.gns_activate_cache.restype = ctypes.c_int
    lib.gns_cache_walk_probability.argtypes = [vp, vp, i64, i32, vp]
    lib.gns_cache_walk_probability.restype = ctypes.c_int
    lib.gns_cache_probability_view.argtypes = [vp, P(vp), P(vp), P(u64), P(i64)]
    lib.gns_cache_probability_view.restype = ctypes.c_int
    lib.gns_cache_view.argtypes = [vp, P(vp), P(i64), P(vp), P(i64)]
    lib.gns_cache_view.restype = ctypes.c_int
    lib.gns_sample_blocks.argtypes = [vp, u64, vp, i32, P(gns_block), vp]
    lib.gns_sample_blocks.restype = ctypes.c_int
    lib.gns_sample_blocks_async.argtypes = [vp, u64, vp, i32, P(gns_block), vp]
    lib.gns_sample_blocks_async.restype = ctypes.c_int
    lib.gns_sample_blocks_group.argtypes = [P(vp), i32, P(u64), P(vp), P(i32), P(P(gns_block)), vp]
    lib.gns_sample_blocks_group.restype = ctypes.c_int
    lib.gns_sample_blocks_group_wait.argtypes = [P(vp), i32, P(P(gns_block)), vp]
    lib.gns_sample_blocks_group_wait.restype = ctypes.c_int
    lib.gns_gather_features_group.argtypes = [P(vp), i32, P(vp), P(i32), P(vp), vp]
    lib.gns_gather_features_group.restype = ctypes.c_int
    lib.gns_aggregate_group.argtypes = [P(vp), i32, P(P(gns_block)), P(vp), i32, P(vp), vp]
    lib.gns_aggregate_group.restype = ctypes.c_int
    lib.gns_sample_blocks_static.argtypes = [vp, u64, vp, i32, P(gns_block), vp]
    lib.gns_sample_blocks_static.restype = ctypes.c_int
    lib.gns_sample_blocks_wait.argtypes = [vp, P(gns_block), vp]
    lib.gns_sample_blocks_wait.restype = ctypes.c_int
    lib.gns_gather_features.argtypes = [vp, vp, i32, vp, vp]
    lib.gns_gather_features.restype = ctypes.c_int
    lib.gns_aggregate.argtypes = [vp, P(gns_block), vp, i32, vp, vp]
    lib.gns_aggregate.restype = ctypes.c_int
    lib.gns_sage_dense.argtypes = [vp, vp, i32, vp, i32, vp, vp, i32, i32, vp, i32, vp]
    lib.gns_sage_dense.restype = ctypes.c_int
    lib.gns_profile_begin.argtypes = [vp, ctypes.c_uint32, i32]
    lib.gns_profile_begin.restype = ctypes.c_int
    lib.gns_profile_collect.argtypes = [vp, i32, P(ctypes.c_double), P(i32)]
    lib.gns_profile_collect.restype = ctypes.c_int
    lib.gns_last_error.argtypes = [vp]
    lib.gns_last_error.restype = ctypes.c_char_p
    return lib


lib = _load()

EXPORTED = ["gns_workspace_bytes", "gns_block_capacity", "gns_create", "gns_destroy", "gns_sample_cache",
            "gns_cache_view", "gns_sample_blocks", "gns_gather_features", "gns_aggregate", "gns_last_error",
            "gns_profile_begin", "gns_profile_collect", "gns_sample_blocks_async", "gns_sample_blocks_wait",
            "gns_fork", "gns_fork_workspace_bytes", "gns_cache_walk_probability", "gns_cache_probability_view", "gns_sage_dense", "gns_sample_cache_async", "gns_activate_cache",
            "gns_sample_blocks_static", "gns_sample_blocks_group", "gns_sample_blocks_group_wait",
            "gns_gather_features_group", "gns_aggregate_group"]
GNS_STATIC_SCRATCH_BYTES = 128 << 20

GNS_STAGE_SAMPLE, GNS_STAGE_FINISH, GNS_STAGE_GATHER, GNS_STAGE_AGGREGATE = 0, 8, 16, 17
GNS_STAGE_DENSE = 21
GNS_STAGE_PLAN, GNS_STAGE_FLAG, GNS_STAGE_SELECT = 18, 19, 20


class GnsError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status, message))
        self.status = status


def _check(status, ctx=None):
    if status != GNS_OK:
        raise GnsError(status, lib.gns_last_error(ctx).decode())


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def make_graph(indptr, indices, feat_dev=None, feat_host_pinned=None, feat_dim=None):
    """gns_graph from torch tensors (indptr/indices on the device; features on the
    device and/or in pinned host memory)."""
    assert indptr.is_cuda and indices.is_cuda and indices.dtype == torch.int32
    assert indptr.dtype in (torch.int32, torch.int64)
    g = gns_graph()
    g.num_nodes = indptr.numel() - 1
    g.num_entries = indices.numel()
    g.indptr = indptr.data_ptr()
    g.indptr_is_i64 = 1 if indptr.dtype == torch.int64 else 0
    g.indices = indices.data_ptr()
    feat = feat_dev if feat_dev is not None else feat_host_pinned
    g.feat_dim = int(feat.shape[1]) if feat is not None else int(feat_dim or 0)
    if feat_dev is not None:
        assert feat_dev.is_cuda and feat_dev.dtype == torch.float32 and feat_dev.is_contiguous()
        g.feat_dev = feat_dev.data_ptr()
    if feat_host_pinned is not None:
        assert feat_host_pinned.is_pinned() and feat_host_pinned.dtype == torch.float32
        g.feat_host_pinned = feat_host_pinned.data_ptr()
    g._keep = (indptr, indices, feat_dev, feat_host_pinned)
    return g


def make_config(fanouts, policies, cache_size, max_seeds, wmode=GNS_W_PRINTED, flag_mode=GNS_FLAGS_PER_BATCH,
                cache_probability=0):
    c = gns_config()
    c.num_layers = len(fanouts)
    for i, (k, p) in enumerate(zip(fanouts, policies)):
        c.fanout[i] = k
        c.policy[i] = p
    c.cache_size = cache_size
    c.wmode = wmode
    c.max_seeds = max_seeds
    c.flag_mode = flag_mode
    c.cache_probability = cache_probability
    return c


def gns_workspace_bytes(graph, config):
    n = lib.gns_workspace_bytes(ctypes.byref(graph), ctypes.byref(config))
    if n == 0:
        raise GnsError(GNS_EINVAL, lib.gns_last_error(None).decode())
    return n


def gns_block_capacity(graph, config, layer_index):
    a, b, c = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib.gns_block_capacity(ctypes.byref(graph), ctypes.byref(config), layer_index,
                                  ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def gns_create(graph, config, workspace, stream=None):
    ctx = ctypes.c_void_p()
    _check(lib.gns_create(ctypes.byref(ctx), ctypes.byref(graph), ctypes.byref(config),
                          workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(stream)))
    return ctx


def gns_fork_workspace_bytes(parent):
    return lib.gns_fork_workspace_bytes(parent)


def gns_fork(parent, workspace, stream=None):
    child = ctypes.c_void_p()
    _check(lib.gns_fork(parent, workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                        _stream_ptr(stream), ctypes.byref(child)), parent)
    return child


def gns_destroy(ctx):
    _check(lib.gns_destroy(ctx))


def gns_sample_cache(ctx, seed, epoch, stream=None):
    _check(lib.gns_sample_cache(ctx, seed, epoch, _stream_ptr(stream)), ctx)


def gns_sample_cache_async(ctx, seed, epoch, stream=None):
    _check(lib.gns_sample_cache_async(ctx, seed, epoch, _stream_ptr(stream)), ctx)


def gns_activate_cache(ctx):
    _check(lib.gns_activate_cache(ctx), ctx)


def gns_cache_walk_probability(ctx, train_nodes_dev, scale_log2, stream=None):
    assert train_nodes_dev.is_cuda and train_nodes_dev.dtype == torch.int32 and train_nodes_dev.is_contiguous()
    _check(lib.gns_cache_walk_probability(ctx, train_nodes_dev.data_ptr(), train_nodes_dev.numel(), scale_log2,
                                          _stream_ptr(stream)), ctx)


def gns_cache_probability_view(ctx):
    """Returns (weights_ptr, prefix_ptr, total, support) -- raw device pointers and host scalars."""
    w, pre = ctypes.c_void_p(), ctypes.c_void_p()
    total, support = ctypes.c_uint64(), ctypes.c_int64()
    _check(lib.gns_cache_probability_view(ctx, ctypes.byref(w), ctypes.byref(pre), ctypes.byref(total),
                                          ctypes.byref(support)), ctx)
    return w.value, pre.value, total.value, support.value


def gns_cache_view(ctx):
    """Returns (cache_nodes_ptr, cache_size, bitmap_ptr, num_draws) -- raw device pointers."""
    nodes, bitmap = ctypes.c_void_p(), ctypes.c_void_p()
    size, draws = ctypes.c_int64(), ctypes.c_int64()
    _check(lib.gns_cache_view(ctx, ctypes.byref(nodes), ctypes.byref(size), ctypes.byref(bitmap),
                              ctypes.byref(draws)), ctx)
    return nodes.value, size.value, bitmap.value, draws.value


def gns_sample_blocks(ctx, seed, seeds_dev, blocks, stream=None):
    """blocks: ctypes array of gns_block (see alloc_blocks)."""
    assert seeds_dev.is_cuda and seeds_dev.dtype == torch.int32 and seeds_dev.is_contiguous()
    _check(lib.gns_sample_blocks(ctx, seed, seeds_dev.data_ptr(), seeds_dev.numel(), blocks, _stream_ptr(stream)), ctx)


def gns_sample_blocks_async(ctx, seed, seeds_dev, blocks, stream=None):
    assert seeds_dev.is_cuda and seeds_dev.dtype == torch.int32 and seeds_dev.is_contiguous()
    _check(lib.gns_sample_blocks_async(ctx, seed, seeds_dev.data_ptr(), seeds_dev.numel(), blocks,
                                       _stream_ptr(stream)), ctx)


def gns_sample_blocks_static(ctx, seed, seeds_dev, blocks, stream=None):
    assert seeds_dev.is_cuda and seeds_dev.dtype == torch.int32 and seeds_dev.is_contiguous()
    _check(lib.gns_sample_blocks_static(ctx, seed, seeds_dev.data_ptr(), seeds_dev.numel(), blocks,
                                        _stream_ptr(stream)), ctx)


class GroupCall:
    """Argument arrays of the gns_*_group calls for a fixed set of contexts and block buffers (marshalling
    only: built once, reused for every call; seeds and per-call pointers are filled in per call)."""

    def __init__(self, ctxs, block_arrays):
        n = len(ctxs)
        assert 1 <= n <= GNS_MAX_GROUP and len(block_arrays) == n
        self.n = n
        self.lead = ctxs[0]
        self.ctxs = (ctypes.c_void_p * n)(*[c.value if isinstance(c, ctypes.c_void_p) else c for c in ctxs])
        self.blocks = (ctypes.POINTER(gns_block) * n)(*[ctypes.cast(b, ctypes.POINTER(gns_block)) for b in block_arrays])
        self.seeds = (ctypes.c_uint64 * n)()
        self.seeds_dev = (ctypes.c_void_p * n)()
        self.num_seeds = (ctypes.c_int32 * n)()
        self.nodes = (ctypes.c_void_p * n)()
        self.num_nodes = (ctypes.c_int32 * n)()
        self.out = (ctypes.c_void_p * n)()
        self.agg_blocks = (ctypes.POINTER(gns_block) * n)()
        self.x_src = (ctypes.c_void_p * n)()
        self.agg_out = (ctypes.c_void_p * n)()
        self._keep = (ctxs, block_arrays)

    def sample(self, seeds, seeds_dev, stream=None):
        """seeds: n integers; seeds_dev: n int32 device tensors.  Enqueue only (counts stay on the device)."""
        for b in range(self.n):
            t = seeds_dev[b]
            assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
            self.seeds[b] = seeds[b]
            self.seeds_dev[b] = t.data_ptr()
            self.num_seeds[b] = t.numel()
        _check(lib.gns_sample_blocks_group(self.ctxs, self.n, self.seeds, self.seeds_dev, self.num_seeds, self.blocks,
                                           _stream_ptr(stream)), self.lead)

    def wait(self, stream=None):
        _check(lib.gns_sample_blocks_group_wait(self.ctxs, self.n, self.blocks, _stream_ptr(stream)), self.lead)

    def gather(self, nodes_dev, num_nodes, out_dev, stream=None):
        for b in range(self.n):
            self.nodes[b] = nodes_dev[b].data_ptr()
            self.num_nodes[b] = num_nodes[b]
            self.out[b] = out_dev[b].data_ptr()
        _check(lib.gns_gather_features_group(self.ctxs, self.n, self.nodes, self.num_nodes, self.out,
                                             _stream_ptr(stream)), self.lead)

    def aggregate(self, layer_index, x_src_dev, feat_dim, out_dev, stream=None):
        for b in range(self.n):
            self.agg_blocks[b] = ctypes.pointer(self.blocks[b][layer_index])
            self.x_src[b] = x_src_dev[b].data_ptr()
            self.agg_out[b] = out_dev[b].data_ptr()
        _check(lib.gns_aggregate_group(self.ctxs, self.n, self.agg_blocks, self.x_src, feat_dim, self.agg_out,
                                       _stream_ptr(stream)), self.lead)


def gns_sample_blocks_wait(ctx, blocks, stream=None):
    _check(lib.gns_sample_blocks_wait(ctx, blocks, _stream_ptr(stream)), ctx)


def gns_gather_features(ctx, nodes_dev, num_nodes, out_dev, stream=None):
    _check(lib.gns_gather_features(ctx, nodes_dev.data_ptr(), num_nodes, out_dev.data_ptr(), _stream_ptr(stream)), ctx)


def gns_aggregate(ctx, block, x_src_dev, feat_dim, out_dev, stream=None):
    _check(lib.gns_aggregate(ctx, ctypes.byref(block), x_src_dev.data_ptr(), feat_dim, out_dev.data_ptr(),
                             _stream_ptr(stream)), ctx)


def gns_sage_dense(ctx, h_self_dev, h_neigh_dev, w_dev, bias_dev, relu, out_dev, num_rows, stream=None):
    f1, f2, hdim = h_self_dev.shape[1], h_neigh_dev.shape[1], w_dev.shape[1]
    assert w_dev.shape[0] == f1 + f2 and all(t.is_contiguous() for t in (h_self_dev, h_neigh_dev, w_dev, out_dev))
    _check(lib.gns_sage_dense(ctx, h_self_dev.data_ptr(), f1, h_neigh_dev.data_ptr(), f2, w_dev.data_ptr(),
                              None if bias_dev is None else bias_dev.data_ptr(), hdim, 1 if relu else 0,
                              out_dev.data_ptr(), num_rows, _stream_ptr(stream)), ctx)


def gns_profile_begin(ctx, stage_mask, capacity):
    _check(lib.gns_profile_begin(ctx, stage_mask, capacity), ctx)


def gns_profile_collect(ctx, stage):
    """Returns (total_ms, launches) of the recorded launches of `stage`."""
    ms, n = ctypes.c_double(), ctypes.c_int32()
    _check(lib.gns_profile_collect(ctx, stage, ctypes.byref(ms), ctypes.byref(n)), ctx)
    return ms.value, n.value


# ---------------------------------------------------------------------------
# Memory plumbing helpers (allocation only).

class BlockBuffers:
    """Worst-case device buffers for the blocks of one mini-batch, plus the
    ctypes array the library fills in."""

    def __init__(self, graph, config, device):
        L = config.num_layers
        self.array = (gns_block * L)()
        self.tensors = []
        for i in range(L):
            cap_dst, cap_src, cap_edges = gns_block_capacity(graph, config, i)
            t = dict(indptr=torch.empty(cap_dst + 1, dtype=torch.int32, device=device),
                     indices=torch.empty(max(cap_edges, 1), dtype=torch.int32, device=device),
                     src_nodes=torch.empty(max(cap_src, 1), dtype=torch.int32, device=device),
                     row_eligible=torch.empty(max(cap_dst, 1), dtype=torch.int32, device=device),
                     weights=torch.empty(max(cap_edges, 1), dtype=torch.float32, device=device))
            self.tensors.append(t)
            b = self.array[i]
            b.indptr, b.indices, b.src_nodes = t["indptr"].data_ptr(), t["indices"].data_ptr(), t["src_nodes"].data_ptr()
            b.row_eligible, b.weights = t["row_eligible"].data_ptr(), t["weights"].data_ptr()
            b.cap_dst, b.cap_src, b.cap_edges = cap_dst, cap_src, cap_edges

    def views(self, i):
        """Tensors of block i trimmed to the counts the library reported."""
        b, t = self.array[i], self.tensors[i]
        return dict(indptr=t["indptr"][:b.num_dst + 1], indices=t["indices"][:b.num_edges],
                    src_nodes=t["src_nodes"][:b.num_src], row_eligible=t["row_eligible"][:b.num_dst],
                    weights=t["weights"][:b.num_edges], num_dst=b.num_dst, num_src=b.num_src,
                    num_edges=b.num_edges)


def alloc_workspace(graph, config, device):
    nbytes = gns_workspace_bytes(graph, config)
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def device_view_i32(ptr, count, device):
    """Copies `count` int32 from a raw device pointer into a new tensor (for tests)."""
    out = torch.empty(count, dtype=torch.int32, device=device)
    if count:
        rc = _hip_memcpy_dtod(out.data_ptr(), ptr, count * 4)
        assert rc == 0
    return out


def device_view_u64(ptr, count, device):
    out = torch.empty(count, dtype=torch.int64, device=device)
    if count:
        rc = _hip_memcpy_dtod(out.data_ptr(), ptr, count * 8)
        assert rc == 0
    return out


_hip = None


def _hip_memcpy_dtod(dst, src, nbytes):
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
        _hip.hipMemcpy.restype = ctypes.c_int
    torch.cuda.synchronize()
    return _hip.hipMemcpy(dst, src, nbytes, 3)  # hipMemcpyDeviceToDevice
