"""Seeded synthetic inputs: power-law (Chung-Lu) graphs, features, seed batches.

This module holds input generation only -- none of the sampling method's
arithmetic -- so that the HIP path and the CPU oracle can be fed the very same
arrays.  The shapes follow the paper's Table 1 workloads (node count, average
degree, feature width, training-split share); the real datasets are not used.

Everything is written with torch ops so the same recipe runs on the CPU (small
graphs, no GPU needed) or on the GPU (the 10^8-node graphs, where a CPU build
would take too long).  Results are deterministic for a given (seed, device
type, torch version).
"""
import math
from dataclasses import dataclass

import torch


@dataclass
class SynthGraph:
    num_nodes: int
    indptr: torch.Tensor    # int32 or int64 [n+1]
    indices: torch.Tensor   # int32 [nnz], rows ascending, no duplicates, no self loops, symmetric
    gamma: float
    max_degree: int

    @property
    def nnz(self):
        return int(self.indices.numel())


def _expected_degree_shape(n, gamma, total_endpoints, cap, device):
    """Weights w_i ~ (i + i0)^(-1/(gamma-1)), i = 1..n, with the shift i0 picked by
    bisection so that the largest expected degree stays below
    min(sqrt(total_endpoints), cap) (keeps Chung-Lu edge probabilities <= 1)."""
    alpha = 1.0 / (gamma - 1.0)
    i = torch.arange(1, n + 1, dtype=torch.float64, device=device)
    limit = min(math.sqrt(total_endpoints), float(cap))

    def top_degree(i0):
        w = (i + i0).pow(-alpha)
        return float(total_endpoints * w[0] / w.sum()), w

    lo, hi = 0.0, 1.0
    while top_degree(hi)[0] > limit:
        hi *= 2.0
        if hi > 1e12:
            break
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if top_degree(mid)[0] > limit:
            lo = mid
        else:
            hi = mid
    return top_degree(hi)[1]


def chung_lu_graph(n, num_undirected_edges, gamma, seed, *, max_degree_cap=20000, index64=False,
                   device="cpu", chunk=1 << 26):
    """Chung-Lu graph: num_undirected_edges endpoint pairs drawn i.i.d. with
    probability proportional to the expected-degree weights; self loops and
    repeated pairs are dropped, ids are shuffled by a seeded permutation (so hubs
    are spread over the id range), the adjacency is symmetrised and each CSR row
    sorted ascending."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    w = _expected_degree_shape(n, gamma, 2.0 * num_undirected_edges, max_degree_cap, dev)
    cdf = torch.cumsum(w, 0)
    cdf = cdf / cdf[-1]
    del w
    keys = []
    remaining = int(num_undirected_edges)
    while remaining > 0:
        m = min(remaining, chunk)
        a = torch.searchsorted(cdf, torch.rand(m, dtype=torch.float64, device=dev, generator=g)).clamp_(max=n - 1)
        b = torch.searchsorted(cdf, torch.rand(m, dtype=torch.float64, device=dev, generator=g)).clamp_(max=n - 1)
        keep = a != b
        a, b = a[keep], b[keep]
        keys.append(torch.minimum(a, b) * n + torch.maximum(a, b))
        remaining -= m
    del cdf
    key = torch.unique(torch.cat(keys))
    del keys
    perm = torch.randperm(n, device=dev, generator=g)
    a = perm[key // n]
    b = perm[key % n]
    del key, perm
    row = torch.cat([a, b])
    col = torch.cat([b, a])
    del a, b
    order_key, _ = torch.sort(row * n + col)
    del row, col
    row = order_key // n
    indices = (order_key % n).to(torch.int32)
    del order_key
    deg = torch.bincount(row, minlength=n)
    del row
    indptr = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    torch.cumsum(deg, 0, out=indptr[1:])
    max_deg = int(deg.max())
    if not index64:
        assert int(indptr[-1]) < 2 ** 31
        indptr = indptr.to(torch.int32)
    return SynthGraph(n, indptr, indices, gamma, max_deg)


def node_features(n, feat_dim, seed, *, device="cpu", pin=False, chunk_rows=1 << 22):
    """fp32 N(0,1) features, generated in row chunks (so a host-resident matrix
    bigger than device memory can be filled from a device generator)."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    if pin:
        out = torch.empty((n, feat_dim), dtype=torch.float32, pin_memory=True)
        for r0 in range(0, n, chunk_rows):
            r1 = min(n, r0 + chunk_rows)
            out[r0:r1].copy_(torch.randn((r1 - r0, feat_dim), dtype=torch.float32, device=dev, generator=g))
        return out
    return torch.randn((n, feat_dim), dtype=torch.float32, device=dev, generator=g)


def uniform_seed_batch(n, batch, seed, *, device="cpu"):
    """`batch` distinct node ids, uniform over V."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    if n <= (1 << 24):
        return torch.randperm(n, device=dev, generator=g)[:batch].to(torch.int32)
    # large n: draw with a margin, keep the first `batch` distinct values in draw order
    draw = torch.randint(0, n, (2 * batch + 64,), device=dev, generator=g)
    uniq, inv = torch.unique(draw, return_inverse=True)
    first = torch.full((uniq.numel(),), draw.numel(), dtype=torch.int64, device=dev)
    first.scatter_reduce_(0, inv, torch.arange(draw.numel(), device=dev), reduce="amin")
    keep = torch.sort(first).values[:batch]
    assert keep.numel() == batch
    return draw[keep].to(torch.int32)


def training_split(n, split_size, seed, *, device="cpu"):
    """A seeded training split: `split_size` distinct node ids."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    return torch.randperm(n, device=dev, generator=g)[:split_size].to(torch.int32)


def epoch_batches(split, batch, seed):
    """One shuffled epoch over a split, as a list of int32 batches (last one ragged)."""
    g = torch.Generator(device=split.device)
    g.manual_seed(int(seed))
    shuffled = split[torch.randperm(split.numel(), device=split.device, generator=g)]
    return [shuffled[i:i + batch].contiguous() for i in range(0, shuffled.numel(), batch)]


# The five workloads of this build (node count, undirected edges, exponent,
# feature width, cache share, fan-outs from the seeds inwards, batch size).
CONFIGS = {
    1: dict(n=10_000, edges=200_000, gamma=2.1, feat=64, cache_frac=0.01, fanouts=(10, 5), batch=256,
            index64=False, cap=20000, feat_on_host=False),
    2: dict(n=1_000_000, edges=20_000_000, gamma=2.1, feat=128, cache_frac=0.01, fanouts=(15, 10, 5), batch=1024,
            index64=False, cap=20000, feat_on_host=False, refresh_every=20, num_batches=100),
    3: dict(n=2_450_000, edges=62_000_000, gamma=2.0, feat=100, cache_frac=0.01, fanouts=(15, 10, 5), batch=1024,
            index64=False, cap=20000, feat_on_host=False, split=200_000),
    4: dict(n=10_000_000, edges=200_000_000, gamma=2.2, feat=256, cache_frac=0.005, fanouts=(15, 10, 5), batch=2048,
            index64=True, cap=20000, feat_on_host=True),
    5: dict(n=111_000_000, edges=800_000_000, gamma=2.1, feat=128, cache_frac=0.01, fanouts=(15, 10, 5), batch=1024,
            index64=True, cap=20000, feat_on_host=True, split=1_200_000, refresh_every=100),
}


def config_seeds(cfg_id):
    return dict(graph=1000 + cfg_id, feat=2000 + cfg_id, split=3000 + cfg_id, batch=4000 + cfg_id,
                cache=5000 + cfg_id)


def make_config_graph(cfg_id, *, device="cpu"):
    c = CONFIGS[cfg_id]
    return chung_lu_graph(c["n"], c["edges"], c["gamma"], config_seeds(cfg_id)["graph"],
                          max_degree_cap=c["cap"], index64=c["index64"], device=device)
