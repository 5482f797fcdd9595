"""gns_sample_blocks_static (the entry point for callers that cannot allocate device memory: its per-batch
scratch is a fixed array inside the library) against gns_sample_blocks, through the C ABI.

Two calls in a row on the same GPU, the second with a smaller input, each compared with what the existing
entry point writes for the same arguments: integers bit for bit, fp32 weights within 1e-5 relative; and, since
both run the same kernels, with the CPU oracle as well.
"""
import numpy as np
import pytest
import torch

import oracle
from conftest import random_symmetric_csr
from paper_2106_06150_amd import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2106_06150_amd import binding as B
    from gpu_harness import GpuGns, compare_blocks, WEIGHT_RTOL

U, C, CF = 0, 1, 2


def _snapshot(bufs, L):
    out = []
    for i in range(L):
        v = bufs.views(i)
        out.append({k: (t.clone() if torch.is_tensor(t) else t) for k, t in v.items()})
    return out


def _same(a, b):
    for x, y in zip(a, b):
        assert (x["num_dst"], x["num_src"], x["num_edges"]) == (y["num_dst"], y["num_src"], y["num_edges"])
        for name in ("indptr", "indices", "src_nodes", "row_eligible"):
            assert torch.equal(x[name], y[name]), name
        wx, wy = x["weights"].double(), y["weights"].double()
        assert bool(torch.all((wx - wy).abs() <= WEIGHT_RTOL * wy.abs()))


@pytest.mark.parametrize("fanouts,policies", [((6, 4, 3), (U, U, C)), ((5, 7), (CF, CF))])
def test_static_scratch_entry_point_matches_the_workspace_one(fanouts, policies):
    ip, ix = random_symmetric_csr(5000, 16, np.random.default_rng(41), hub_boost=1)
    ip, ix = torch.from_numpy(ip), torch.from_numpy(ix)
    n = ip.numel() - 1
    csize, bs = 350, 160
    gns = GpuGns(ip, ix, None, fanouts=fanouts, policies=policies, cache_size=csize, max_seeds=bs, flag_mode=1)
    other = B.BlockBuffers(gns.graph, gns.config, gns.device)
    L = len(fanouts)
    try:
        B.gns_sample_cache(gns.ctx, 17, 0)
        cache = oracle.sample_cache(ip.numpy(), 17, 0, csize)
        # two calls in a row; the second has fewer seeds (a smaller input on the same array)
        for call, count in enumerate((bs, 37)):
            seeds = synth.uniform_seed_batch(n, count, 500 + call).cuda()
            B.gns_sample_blocks_static(gns.ctx, 90 + call, seeds, other.array)
            got = _snapshot(other, L)
            B.gns_sample_blocks(gns.ctx, 90 + call, seeds, gns.blocks.array)
            want = _snapshot(gns.blocks, L)
            _same(got, want)
            ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], csize, 90 + call, seeds.cpu().numpy(),
                                       list(fanouts), list(policies))
            compare_blocks(got, ref)
        # bad seeds are reported by the static call itself
        dup = synth.uniform_seed_batch(n, 20, 7).cuda()
        dup[3] = dup[11]
        with pytest.raises(B.GnsError) as e:
            B.gns_sample_blocks_static(gns.ctx, 5, dup, other.array)
        assert e.value.status == B.GNS_EINVAL
        # and the array is usable again afterwards, from a fork of the context as well
        ws = torch.empty(B.gns_fork_workspace_bytes(gns.ctx), dtype=torch.uint8, device=gns.device)
        fork = B.gns_fork(gns.ctx, ws)
        try:
            seeds = synth.uniform_seed_batch(n, 64, 900).cuda()
            B.gns_sample_blocks_static(fork, 123, seeds, other.array)
            ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], csize, 123, seeds.cpu().numpy(),
                                       list(fanouts), list(policies))
            compare_blocks(_snapshot(other, L), ref)
        finally:
            B.gns_destroy(fork)
    finally:
        gns.close()


def test_static_scratch_rejects_what_does_not_fit():
    """A config whose per-batch scratch exceeds the library's array is refused before anything is launched."""
    ip, ix = random_symmetric_csr(300000, 6, np.random.default_rng(5))
    ip, ix = torch.from_numpy(ip), torch.from_numpy(ix)
    n = ip.numel() - 1
    # fan-out 64 from up to 300000 seeds: the sampler scratch alone (19.2 M slots, twice, ids and weights) is
    # beyond the array
    gns = GpuGns(ip, ix, None, fanouts=(64,), policies=(U,), cache_size=0, max_seeds=300000)
    try:
        assert B.gns_fork_workspace_bytes(gns.ctx) > B.GNS_STATIC_SCRATCH_BYTES
        seeds = synth.uniform_seed_batch(n, 16, 1).cuda()
        with pytest.raises(B.GnsError) as e:
            B.gns_sample_blocks_static(gns.ctx, 1, seeds, gns.blocks.array)
        assert e.value.status == B.GNS_ECAPACITY
    finally:
        gns.close()
