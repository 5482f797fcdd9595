"""GPU parity: the HIP library, called through the C ABI, against the CPU oracle.

Integer outputs (cache list, bitmap, draw count, block CSRs, src lists,
eligible counts, gathered rows) must be bit-exact; fp32 weights within 1e-5
relative; aggregates within 1e-5 of (1/n_v) * sum |w_e x_e| per element.
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
    from gpu_harness import GpuGns, full_parity, compare_cache, compare_blocks, AGG_RTOL

U, C, CF = 0, 1, 2          # UNIFORM, CACHE_ONLY, CACHE_FIRST


def _small(n=3000, avg=14, seed=3, hub=1):
    ip, ix = random_symmetric_csr(n, avg, np.random.default_rng(seed), hub_boost=hub)
    return torch.from_numpy(ip), torch.from_numpy(ix)


def _feat(n, F, seed=0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn((n, F), dtype=torch.float32, generator=g)


@pytest.mark.parametrize("flag_mode", [0, 1])
@pytest.mark.parametrize("offsets", [torch.int32, torch.int64])
@pytest.mark.parametrize("fanouts,policies", [((10, 5), (U, C)), ((15, 10, 5), (U, U, C)), ((3, 2, 1), (C, C, C)),
                                              ((4, 4), (U, U)), ((20, 17), (U, C)), ((6, 12), (U, C)),
                                              ((15, 10, 5), (CF, CF, C)), ((6, 9), (CF, CF)), ((20, 40), (U, CF))])
def test_small_graph_parity(offsets, fanouts, policies, flag_mode):
    ip, ix = _small()
    n = ip.numel() - 1
    feat = _feat(n, 64)
    gns = GpuGns(ip.to(offsets), ix, feat, fanouts=fanouts, policies=policies, cache_size=300, max_seeds=200,
                 flag_mode=flag_mode)
    try:
        for trial in range(3):
            seeds = synth.uniform_seed_batch(n, 200 - 37 * trial, 100 + trial)
            full_parity(gns, cache_seed=9, epoch=trial, batch_seed=1000 + trial, seeds=seeds)
    finally:
        gns.close()


@pytest.mark.parametrize("F", [1, 3, 4, 32, 64, 96, 100, 128, 256, 260, 1024])
def test_feature_widths_and_host_store(F):
    ip, ix = _small(n=1500)
    n = ip.numel() - 1
    feat = _feat(n, F, seed=F)
    for on_host in (False, True):
        gns = GpuGns(ip, ix, feat, fanouts=(6, 4), policies=(U, C), cache_size=150, max_seeds=64, feat_on_host=on_host)
        try:
            seeds = synth.uniform_seed_batch(n, 64, 5)
            full_parity(gns, cache_seed=1, epoch=0, batch_seed=77, seeds=seeds)
        finally:
            gns.close()


@pytest.mark.parametrize("F,rows,max_deg", [(128, 70_000, 5), (128, 3_000, 20), (64, 40_000, 9), (256, 20_000, 12),
                                            (100, 40_000, 9), (8, 5_000, 20), (1024, 600, 9)])
def test_aggregate_on_hand_made_blocks(F, rows, max_deg):
    """gns_aggregate alone on a block that no sampler made: rows with 0..max_deg edges (several rounds of the
    kernel's inner loop), more rows than one pass of the grid covers (the kernel's pipeline over rows), empty rows
    next to full ones, non-finite values in source row 0 (empty rows must still give 0), repeated sources."""
    rng = np.random.default_rng(F * 1000 + max_deg)
    num_src = rows + 500
    deg = rng.integers(0, max_deg + 1, size=rows)
    deg[rng.integers(0, rows, size=rows // 10)] = 0
    indptr = np.zeros(rows + 1, dtype=np.int32)
    indptr[1:] = np.cumsum(deg)
    E = int(indptr[-1])
    indices = rng.integers(1, num_src, size=E).astype(np.int32)          # source row 0 is only reached by padding
    weights = rng.uniform(0.5, 40.0, size=E).astype(np.float32)
    x = rng.standard_normal((num_src, F)).astype(np.float32)
    x[0, :] = np.inf
    x[0, ::2] = np.nan
    ref = oracle.aggregate(indptr, indices, weights, x)
    scale = np.zeros((rows, F))
    np.add.at(scale, np.repeat(np.arange(rows), deg), np.abs(weights[:, None].astype(np.float64) * x[indices]))
    scale /= np.maximum(deg, 1)[:, None]
    dev = torch.device("cuda:0")
    ip, ix = _small(n=300)
    gns = GpuGns(ip, ix, None, fanouts=(2,), policies=(U,), cache_size=10, max_seeds=8)      # a context to call through
    try:
        t = {k: torch.from_numpy(v).to(dev) for k, v in dict(indptr=indptr, indices=indices, weights=weights, x=x).items()}
        blk = B.gns_block()
        blk.num_dst, blk.num_src, blk.num_edges = rows, num_src, E
        blk.indptr, blk.indices, blk.weights = t["indptr"].data_ptr(), t["indices"].data_ptr(), t["weights"].data_ptr()
        out = torch.full((rows, F), 7.0, dtype=torch.float32, device=dev)
        B.gns_aggregate(gns.ctx, blk, t["x"], F, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.isfinite(got).all()
        assert (got[deg == 0] == 0).all()
        assert (np.abs(got.astype(np.float64) - ref) <= AGG_RTOL * scale + 1e-30).all()
    finally:
        gns.close()


@pytest.mark.parametrize("policies", [(U, C), (CF, CF)])
def test_unbiased_weight_mode(policies):
    ip, ix = _small()
    n = ip.numel() - 1
    gns = GpuGns(ip, ix, _feat(n, 32), fanouts=(8, 3), policies=policies, cache_size=400, max_seeds=128,
                 wmode=B.GNS_W_UNBIASED)
    try:
        full_parity(gns, cache_seed=4, epoch=2, batch_seed=5, seeds=synth.uniform_seed_batch(n, 128, 9))
    finally:
        gns.close()


def _star_graph(n, hub_degree, extra_avg, seed):
    """A hub joined to `hub_degree` nodes plus a sparse random background, so one
    row spans several LDS segments of the per-row sampler."""
    rng = np.random.default_rng(seed)
    leaves = rng.choice(np.arange(1, n), size=hub_degree, replace=False)
    a = np.concatenate([np.zeros(hub_degree, dtype=np.int64), rng.integers(1, n, size=n * extra_avg // 2)])
    b = np.concatenate([leaves, rng.integers(1, n, size=n * extra_avg // 2)])
    keep = a != b
    a, b = a[keep], b[keep]
    key = np.unique(np.minimum(a, b) * n + np.maximum(a, b))
    a, b = key // n, key % n
    row = np.concatenate([a, b])
    col = np.concatenate([b, a])
    order = np.lexsort((col, row))
    row, col = row[order], col[order]
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(row, minlength=n), out=indptr[1:])
    return torch.from_numpy(indptr), torch.from_numpy(col.astype(np.int32))


@pytest.mark.parametrize("flag_mode", [0, 1])
@pytest.mark.parametrize("policy", [C, CF])
@pytest.mark.parametrize("hub_degree", [1000, 16385, 40000])
def test_hub_row_spanning_many_flag_words(hub_degree, policy, flag_mode):
    n = 60000
    ip, ix = _star_graph(n, hub_degree, 6, hub_degree)
    assert int(ip[1] - ip[0]) == hub_degree
    gns = GpuGns(ip, ix, None, fanouts=(5, 7), policies=(policy, policy), cache_size=3000, max_seeds=16,
                 flag_mode=flag_mode)
    try:
        seeds = torch.tensor([0, 5, 17, 9, 33], dtype=torch.int32)       # the hub is a seed
        full_parity(gns, cache_seed=2, epoch=0, batch_seed=3, seeds=seeds)
        views, ref = full_parity(gns, cache_seed=2, epoch=1, batch_seed=4, seeds=seeds)
        assert ref[0].row_eligible[0] > 7                                 # the hub really drew a subset
    finally:
        gns.close()


def test_rows_with_no_neighbors_and_no_cached_neighbors():
    # nodes 0..9 isolated, the rest a ring; tiny cache -> most rows have N_C = 0
    n = 200
    ring = np.arange(10, n)
    a = ring
    b = np.concatenate([ring[1:], ring[:1]])
    row = np.concatenate([a, b])
    col = np.concatenate([b, a])
    order = np.lexsort((col, row))
    row, col = row[order], col[order]
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(row, minlength=n), out=indptr[1:])
    ip, ix = torch.from_numpy(indptr), torch.from_numpy(col.astype(np.int32))
    gns = GpuGns(ip, ix, _feat(n, 8), fanouts=(2, 2), policies=(U, C), cache_size=3, max_seeds=50)
    try:
        seeds = torch.arange(0, 50, dtype=torch.int32)                   # includes the isolated nodes
        views, ref = full_parity(gns, cache_seed=6, epoch=0, batch_seed=8, seeds=seeds)
        assert (np.diff(ref[1].indptr) == 0).any()
    finally:
        gns.close()


def test_maximum_fanout_and_maximum_depth():
    """The limits of the config: fan-out 64 at every policy, and 8 layers."""
    ip, ix = _small(n=2000, avg=40, seed=13, hub=4)
    n = ip.numel() - 1
    for policies in [(U, C), (CF, CF)]:
        gns = GpuGns(ip, ix, None, fanouts=(64, 64), policies=policies, cache_size=600, max_seeds=24)
        try:
            full_parity(gns, cache_seed=3, epoch=0, batch_seed=14, seeds=synth.uniform_seed_batch(n, 24, 2))
        finally:
            gns.close()
    gns = GpuGns(ip, ix, _feat(n, 8), fanouts=(2, 1, 2, 1, 2, 1, 2, 3), policies=(U, CF, U, CF, U, C, U, C), cache_size=300,
                 max_seeds=16)
    try:
        views, ref = full_parity(gns, cache_seed=5, epoch=1, batch_seed=15, seeds=synth.uniform_seed_batch(n, 16, 3))
        assert len(ref) == 8
    finally:
        gns.close()


def test_single_seed_and_repeatability():
    ip, ix = _small()
    n = ip.numel() - 1
    gns = GpuGns(ip, ix, _feat(n, 16), fanouts=(5, 5), policies=(U, C), cache_size=100, max_seeds=8)
    try:
        seeds = torch.tensor([42], dtype=torch.int32)
        v1, _ = full_parity(gns, cache_seed=1, epoch=0, batch_seed=2, seeds=seeds)
        snap = [{k: (t.clone() if torch.is_tensor(t) else t) for k, t in v.items()} for v in v1]
        v2, _ = full_parity(gns, cache_seed=1, epoch=0, batch_seed=2, seeds=seeds)
        for a, b in zip(snap, v2):
            for k in ("indptr", "indices", "src_nodes", "weights"):
                assert torch.equal(a[k], b[k])
    finally:
        gns.close()


def test_graph_replays_and_eager_launches_agree_with_the_oracle():
    """The batch's launch sequence is captured once per hash-map parity and replayed; with stage timing on
    it is issued kernel by kernel instead.  Replays, eager runs and replays again, with different seeds and
    batch sizes on the same buffers, all against the oracle."""
    ip, ix = _small(n=4000, avg=18, seed=17)
    n = ip.numel() - 1
    gns = GpuGns(ip, ix, _feat(n, 32), fanouts=(7, 5, 4), policies=(CF, U, C), cache_size=350, max_seeds=120)
    try:
        step = 0
        for mode in ("graph", "eager", "graph"):
            if mode == "eager":
                B.gns_profile_begin(gns.ctx, (1 << B.GNS_STAGE_SAMPLE) | (1 << B.GNS_STAGE_GATHER), 64)
            else:
                B.gns_profile_begin(gns.ctx, 0, 0)
            for _ in range(5):                                            # both parities, several times over
                seeds = synth.uniform_seed_batch(n, 120 - 11 * (step % 4), 50 + step)
                full_parity(gns, cache_seed=8, epoch=step // 4, batch_seed=900 + step, seeds=seeds)
                step += 1
            if mode == "eager":
                ms, launches = B.gns_profile_collect(gns.ctx, B.GNS_STAGE_SAMPLE)
                assert launches == 5 and ms > 0
    finally:
        gns.close()


def test_error_paths():
    ip, ix = _small(n=500)
    n = ip.numel() - 1
    gns = GpuGns(ip, ix, None, fanouts=(3, 2), policies=(U, C), cache_size=50, max_seeds=32)
    try:
        seeds = synth.uniform_seed_batch(n, 32, 1).cuda()
        with pytest.raises(B.GnsError) as e:                               # no cache drawn yet
            B.gns_sample_blocks(gns.ctx, 1, seeds, gns.blocks.array)
        assert e.value.status == B.GNS_ESTATE
        B.gns_sample_cache(gns.ctx, 1, 0)
        dup = seeds.clone()
        dup[5] = dup[4]
        with pytest.raises(B.GnsError) as e:
            B.gns_sample_blocks(gns.ctx, 1, dup, gns.blocks.array)
        assert e.value.status == B.GNS_EINVAL
        bad = seeds.clone()
        bad[0] = n
        with pytest.raises(B.GnsError) as e:
            B.gns_sample_blocks(gns.ctx, 1, bad, gns.blocks.array)
        assert e.value.status == B.GNS_EINVAL
        B.gns_sample_blocks(gns.ctx, 1, seeds, gns.blocks.array)          # still healthy afterwards
        ref_cache = oracle.sample_cache(ip.numpy(), 1, 0, 50)
        ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), ref_cache[1], 50, 1, seeds.cpu().numpy(), [3, 2], [U, C])
        compare_blocks([gns.blocks.views(i) for i in range(2)], ref)
        small = gns.blocks.array[1].cap_edges
        gns.blocks.array[1].cap_edges = small - 1
        with pytest.raises(B.GnsError) as e:
            B.gns_sample_blocks(gns.ctx, 1, seeds, gns.blocks.array)
        assert e.value.status == B.GNS_ECAPACITY
        gns.blocks.array[1].cap_edges = small
        with pytest.raises(B.GnsError) as e:                               # too many seeds
            B.gns_sample_blocks(gns.ctx, 1, torch.arange(33, dtype=torch.int32).cuda(), gns.blocks.array)
        assert e.value.status == B.GNS_EINVAL
        with pytest.raises(B.GnsError) as e:                               # no features configured
            B.gns_gather_features(gns.ctx, seeds, 4, torch.empty(4, device="cuda"))
        assert e.value.status == B.GNS_ESTATE
        with pytest.raises(B.GnsError) as e:                               # the config draws the cache by degree
            B.gns_cache_walk_probability(gns.ctx, seeds, 10)
        assert e.value.status == B.GNS_ESTATE
        with pytest.raises(B.GnsError) as e:
            B.gns_cache_probability_view(gns.ctx)
        assert e.value.status == B.GNS_ESTATE
    finally:
        gns.close()


def test_create_rejects_bad_graphs_and_configs():
    ip, ix = _small(n=300)
    n = ip.numel() - 1
    dev = torch.device("cuda:0")

    def create(indptr, indices, fanouts=(2,), policies=(C,), cache_size=10, ws_shrink=0):
        g = B.make_graph(indptr.to(dev), indices.to(dev))
        c = B.make_config(fanouts, policies, cache_size, 8)
        ws = B.alloc_workspace(g, c, dev)
        if ws_shrink:
            ws = ws[:ws.numel() - ws_shrink]
        ctx = B.gns_create(g, c, ws)
        B.gns_destroy(ctx)

    create(ip, ix)
    unsorted = ix.clone()
    b, e = int(ip[7]), int(ip[8])
    assert e - b >= 2
    unsorted[b], unsorted[b + 1] = ix[b + 1], ix[b]
    with pytest.raises(B.GnsError) as err:
        create(ip, unsorted)
    assert err.value.status == B.GNS_EINVAL
    out_of_range = ix.clone()
    out_of_range[3] = n
    with pytest.raises(B.GnsError):
        create(ip, out_of_range)
    bad_ip = ip.clone()
    bad_ip[5] = bad_ip[6] + 1
    with pytest.raises(B.GnsError):
        create(bad_ip, ix)
    with pytest.raises(B.GnsError) as err:                                  # more cache than nodes with neighbors
        create(ip, ix, cache_size=n + 1)
    assert err.value.status == B.GNS_EINVAL
    with pytest.raises(B.GnsError) as err:
        create(ip, ix, policies=(7,))
    assert err.value.status == B.GNS_EINVAL
    with pytest.raises(B.GnsError) as err:
        create(ip, ix, ws_shrink=256)
    assert err.value.status == B.GNS_ECAPACITY


@pytest.mark.parametrize("offsets", [torch.int32, torch.int64])
def test_walk_probability_cache_and_weights(offsets):
    """Section 3.2's random-walk cache probability: the integer weight vector, its prefix, the cache
    drawn from it and the Section 3.4 weights that use it, all against the oracle."""
    ip, ix = _small(n=5000, avg=12, seed=21)
    n = ip.numel() - 1
    train = torch.from_numpy(np.random.default_rng(4).permutation(n)[:150].astype(np.int32))
    fanouts, policies = (6, 4, 3), (CF, CF, C)
    gns = GpuGns(ip.to(offsets), ix, _feat(n, 16), fanouts=fanouts, policies=policies, cache_size=120, max_seeds=64,
                 cache_probability=B.GNS_PROB_WALK)
    try:
        with pytest.raises(B.GnsError) as err:                     # the probability has to be computed first
            B.gns_sample_cache(gns.ctx, 1, 0)
        assert err.value.status == B.GNS_ESTATE
        for scale in (12, 30):
            w, pre, total, support = gns.walk_probability(train, scale)
            w_ref, pre_ref = oracle.walk_weights(ip.numpy(), ix.numpy(), train.numpy(), list(fanouts), scale_log2=scale)
            assert np.array_equal(w, w_ref) and np.array_equal(pre, pre_ref)
            assert total == int(pre_ref[-1]) and support == int(np.count_nonzero(w_ref))
            gns.prob_prefix = pre_ref
            for trial in range(2):
                seeds = train[trial * 64:(trial + 1) * 64]
                full_parity(gns, cache_seed=31, epoch=trial, batch_seed=700 + trial, seeds=seeds)
        with pytest.raises(B.GnsError) as err:                     # 40 bits per node times fan-outs up to 6: too much
            big = GpuGns(ip, ix, None, fanouts=(60, 60, 60, 60, 60, 60, 60, 60), policies=(U,) * 7 + (C,), cache_size=50,
                         max_seeds=8, cache_probability=B.GNS_PROB_WALK)
            try:
                B.gns_cache_walk_probability(big.ctx, torch.arange(0, 200, dtype=torch.int32).cuda(), 40)
            finally:
                big.close()
        assert err.value.status == B.GNS_ECAPACITY
    finally:
        gns.close()


def test_cache_nearly_all_nodes():
    # the cache takes every node that has a neighbor: the stream must run until the rarest node shows up
    ip, ix = _small(n=300, avg=6)
    deg = (ip[1:] - ip[:-1])
    support = int((deg > 0).sum())
    gns = GpuGns(ip, ix, None, fanouts=(2,), policies=(C,), cache_size=support, max_seeds=8)
    try:
        compare_cache(gns.sample_cache(3, 0), oracle.sample_cache(ip.numpy(), 3, 0, support))
    finally:
        gns.close()


def _release_cached_memory():
    """Hand torch's cached device and pinned-host blocks back: the giant workloads need tens of
    GB of each, and blocks cached for an earlier test's shapes would be counted twice."""
    import gc
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch._C._host_emptyCache()


def _config_parity(cfg_id, batches, device_gen="cpu", flag_mode=0, check_features=True, upper=U):
    """Whole path on one of the five workloads against the oracle.  The big graphs are generated
    on the GPU (same recipe) and copied to the host for the oracle."""
    import time
    t0 = time.time()
    _release_cached_memory()
    c = synth.CONFIGS[cfg_id]
    sd = synth.config_seeds(cfg_id)
    g = synth.make_config_graph(cfg_id, device=device_gen)
    indptr, indices = g.indptr.cpu(), g.indices.cpu()
    print("cfg%d: n=%d nnz=%d max_degree=%d (generated in %.1fs)" % (cfg_id, c["n"], g.nnz, g.max_degree, time.time() - t0),
          flush=True)
    del g
    feat = None
    if check_features:
        feat = synth.node_features(c["n"], c["feat"], sd["feat"], device=device_gen, pin=c["feat_on_host"])
        if not c["feat_on_host"]:
            feat = feat.cpu()
    print("cfg%d: features ready after %.1fs" % (cfg_id, time.time() - t0), flush=True)
    cache_size = int(c["n"] * c["cache_frac"])
    L = len(c["fanouts"])
    policies = [upper] * (L - 1) + [C]
    gns = GpuGns(indptr, indices, feat, fanouts=c["fanouts"], policies=policies, cache_size=cache_size,
                 max_seeds=c["batch"], feat_on_host=c["feat_on_host"], flag_mode=flag_mode)
    try:
        epoch = None
        if "split" in c:                      # batches of one shuffled epoch over the training split
            split = synth.training_split(c["n"], c["split"], sd["split"])
            epoch = synth.epoch_batches(split, c["batch"], sd["split"] + 1)
        for b in range(batches):
            if epoch is not None:
                seeds = epoch[-1] if b == batches - 1 else epoch[b]      # the last one is the ragged tail
            else:
                seeds = synth.uniform_seed_batch(c["n"], c["batch"], sd["batch"] + b)
            views, ref = full_parity(gns, cache_seed=sd["cache"], epoch=b, batch_seed=sd["batch"] + b, seeds=seeds)
            print("cfg%d batch %d after %.1fs: rows/src/edges per layer %s" % (
                cfg_id, b, time.time() - t0, [(r.num_dst, r.num_src, r.num_edges) for r in ref]), flush=True)
    finally:
        gns.close()
        del gns, feat, indptr, indices
        _release_cached_memory()


def test_config1_tiny_graph():
    _config_parity(1, batches=3)


@pytest.mark.parametrize("flag_mode", [0, 1])
def test_config2_medium_graph(flag_mode):
    _config_parity(2, batches=2, flag_mode=flag_mode)


@pytest.mark.parametrize("flag_mode", [0, 1])
def test_config2_cache_first_on_the_upper_layers(flag_mode):
    """The paper's experimental setting (Section 4.1): GNS sampling on layers 3 and 2 with fan-outs
    15 and 10, the input layer only from the cache."""
    _config_parity(2, batches=1, flag_mode=flag_mode, upper=CF)


def test_async_pipeline_on_forked_contexts():
    """Three mini-batches in flight on three streams (the created context and two
    forks sharing its cache), no host synchronisation between sampling, gather and
    aggregation (counts stay on the device); every batch must still match the oracle."""
    ip, ix = _small(n=4000, avg=16, seed=11)
    n = ip.numel() - 1
    F = 32
    feat = _feat(n, F, seed=5)
    fanouts, policies, csize, bs = (6, 4, 3), (U, U, C), 250, 96
    gns = GpuGns(ip, ix, feat, fanouts=fanouts, policies=policies, cache_size=csize, max_seeds=bs)
    forks, fork_ws = [], []
    try:
        ref_cache = oracle.sample_cache(ip.numpy(), 21, 3, csize)
        compare_cache(gns.sample_cache(21, 3), ref_cache)
        ctxs = [gns.ctx]
        for _ in range(2):
            ws = torch.empty(B.gns_fork_workspace_bytes(gns.ctx), dtype=torch.uint8, device=gns.device)
            fork_ws.append(ws)
            child = B.gns_fork(gns.ctx, ws)
            forks.append(child)
            ctxs.append(child)
        streams = [torch.cuda.Stream() for _ in ctxs]
        bufs = [B.BlockBuffers(gns.graph, gns.config, gns.device) for _ in ctxs]
        last = len(fanouts) - 1
        xin = [torch.zeros((b.array[last].cap_src, F), dtype=torch.float32, device=gns.device) for b in bufs]
        out = [torch.zeros((b.array[last].cap_dst, F), dtype=torch.float32, device=gns.device) for b in bufs]
        H = 24                                                # the update step rides along, counts on the device too
        gw = torch.Generator().manual_seed(77)
        w_dense = torch.randn((2 * F, H), generator=gw) / np.sqrt(2 * F)
        b_dense = torch.randn(H, generator=gw)
        w_dev, b_dev = w_dense.cuda(), b_dense.cuda()
        z = [torch.zeros((b.array[last].cap_dst, H), dtype=torch.float32, device=gns.device) for b in bufs]
        for rnd in range(2):
            seeds = [synth.uniform_seed_batch(n, bs - 7 * i, 300 + 10 * rnd + i).cuda() for i in range(len(ctxs))]
            torch.cuda.synchronize()
            for i, ctx in enumerate(ctxs):
                with torch.cuda.stream(streams[i]):
                    B.gns_sample_blocks_async(ctx, 900 + 10 * rnd + i, seeds[i], bufs[i].array, streams[i])
                    assert bufs[i].array[last].num_dst == -1 - last
                    B.gns_gather_features(ctx, bufs[i].tensors[last]["src_nodes"], -1, xin[i], streams[i])
                    B.gns_aggregate(ctx, bufs[i].array[last], xin[i], F, out[i], streams[i])
                    B.gns_sage_dense(ctx, xin[i], out[i], w_dev, b_dev, True, z[i], -1 - last, streams[i])
            for i, ctx in enumerate(ctxs):
                B.gns_sample_blocks_wait(ctx, bufs[i].array, streams[i])
            torch.cuda.synchronize()
            for i in range(len(ctxs)):
                ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), ref_cache[1], csize, 900 + 10 * rnd + i,
                                           seeds[i].cpu().numpy(), list(fanouts), list(policies))
                compare_blocks([bufs[i].views(j) for j in range(len(fanouts))], ref)
                x_ref = oracle.gather(feat.numpy(), ref[last].src_nodes)
                assert xin[i][:ref[last].num_src].cpu().numpy().tobytes() == x_ref.tobytes()
                o_ref = oracle.aggregate(ref[last].indptr, ref[last].indices, ref[last].weights, x_ref)
                from gpu_harness import compare_aggregate, aggregate_scale
                compare_aggregate(out[i][:ref[last].num_dst].cpu().numpy(), o_ref, aggregate_scale(ref[last], x_ref))
                # the update step saw the GPU's own aggregate; feed the oracle the same fp32 rows
                nd = ref[last].num_dst
                hs, hn = xin[i][:nd].cpu().numpy(), out[i][:nd].cpu().numpy()
                z_ref = oracle.sage_dense(hs, hn, w_dense.numpy(), b_dense.numpy(), True)
                scale = np.abs(np.concatenate([hs, hn], axis=1).astype(np.float64)) @ np.abs(w_dense.numpy().astype(np.float64)) \
                    + np.abs(b_dense.numpy().astype(np.float64))
                err = np.abs(z[i][:nd].cpu().numpy().astype(np.float64) - z_ref.astype(np.float64))
                assert np.all(err <= (2 * F + 3) * 2.0 ** -24 * scale)
        with pytest.raises(B.GnsError):                       # the cache belongs to the created context
            B.gns_sample_cache(forks[0], 1, 0)
    finally:
        for f in forks:
            B.gns_destroy(f)
        gns.close()


def test_bad_seed_in_an_earlier_batch_is_still_reported():
    """Three mini-batches enqueued before one wait, the first of them with a repeated seed: the wait reports
    it although the last batch was fine; the next wait is clean again."""
    ip, ix = _small(n=2000)
    n = ip.numel() - 1
    gns = GpuGns(ip, ix, None, fanouts=(4, 3), policies=(U, C), cache_size=150, max_seeds=48)
    try:
        B.gns_sample_cache(gns.ctx, 3, 0)
        good = [synth.uniform_seed_batch(n, 48, 70 + i).cuda() for i in range(3)]
        bad = good[0].clone()
        bad[7] = bad[3]
        for sd_, t in ((1, bad), (2, good[1]), (3, good[2])):
            B.gns_sample_blocks_async(gns.ctx, sd_, t, gns.blocks.array)
        with pytest.raises(B.GnsError) as e:
            B.gns_sample_blocks_wait(gns.ctx, gns.blocks.array)
        assert e.value.status == B.GNS_EINVAL
        B.gns_sample_blocks_async(gns.ctx, 4, good[0], gns.blocks.array)
        B.gns_sample_blocks_wait(gns.ctx, gns.blocks.array)
        cache = oracle.sample_cache(ip.numpy(), 3, 0, 150)
        ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], 150, 4, good[0].cpu().numpy(), [4, 3], [U, C])
        compare_blocks([gns.blocks.views(i) for i in range(2)], ref)
    finally:
        gns.close()


def test_walk_probability_recomputed_while_batches_are_in_flight():
    """gns_cache_walk_probability invalidates the cache; mini-batches enqueued before it (on another stream,
    not yet waited for) keep the cache they were enqueued with, and the draw that follows fills the other
    copy of the cache structures instead of the one they read."""
    ip, ix = _small(n=6000, avg=18, seed=31)
    n = ip.numel() - 1
    F = 16
    feat = _feat(n, F, seed=2)
    fanouts, policies, csize, bs = (5, 4), (CF, C), 300, 80
    train = torch.from_numpy(np.random.default_rng(9).permutation(n)[:400].astype(np.int32))
    gns = GpuGns(ip, ix, feat, fanouts=fanouts, policies=policies, cache_size=csize, max_seeds=bs, flag_mode=1,
                 cache_probability=B.GNS_PROB_WALK)
    try:
        work = torch.cuda.Stream()
        nb = 6
        bufs = [B.BlockBuffers(gns.graph, gns.config, gns.device) for _ in range(nb)]
        xin = [torch.zeros((b.array[1].cap_src, F), dtype=torch.float32, device=gns.device) for b in bufs]
        seeds = [train[40 * b:40 * b + bs].contiguous().cuda() for b in range(nb)]
        prefixes = []
        for rnd, scale in enumerate((10, 20)):
            w, pre, total, support = gns.walk_probability(train, scale)     # while the previous pass's batches may still run
            w_ref, pre_ref = oracle.walk_weights(ip.numpy(), ix.numpy(), train.numpy(), list(fanouts), scale_log2=scale)
            assert np.array_equal(pre, pre_ref)
            prefixes.append(pre_ref)
            B.gns_sample_cache(gns.ctx, 12, rnd)
            for b in range(3 * rnd, 3 * rnd + 3):
                B.gns_sample_blocks_async(gns.ctx, 300 + b, seeds[b], bufs[b].array, work)
                B.gns_gather_features(gns.ctx, bufs[b].tensors[1]["src_nodes"], -1, xin[b], work)
        torch.cuda.synchronize()
        for b in range(nb):
            pre_ref = prefixes[b // 3]
            cache = oracle.sample_cache(pre_ref, 12, b // 3, csize)
            ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], csize, 300 + b, seeds[b].cpu().numpy(),
                                       list(fanouts), list(policies), prob_prefix=pre_ref)
            for j, r in enumerate(ref):
                t = bufs[b].tensors[j]
                assert np.array_equal(t["indptr"][:r.num_dst + 1].cpu().numpy(), r.indptr)
                assert np.array_equal(t["indices"][:r.num_edges].cpu().numpy(), r.indices)
                assert np.array_equal(t["src_nodes"][:r.num_src].cpu().numpy(), r.src_nodes)
                gw = t["weights"][:r.num_edges].cpu().numpy().astype(np.float64)
                assert np.all(np.abs(gw - r.weights) <= 1e-5 * np.abs(r.weights))
            x_ref = oracle.gather(feat.numpy(), ref[1].src_nodes)
            assert xin[b][:ref[1].num_src].cpu().numpy().tobytes() == x_ref.tobytes()
    finally:
        gns.close()


def test_cache_refresh_while_batches_are_in_flight():
    """A cache draw fills the copy of the cache structures that is not in use: batches enqueued before it
    (here on two forks, not yet waited for) must come out with the old cache, batches enqueued after it
    with the new one."""
    ip, ix = _small(n=6000, avg=20, seed=19)
    n = ip.numel() - 1
    F = 16
    feat = _feat(n, F, seed=6)
    fanouts, policies, csize, bs = (5, 4), (CF, C), 400, 64
    gns = GpuGns(ip, ix, feat, fanouts=fanouts, policies=policies, cache_size=csize, max_seeds=bs, flag_mode=1)
    forks, keep = [], []
    try:
        caches = [oracle.sample_cache(ip.numpy(), 77, e, csize) for e in range(3)]
        compare_cache(gns.sample_cache(77, 0), caches[0])
        for _ in range(2):
            ws = torch.empty(B.gns_fork_workspace_bytes(gns.ctx), dtype=torch.uint8, device=gns.device)
            keep.append(ws)
            forks.append(B.gns_fork(gns.ctx, ws))
        streams = [torch.cuda.Stream() for _ in forks]
        draw_stream = torch.cuda.Stream()
        bufs = [B.BlockBuffers(gns.graph, gns.config, gns.device) for _ in forks]
        xin = [torch.zeros((b.array[1].cap_src, F), dtype=torch.float32, device=gns.device) for b in bufs]
        for epoch in (1, 2):
            seeds = [synth.uniform_seed_batch(n, bs, 40 + 2 * epoch + i).cuda() for i in range(2)]
            torch.cuda.synchronize()
            for i, f in enumerate(forks):                       # enqueued with the cache of epoch - 1
                B.gns_sample_blocks_async(f, 500 + i, seeds[i], bufs[i].array, streams[i])
                B.gns_gather_features(f, bufs[i].tensors[1]["src_nodes"], -1, xin[i], streams[i])
            B.gns_sample_cache(gns.ctx, 77, epoch, draw_stream)   # overlaps them
            for i, f in enumerate(forks):
                B.gns_sample_blocks_wait(f, bufs[i].array, streams[i])
            torch.cuda.synchronize()
            for i in range(2):
                ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), caches[epoch - 1][1], csize, 500 + i,
                                           seeds[i].cpu().numpy(), list(fanouts), list(policies))
                compare_blocks([bufs[i].views(j) for j in range(2)], ref)
                x_ref = oracle.gather(feat.numpy(), ref[1].src_nodes)
                assert xin[i][:ref[1].num_src].cpu().numpy().tobytes() == x_ref.tobytes()
            nodes_ptr, size, bitmap_ptr, _ = B.gns_cache_view(gns.ctx)
            assert np.array_equal(B.device_view_i32(nodes_ptr, size, gns.device).cpu().numpy(), caches[epoch][0])
            # and a batch enqueued now sees the new cache
            B.gns_sample_blocks(forks[0], 900, seeds[0], bufs[0].array, streams[0])
            ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), caches[epoch][1], csize, 900, seeds[0].cpu().numpy(),
                                       list(fanouts), list(policies))
            compare_blocks([bufs[0].views(j) for j in range(2)], ref)
    finally:
        for f in forks:
            B.gns_destroy(f)
        gns.close()


def test_cache_prepared_ahead_and_activated_later():
    """gns_sample_cache_async fills the copy of the cache structures that is not in use while batches of the
    current cache run; gns_activate_cache switches over.  Nothing here synchronises between the draws, the
    activations and the batches; every batch must match the oracle for the cache of its own period."""
    ip, ix = _small(n=7000, avg=22, seed=29)
    n = ip.numel() - 1
    F = 16
    feat = _feat(n, F, seed=4)
    fanouts, policies, csize, bs = (5, 4), (CF, C), 450, 96
    gns = GpuGns(ip, ix, feat, fanouts=fanouts, policies=policies, cache_size=csize, max_seeds=bs, flag_mode=1)
    try:
        work, draws = torch.cuda.Stream(), torch.cuda.Stream()
        periods, per = 4, 3
        nb = periods * per
        bufs = [B.BlockBuffers(gns.graph, gns.config, gns.device) for _ in range(nb)]
        xin = [torch.zeros((b.array[1].cap_src, F), dtype=torch.float32, device=gns.device) for b in bufs]
        seeds = [synth.uniform_seed_batch(n, bs, 800 + b).cuda() for b in range(nb)]
        with pytest.raises(B.GnsError) as err:                     # nothing drawn yet
            B.gns_activate_cache(gns.ctx)
        assert err.value.status == B.GNS_ESTATE
        torch.cuda.synchronize()
        B.gns_sample_cache_async(gns.ctx, 66, 0, draws)
        for b in range(nb):
            if b % per == 0:
                B.gns_activate_cache(gns.ctx)                      # the cache of period b // per, drawn one period ago
                if b // per + 1 < periods:
                    B.gns_sample_cache_async(gns.ctx, 66, b // per + 1, draws)
            B.gns_sample_blocks_async(gns.ctx, 2000 + b, seeds[b], bufs[b].array, work)
            B.gns_gather_features(gns.ctx, bufs[b].tensors[1]["src_nodes"], -1, xin[b], work)
        torch.cuda.synchronize()
        for b in range(nb):
            cache = oracle.sample_cache(ip.numpy(), 66, b // per, csize)
            ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], csize, 2000 + b, seeds[b].cpu().numpy(),
                                       list(fanouts), list(policies))
            for j, r in enumerate(ref):
                t = bufs[b].tensors[j]
                assert np.array_equal(t["indptr"][:r.num_dst + 1].cpu().numpy(), r.indptr)
                assert np.array_equal(t["indices"][:r.num_edges].cpu().numpy(), r.indices)
                assert np.array_equal(t["src_nodes"][:r.num_src].cpu().numpy(), r.src_nodes)
                gw = t["weights"][:r.num_edges].cpu().numpy().astype(np.float64)
                assert np.all(np.abs(gw - r.weights) <= 1e-5 * np.abs(r.weights))
            x_ref = oracle.gather(feat.numpy(), ref[1].src_nodes)
            assert xin[b][:ref[1].num_src].cpu().numpy().tobytes() == x_ref.tobytes()
        last = oracle.sample_cache(ip.numpy(), 66, periods - 1, csize)
        nodes_ptr, size, _, num_draws = B.gns_cache_view(gns.ctx)   # reads the asynchronous draw's outcome back
        assert np.array_equal(B.device_view_i32(nodes_ptr, size, gns.device).cpu().numpy(), last[0]) and num_draws == last[2]
    finally:
        gns.close()


def test_host_far_ahead_of_the_device_across_cache_refreshes():
    """Many mini-batches and several cache draws enqueued without waiting for any of them, the draws on a
    stream of their own: a draw must not overwrite the copy of the cache structures that batches the device
    has not reached yet still read (the library makes it wait for them on the device)."""
    ip, ix = _small(n=8000, avg=24, seed=23)
    n = ip.numel() - 1
    F = 32
    feat = _feat(n, F, seed=9)
    fanouts, policies, csize, bs = (6, 5), (U, C), 500, 128
    gns = GpuGns(ip, ix, feat, fanouts=fanouts, policies=policies, cache_size=csize, max_seeds=bs, flag_mode=1)
    try:
        work, draws = torch.cuda.Stream(), torch.cuda.Stream()
        nb, period = 24, 3
        bufs = [B.BlockBuffers(gns.graph, gns.config, gns.device) for _ in range(nb)]
        xin = [torch.zeros((b.array[1].cap_src, F), dtype=torch.float32, device=gns.device) for b in bufs]
        seeds = [synth.uniform_seed_batch(n, bs, 600 + b).cuda() for b in range(nb)]
        torch.cuda.synchronize()
        for b in range(nb):
            if b % period == 0:
                B.gns_sample_cache(gns.ctx, 55, b // period, draws)
            B.gns_sample_blocks_async(gns.ctx, 1000 + b, seeds[b], bufs[b].array, work)
            B.gns_gather_features(gns.ctx, bufs[b].tensors[1]["src_nodes"], -1, xin[b], work)
        torch.cuda.synchronize()
        for b in range(nb):
            bufs[b].array[0].num_dst = 0                      # counts were never waited for: take them from the oracle
            cache = oracle.sample_cache(ip.numpy(), 55, b // period, csize)
            ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], csize, 1000 + b, seeds[b].cpu().numpy(),
                                       list(fanouts), list(policies))
            for j, r in enumerate(ref):
                t = bufs[b].tensors[j]
                assert np.array_equal(t["indptr"][:r.num_dst + 1].cpu().numpy(), r.indptr)
                assert np.array_equal(t["indices"][:r.num_edges].cpu().numpy(), r.indices)
                assert np.array_equal(t["src_nodes"][:r.num_src].cpu().numpy(), r.src_nodes)
            x_ref = oracle.gather(feat.numpy(), ref[1].src_nodes)
            assert xin[b][:ref[1].num_src].cpu().numpy().tobytes() == x_ref.tobytes()
    finally:
        gns.close()


def test_config3_products_shaped_graph():
    _config_parity(3, batches=2, device_gen="cuda")


def test_config3_cache_first_per_cache_flags():
    _config_parity(3, batches=1, device_gen="cuda", flag_mode=1, upper=CF, check_features=False)


def test_config3_per_cache_flags_with_features():
    """The benchmark's default mode (one flag per CSR entry, built when the cache is drawn) on the
    products-shaped graph, gather and aggregation included."""
    _config_parity(3, batches=2, device_gen="cuda", flag_mode=1)


def test_config3_input_nodes_of_node_wise_sampling_against_gns():
    """Shape check after the paper's Table 3: on the products-shaped graph plain node-wise sampling (every layer
    UNIFORM) reaches several times more input nodes per mini-batch than GNS in the paper's setting (upper layers
    cache first, input layer from the cache only), a good share of the GNS input nodes are cached, and at the
    input layer the cached share of a row's neighbors, N_C(v)/deg(v), is about the share of all edge endpoints
    that cached nodes own.  The GPU counts are also the oracle's (first batch of every setting)."""
    _release_cached_memory()
    c = synth.CONFIGS[3]
    sd = synth.config_seeds(3)
    g = synth.make_config_graph(3, device="cuda")
    indptr, indices = g.indptr.cpu(), g.indices.cpu()
    del g
    ip, ix = indptr.numpy(), indices.numpy()
    cache_size = int(c["n"] * c["cache_frac"])
    cache_nodes, bitmap, _ = oracle.sample_cache(ip, sd["cache"], 0, cache_size)
    deg = np.diff(ip)
    endpoint_share = deg[cache_nodes].sum() / ip[-1]
    is_cached = np.zeros(c["n"], dtype=bool)
    is_cached[cache_nodes] = True
    batches = 3
    stats = {}
    for name, pol in (("ns", (U, U, U)), ("gns", (CF, CF, C))):
        gns = GpuGns(indptr, indices, None, fanouts=c["fanouts"], policies=pol, cache_size=cache_size,
                     max_seeds=c["batch"], flag_mode=1)
        try:
            if name == "gns":                       # a config with no cache layer has no cache to draw
                gns.sample_cache(sd["cache"], 0)
            inputs = cached = 0
            elig = degs = 0
            for b in range(batches):
                seeds = synth.uniform_seed_batch(c["n"], c["batch"], sd["batch"] + b)
                views = gns.sample_blocks(sd["batch"] + b, seeds)
                v = views[-1]
                src = v["src_nodes"].cpu().numpy()
                inputs += src.size
                cached += int(is_cached[src].sum())
                if name == "gns":
                    rows = v["row_eligible"].numel()
                    elig += int(v["row_eligible"].sum())
                    degs += int(deg[src[:rows]].sum())
                if b == 0:
                    ref = oracle.sample_blocks(ip, ix, bitmap, cache_size, sd["batch"], seeds.numpy(), list(c["fanouts"]),
                                               list(pol))
                    assert [r.num_src for r in ref] == [int(w["src_nodes"].numel()) for w in views]
            stats[name] = (inputs / batches, cached / batches, elig, degs)
        finally:
            gns.close()
            del gns
            _release_cached_memory()
    ns_in, gns_in, gns_cached = stats["ns"][0], stats["gns"][0], stats["gns"][1]
    row_share = stats["gns"][2] / stats["gns"][3]
    print("cfg3 input nodes per mini-batch: NS %.0f, GNS %.0f (%.0f cached); N_C/deg over the input layer's rows %.4f, "
          "cached share of edge endpoints %.4f" % (ns_in, gns_in, gns_cached, row_share, endpoint_share), flush=True)
    # Table 3 reports a factor 4.9 on OGBN-products (3.3 to 7.9 over its datasets): the same order here
    assert 2.0 < ns_in / gns_in < 20.0
    assert gns_cached > 0.1 * gns_in
    assert 0.5 * endpoint_share < row_share < 2.0 * endpoint_share


def test_config2_walk_probability_at_scale():
    """The random-walk cache probability on the medium graph from a 10 % training split: weights and prefix
    bit for bit, then one mini-batch drawn with that cache."""
    c = synth.CONFIGS[2]
    sd = synth.config_seeds(2)
    g = synth.make_config_graph(2)
    ip, ix = g.indptr, g.indices
    train = synth.training_split(c["n"], 100_000, sd["split"])
    gns = GpuGns(ip, ix, None, fanouts=c["fanouts"], policies=(CF, CF, C), cache_size=int(c["n"] * c["cache_frac"]),
                 max_seeds=c["batch"], flag_mode=1, cache_probability=B.GNS_PROB_WALK)
    try:
        w, pre, total, support = gns.walk_probability(train, 24)
        w_ref, pre_ref = oracle.walk_weights(ip.numpy(), ix.numpy(), train.numpy(), list(c["fanouts"]), scale_log2=24)
        assert np.array_equal(w, w_ref) and np.array_equal(pre, pre_ref) and total == int(pre_ref[-1])
        gns.prob_prefix = pre_ref
        full_parity(gns, cache_seed=sd["cache"], epoch=0, batch_seed=sd["batch"], seeds=train[:c["batch"]])
    finally:
        gns.close()


def test_config4_int64_offsets_and_host_features():
    _config_parity(4, batches=1, device_gen="cuda", flag_mode=1)


def test_config5_giant_graph():
    _config_parity(5, batches=2, device_gen="cuda", flag_mode=0)


def test_config5_giant_graph_per_cache_flags():
    """The flag pass over all 1.6 G CSR entries with the cache bitmap in global memory, then mini-batches that
    only read their rows' flag words: the mode the benchmark runs on this workload."""
    _config_parity(5, batches=2, device_gen="cuda", flag_mode=1)


@pytest.mark.parametrize("rows,f1,f2,hdim,relu,use_bias", [(1000, 128, 128, 256, True, True), (1, 4, 8, 12, False, False),
                                                            (129, 100, 128, 132, True, False), (517, 64, 32, 40, False, True)])
def test_sage_dense_update_step(rows, f1, f2, hdim, relu, use_bias):
    """h_u = g(W . (h_u, h_N(u))) on the matrix cores against the fp64 oracle.  fp32 products are
    exact in the fp32 accumulator up to one rounding per addition: K + 1 additions of terms bounded
    by S = sum |a||w| + |b| give an error of at most (K + 2) * 2^-24 * S; the oracle's own final
    rounding adds 2^-24 of the result."""
    ip, ix = _small(n=600)
    gns = GpuGns(ip, ix, None, fanouts=(2,), policies=(U,), cache_size=0, max_seeds=8)
    try:
        g = torch.Generator().manual_seed(rows + hdim)
        hs = torch.randn((rows, f1), generator=g)
        hn = torch.randn((rows, f2), generator=g)
        w = torch.randn((f1 + f2, hdim), generator=g) / np.sqrt(f1 + f2)
        b = torch.randn(hdim, generator=g) if use_bias else None
        out = torch.full((rows, hdim), float("nan"), device=gns.device)
        B.gns_sage_dense(gns.ctx, hs.cuda(), hn.cuda(), w.cuda(), None if b is None else b.cuda(), relu, out, rows)
        torch.cuda.synchronize()
        ref = oracle.sage_dense(hs.numpy(), hn.numpy(), w.numpy(), None if b is None else b.numpy(), relu)
        a = np.concatenate([hs.numpy(), hn.numpy()], axis=1).astype(np.float64)
        scale = np.abs(a) @ np.abs(w.numpy().astype(np.float64)) + (0.0 if b is None else np.abs(b.numpy().astype(np.float64)))
        bound = (f1 + f2 + 3) * 2.0 ** -24 * scale
        err = np.abs(out.cpu().numpy().astype(np.float64) - ref.astype(np.float64))
        assert np.all(err <= bound), float(np.max(err / bound))
        with pytest.raises(B.GnsError):                           # widths must be multiples of 4
            B.gns_sage_dense(gns.ctx, hs.cuda()[:, :f1 - 1].contiguous(), hn.cuda(),
                             w.cuda()[1:].contiguous(), None, relu, out, rows)
    finally:
        gns.close()


def _group_setup(gns, count):
    """count contexts (the created one and forks) with their own block buffers, feature buffers and a GroupCall."""
    ctxs, keep = [gns.ctx], []
    for _ in range(count - 1):
        ws = torch.empty(B.gns_fork_workspace_bytes(gns.ctx), dtype=torch.uint8, device=gns.device)
        keep.append(ws)
        ctxs.append(B.gns_fork(gns.ctx, ws))
    bufs = [gns.blocks] + [B.BlockBuffers(gns.graph, gns.config, gns.device) for _ in range(count - 1)]
    call = B.GroupCall(ctxs, [b.array for b in bufs])
    return ctxs, keep, bufs, call


def _check_group_batch(gns, buf, ref, feat, xin, hout, F):
    from gpu_harness import compare_aggregate, aggregate_scale
    L = len(ref)
    compare_blocks([buf.views(j) for j in range(L)], ref)
    if feat is None:
        return
    last = L - 1
    x_ref = oracle.gather(feat.numpy(), ref[last].src_nodes)
    assert xin[:ref[last].num_src].cpu().numpy().tobytes() == x_ref.tobytes()
    o_ref = oracle.aggregate(ref[last].indptr, ref[last].indices, ref[last].weights, x_ref)
    compare_aggregate(hout[:ref[last].num_dst].cpu().numpy(), o_ref, aggregate_scale(ref[last], x_ref))


@pytest.mark.parametrize("flag_mode", [0, 1])
@pytest.mark.parametrize("count,fanouts,policies", [(8, (6, 4, 3), (U, U, C)), (3, (5, 7), (CF, CF)), (1, (4, 4), (U, C)),
                                                    (5, (20, 3), (U, C))])
def test_group_of_mini_batches_in_one_launch_sequence(count, fanouts, policies, flag_mode):
    """gns_*_group: `count` mini-batches of different sizes per launch sequence, several rounds (both hash-map
    parities, graph replays), a cache refresh in the middle; every batch against the oracle."""
    ip, ix = _small(n=5000, avg=16, seed=37)
    n = ip.numel() - 1
    F = 24
    feat = _feat(n, F, seed=8)
    csize, bs = 300, 90
    gns = GpuGns(ip, ix, feat, fanouts=fanouts, policies=policies, cache_size=csize, max_seeds=bs, flag_mode=flag_mode)
    ctxs, keep, bufs, call = _group_setup(gns, count)
    try:
        L = len(fanouts)
        last = L - 1
        st = torch.cuda.Stream()
        xin = [torch.zeros((b.array[last].cap_src, F), dtype=torch.float32, device=gns.device) for b in bufs]
        hout = [torch.zeros((b.array[last].cap_dst, F), dtype=torch.float32, device=gns.device) for b in bufs]
        for rnd in range(5):
            epoch = rnd // 2
            if rnd % 2 == 0:
                B.gns_sample_cache(gns.ctx, 44, epoch, st)
            cache = oracle.sample_cache(ip.numpy(), 44, epoch, csize)
            seeds = [synth.uniform_seed_batch(n, bs - 11 * ((b + rnd) % 7), 100 * rnd + b).cuda() for b in range(count)]
            bseeds = [7000 + 10 * rnd + b for b in range(count)]
            call.sample(bseeds, seeds, st)
            call.gather([b.tensors[last]["src_nodes"] for b in bufs], [-1] * count, xin, st)
            call.aggregate(last, xin, F, hout, st)
            call.wait(st)
            torch.cuda.synchronize()
            for b in range(count):
                ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], csize, bseeds[b], seeds[b].cpu().numpy(),
                                           list(fanouts), list(policies))
                _check_group_batch(gns, bufs[b], ref, feat, xin[b], hout[b], F)
        # a context of the group used on its own in between, then the group again (parities now differ)
        solo = synth.uniform_seed_batch(n, 33, 999).cuda()
        B.gns_sample_blocks(ctxs[-1], 31337, solo, bufs[-1].array, st)
        ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], csize, 31337, solo.cpu().numpy(), list(fanouts),
                                   list(policies))
        compare_blocks([bufs[-1].views(j) for j in range(L)], ref)
        seeds = [synth.uniform_seed_batch(n, bs, 5000 + b).cuda() for b in range(count)]
        call.sample(list(range(count)), seeds, st)
        call.wait(st)
        for b in range(count):
            ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], csize, b, seeds[b].cpu().numpy(), list(fanouts),
                                       list(policies))
            compare_blocks([bufs[b].views(j) for j in range(L)], ref)
        # a bad seed in one batch of a group is reported by the group's wait
        bad = seeds[count // 2].clone()
        bad[1] = bad[0]
        seeds2 = list(seeds)
        seeds2[count // 2] = bad
        call.sample(list(range(count)), seeds2, st)
        with pytest.raises(B.GnsError) as e:
            call.wait(st)
        assert e.value.status == B.GNS_EINVAL
    finally:
        for f in ctxs[1:]:
            B.gns_destroy(f)
        gns.close()


def test_group_argument_checks():
    ip, ix = _small(n=800)
    n = ip.numel() - 1
    gns = GpuGns(ip, ix, None, fanouts=(3, 2), policies=(U, U), cache_size=0, max_seeds=16)
    other = GpuGns(ip, ix, None, fanouts=(3, 2), policies=(U, U), cache_size=0, max_seeds=16)
    try:
        seeds = synth.uniform_seed_batch(n, 16, 1).cuda()
        twice = B.GroupCall([gns.ctx, gns.ctx], [gns.blocks.array, other.blocks.array])
        with pytest.raises(B.GnsError) as e:
            twice.sample([1, 2], [seeds, seeds])
        assert e.value.status == B.GNS_EINVAL
        strangers = B.GroupCall([gns.ctx, other.ctx], [gns.blocks.array, other.blocks.array])
        with pytest.raises(B.GnsError) as e:
            strangers.sample([1, 2], [seeds, seeds])
        assert e.value.status == B.GNS_EINVAL
    finally:
        other.close()
        gns.close()


def test_config2_pipeline_as_the_benchmark_drives_it():
    """The medium workload driven the way bench.py times it: groups of mini-batches on two streams, device-side
    counts, graph replays, no host synchronisation between batches, a cache refresh in the middle; every
    batch compared with the oracle afterwards (blocks, gathered rows, aggregate)."""
    _release_cached_memory()
    cfg_id = 2
    c = synth.CONFIGS[cfg_id]
    sd = synth.config_seeds(cfg_id)
    g = synth.make_config_graph(cfg_id)
    n, F = c["n"], c["feat"]
    feat = synth.node_features(n, F, sd["feat"])
    fanouts, policies = list(c["fanouts"]), [U, U, C]
    csize = int(n * c["cache_frac"])
    gns = GpuGns(g.indptr, g.indices, feat, fanouts=fanouts, policies=policies, cache_size=csize, max_seeds=c["batch"],
                 flag_mode=1)
    G, S = 4, 2                                       # batches per group, groups in flight
    ctxs, keep, bufs, _ = _group_setup(gns, G * S)
    try:
        calls = [B.GroupCall(ctxs[s * G:(s + 1) * G], [b.array for b in bufs[s * G:(s + 1) * G]]) for s in range(S)]
        streams = [torch.cuda.Stream() for _ in range(S)]
        last = len(fanouts) - 1
        rounds, refresh_at = 3, 2 * G                # 3 rounds of S groups of G batches; a refresh after 8 batches
        nb = rounds * S * G
        seeds = [synth.uniform_seed_batch(n, c["batch"], sd["batch"] + b).cuda() for b in range(nb)]
        # results are copied out of the reused buffers on the batch's own stream right behind the batch
        snap = {}
        xin = [torch.zeros((bufs[i].array[last].cap_src, F), dtype=torch.float32, device=gns.device) for i in range(G * S)]
        hout = [torch.zeros((bufs[i].array[last].cap_dst, F), dtype=torch.float32, device=gns.device) for i in range(G * S)]
        torch.cuda.synchronize()
        b0 = 0
        for rnd in range(rounds):
            for s in range(S):
                ids = list(range(b0, b0 + G))
                if b0 % refresh_at == 0:
                    B.gns_sample_cache(gns.ctx, sd["cache"], b0 // refresh_at, streams[0])
                sl = slice(s * G, (s + 1) * G)
                with torch.cuda.stream(streams[s]):
                    calls[s].sample([sd["batch"] + b for b in ids], [seeds[b] for b in ids], streams[s])
                    calls[s].gather([bf.tensors[last]["src_nodes"] for bf in bufs[sl]], [-1] * G, xin[sl], streams[s])
                    calls[s].aggregate(last, xin[sl], F, hout[sl], streams[s])
                    for k, b in enumerate(ids):
                        i = s * G + k
                        snap[b] = ([{name: t.clone() for name, t in bufs[i].tensors[j].items()} for j in range(last + 1)],
                                   xin[i].clone(), hout[i].clone())
                b0 += G
        torch.cuda.synchronize()
        ip, ix = g.indptr.numpy(), g.indices.numpy()
        from gpu_harness import compare_aggregate, aggregate_scale
        caches = {}
        for b in (0, 1, G, 2 * G, 2 * G + 1, nb - 1):          # first group, across the refresh, the last batch
            epoch = b // refresh_at
            if epoch not in caches:
                caches[epoch] = oracle.sample_cache(ip, sd["cache"], epoch, csize)
            ref = oracle.sample_blocks(ip, ix, caches[epoch][1], csize, sd["batch"] + b, seeds[b].cpu().numpy(), fanouts, policies)
            tens, x, h = snap[b]
            for j, r in enumerate(ref):
                t = tens[j]
                assert np.array_equal(t["indptr"][:r.num_dst + 1].cpu().numpy(), r.indptr), (b, j)
                assert np.array_equal(t["indices"][:r.num_edges].cpu().numpy(), r.indices), (b, j)
                assert np.array_equal(t["src_nodes"][:r.num_src].cpu().numpy(), r.src_nodes), (b, j)
                assert np.array_equal(t["row_eligible"][:r.num_dst].cpu().numpy(), r.row_eligible), (b, j)
                gw = t["weights"][:r.num_edges].cpu().numpy().astype(np.float64)
                assert np.all(np.abs(gw - r.weights) <= 1e-5 * np.abs(r.weights)), (b, j)
            x_ref = oracle.gather(feat.numpy(), ref[last].src_nodes)
            assert x[:ref[last].num_src].cpu().numpy().tobytes() == x_ref.tobytes(), b
            o_ref = oracle.aggregate(ref[last].indptr, ref[last].indices, ref[last].weights, x_ref)
            compare_aggregate(h[:ref[last].num_dst].cpu().numpy(), o_ref, aggregate_scale(ref[last], x_ref))
    finally:
        for f in ctxs[1:]:
            B.gns_destroy(f)
        gns.close()
        _release_cached_memory()


@pytest.mark.parametrize("fanouts,policies,flag_mode", [((6, 4, 3), (U, U, C), 1), ((5, 7), (CF, CF), 0), ((20, 5), (U, C), 0)])
def test_mark_bitmap_summary_on_a_small_graph(fanouts, policies, flag_mode, monkeypatch):
    """Graphs with millions of nodes keep a summary of the frontier mark bitmap (one bit per word) so that the
    union step only reads words that carry marks.  Forced here on a small graph whose bitmap spans several
    summary words and tiles; group launches and repeated batches check that both levels are left clean."""
    monkeypatch.setenv("GNS_MARK_SUMMARY_MIN_WORDS", "1")
    ip, ix = _small(n=20000, avg=10, seed=43)
    n = ip.numel() - 1
    F = 8
    feat = _feat(n, F, seed=3)
    csize, bs, count = 500, 70, 3
    gns = GpuGns(ip, ix, feat, fanouts=fanouts, policies=policies, cache_size=csize, max_seeds=bs, flag_mode=flag_mode)
    ctxs, keep, bufs, call = _group_setup(gns, count)
    try:
        L = len(fanouts)
        last = L - 1
        cache = oracle.sample_cache(ip.numpy(), 4, 0, csize)
        B.gns_sample_cache(gns.ctx, 4, 0)
        xin = [torch.zeros((b.array[last].cap_src, F), dtype=torch.float32, device=gns.device) for b in bufs]
        hout = [torch.zeros((b.array[last].cap_dst, F), dtype=torch.float32, device=gns.device) for b in bufs]
        for rnd in range(3):
            seeds = [synth.uniform_seed_batch(n, bs - 9 * b, 40 * rnd + b).cuda() for b in range(count)]
            bseeds = [600 + 10 * rnd + b for b in range(count)]
            call.sample(bseeds, seeds)
            call.gather([b.tensors[last]["src_nodes"] for b in bufs], [-1] * count, xin)
            call.aggregate(last, xin, F, hout)
            call.wait()
            torch.cuda.synchronize()
            for b in range(count):
                ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], csize, bseeds[b], seeds[b].cpu().numpy(),
                                           list(fanouts), list(policies))
                _check_group_batch(gns, bufs[b], ref, feat, xin[b], hout[b], F)
    finally:
        for f in ctxs[1:]:
            B.gns_destroy(f)
        gns.close()


@pytest.mark.parametrize("env", [{"GNS_LANE_ROWS_MIN": "1"}, {"GNS_NO_LANE_SAMPLER": "1"}, {"GNS_NO_GRAPH": "1"}])
@pytest.mark.parametrize("fanouts,policies,flag_mode", [((15, 10, 5), (U, U, U), 0), ((16, 8), (U, C), 1), ((4, 10, 3), (U, U, C), 1),
                                                        ((6, 5), (CF, C), 1)])
def test_sampler_kernel_choices_give_the_same_blocks(env, fanouts, policies, flag_mode, monkeypatch):
    """Which sampler kernel serves a layer is a matter of size: one row per lane for large UNIFORM launches and
    for CACHE_ONLY on the induced subgraph, a lane group per row otherwise, flag words where there is no induced
    subgraph; launches replayed from a captured graph or enqueued one by one.  Each choice forced here on a small
    graph (the switches are the library's testing aids), in groups of three mini-batches, against the oracle."""
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    ip, ix = _small(n=20000, avg=12, seed=61)
    n = ip.numel() - 1
    F = 8
    feat = _feat(n, F, seed=6)
    csize, bs, count = 2000, 80, 3
    gns = GpuGns(ip, ix, feat, fanouts=fanouts, policies=policies, cache_size=csize, max_seeds=bs, flag_mode=flag_mode)
    ctxs, keep, bufs, call = _group_setup(gns, count)
    try:
        last = len(fanouts) - 1
        uses_cache = any(p != U for p in policies)
        cache = oracle.sample_cache(ip.numpy(), 4, 0, csize)
        if uses_cache:
            B.gns_sample_cache(gns.ctx, 4, 0)
        xin = [torch.zeros((b.array[last].cap_src, F), dtype=torch.float32, device=gns.device) for b in bufs]
        hout = [torch.zeros((b.array[last].cap_dst, F), dtype=torch.float32, device=gns.device) for b in bufs]
        for rnd in range(2):
            seeds = [synth.uniform_seed_batch(n, bs - 13 * b, 60 * rnd + b).cuda() for b in range(count)]
            bseeds = [900 + 10 * rnd + b for b in range(count)]
            call.sample(bseeds, seeds)
            call.gather([b.tensors[last]["src_nodes"] for b in bufs], [-1] * count, xin)
            call.aggregate(last, xin, F, hout)
            call.wait()
            torch.cuda.synchronize()
            for b in range(count):
                ref = oracle.sample_blocks(ip.numpy(), ix.numpy(), cache[1], csize, bseeds[b], seeds[b].cpu().numpy(),
                                           list(fanouts), list(policies))
                _check_group_batch(gns, bufs[b], ref, feat, xin[b], hout[b], F)
    finally:
        for f in ctxs[1:]:
            B.gns_destroy(f)
        gns.close()


@pytest.mark.parametrize("summary", [False, True])
def test_union_step_with_large_tiles_and_several_lds_passes(summary, monkeypatch):
    """The union step walks the frontier mark bitmap in tiles of up to 8192 words and passes a tile's marked
    words through LDS 1024 at a time.  Forced here: one tile of 4096 words over a 300 K-node graph, and a batch
    whose new nodes mark nearly every word of it (several passes), with and without the bitmap's summary."""
    monkeypatch.setenv("GNS_MARK_TILE_WORDS", "4096")
    monkeypatch.setenv("GNS_MARK_SUMMARY_MIN_WORDS", "1" if summary else "1000000000")
    ip, ix = random_symmetric_csr(300000, 8, np.random.default_rng(47))
    ip, ix = torch.from_numpy(ip), torch.from_numpy(ix)
    n = ip.numel() - 1
    gns = GpuGns(ip, ix, None, fanouts=(12, 6), policies=(U, CF), cache_size=3000, max_seeds=3000, flag_mode=1)
    try:
        for trial in range(2):
            seeds = synth.uniform_seed_batch(n, 3000 - 500 * trial, 70 + trial)
            views, ref = full_parity(gns, cache_seed=5, epoch=trial, batch_seed=80 + trial, seeds=seeds)
            assert ref[1].num_src - ref[1].num_dst > 40000          # new nodes of the input layer: most words marked
    finally:
        gns.close()


def test_directed_adjacency():
    """Nothing in the path assumes a symmetric adjacency (deg(i) is the row length, the cache draw takes the
    owner row of a uniform entry): the symmetric graph and a directed thinning of it, both against the oracle."""
    ip, ix = _small(n=4000, avg=16, seed=53)
    n = ip.numel() - 1
    rng = np.random.default_rng(3)
    keep = rng.random(ix.numel()) < 0.7                                   # drop 30 % of the entries, one direction at a time
    row = np.repeat(np.arange(n), np.diff(ip.numpy()))
    ip_d = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(row[keep], minlength=n), out=ip_d[1:])
    ix_d = ix.numpy()[keep]
    for indptr, indices in ((ip, ix), (torch.from_numpy(ip_d), torch.from_numpy(ix_d))):
        gns = GpuGns(indptr, indices, _feat(n, 16), fanouts=(6, 5), policies=(CF, C), cache_size=300, max_seeds=100,
                     flag_mode=1)
        try:
            for trial in range(2):
                seeds = synth.uniform_seed_batch(n, 100 - 30 * trial, 11 + trial)
                full_parity(gns, cache_seed=14, epoch=trial, batch_seed=15 + trial, seeds=seeds)
        finally:
            gns.close()
