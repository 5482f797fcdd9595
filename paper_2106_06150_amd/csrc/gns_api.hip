// C ABI of the GNS library: argument validation, workspace layout and the
// per-call launch sequences.  See include/gns.h for the contract.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <new>
#include "gns_internal.h"
#include "gns_kernels.hpp"

namespace gns {

static thread_local char g_create_err[256] = "";

static inline size_t align_up(size_t x) { return (x + 255u) & ~(size_t) 255u; }

static inline uint32_t pow2_at_least(uint64_t x)
{
    uint64_t p = 1024;
    while (p < x) p <<= 1;
    return (uint32_t) p;
}

static bool config_uses_cache(const gns_config* cfg)
{
    for (int i = 0; i < cfg->num_layers; ++i)
        if (cfg->policy[i] != GNS_UNIFORM) return true;
    return false;
}

bool compute_layout(const gns_graph* g, const gns_config* cfg, Layout* out, char* err, size_t errlen)
{
#define GNS_BAD(msg) do { snprintf(err, errlen, "%s", msg); return false; } while (0)
    if (!g || !cfg) GNS_BAD("null graph or config");
    if (g->num_nodes < 1 || g->num_nodes >= (int64_t) 1 << 31) GNS_BAD("num_nodes must be in [1, 2^31)");
    if (g->num_entries < 1) GNS_BAD("num_entries must be >= 1");
    if (!g->indptr || !g->indices) GNS_BAD("null CSR arrays");
    if (!g->indptr_is_i64 && g->num_entries >= (int64_t) 1 << 31) GNS_BAD("int32 offsets cannot address num_entries");
    if (g->feat_dim < 0) GNS_BAD("feat_dim must be >= 0");
    if (g->feat_dim > 0 && !g->feat_dev && !g->feat_host_pinned) GNS_BAD("feat_dim > 0 but no feature store given");
    if (cfg->num_layers < 1 || cfg->num_layers > GNS_MAX_LAYERS) GNS_BAD("num_layers out of range");
    if (cfg->max_seeds < 1) GNS_BAD("max_seeds must be >= 1");
    if (cfg->wmode != GNS_W_PRINTED && cfg->wmode != GNS_W_UNBIASED) GNS_BAD("unknown weight mode");
    if (cfg->flag_mode != GNS_FLAGS_PER_BATCH && cfg->flag_mode != GNS_FLAGS_PER_CACHE) GNS_BAD("unknown flag mode");
    if (cfg->cache_probability != GNS_PROB_DEGREE && cfg->cache_probability != GNS_PROB_WALK)
        GNS_BAD("unknown cache_probability");
    for (int i = 0; i < cfg->num_layers; ++i) {
        if (cfg->fanout[i] < 1 || cfg->fanout[i] > GNS_MAX_FANOUT) GNS_BAD("fanout out of range");
        if (cfg->policy[i] != GNS_UNIFORM && cfg->policy[i] != GNS_CACHE_ONLY && cfg->policy[i] != GNS_CACHE_FIRST)
            GNS_BAD("unknown policy");
    }
    const bool uses_cache = config_uses_cache(cfg);
    if (uses_cache && (cfg->cache_size < 1 || cfg->cache_size > g->num_nodes)) GNS_BAD("cache_size out of range");
    if (!uses_cache && cfg->cache_size < 0) GNS_BAD("cache_size must be >= 0");

    Layout L;
    memset(&L, 0, sizeof(L));
    const int64_t n = g->num_nodes;
    const int64_t C = uses_cache ? cfg->cache_size : 0;
    L.words = (n + 63) / 64;
    L.word_tiles = (L.words + kTile - 1) / kTile;
    L.mark_tile_words = kMarkTileMin;
    // about a hundred tiles per mini-batch (measured best on the 1 M-, 2.4 M- and 111 M-node graphs: more tiles mean
    // more blocks that each add up the tile sums before them, fewer mean more new nodes per thread, one after the other)
    while (L.mark_tile_words < kMarkTileMax && L.words / L.mark_tile_words > 128) L.mark_tile_words *= 2;
    if (const char* e = getenv("GNS_MARK_TILE_WORDS")) {           // testing aid: a power of two in [64, kMarkTileMax]
        const int t = atoi(e);
        if (t >= kMarkTileMin && t <= kMarkTileMax && (t & (t - 1)) == 0) L.mark_tile_words = t;
    }
    L.mark_tiles = (L.words + L.mark_tile_words - 1) / L.mark_tile_words;

    // worst-case frontier growth: rows[i+1] = min(rows[i] * (1 + k_i), n)
    L.rows[0] = cfg->max_seeds;
    L.max_rows = 0;
    L.max_edges = 0;
    for (int i = 0; i < cfg->num_layers; ++i) {
        L.edges[i] = L.rows[i] * cfg->fanout[i];
        int64_t src = L.rows[i] + L.edges[i];
        if (src > n) src = n;
        L.rows[i + 1] = src;
        if (L.rows[i] > L.max_rows) L.max_rows = L.rows[i];
        if (L.edges[i] > L.max_edges) L.max_edges = L.edges[i];
        if (L.edges[i] >= (int64_t) 1 << 31) GNS_BAD("a layer's worst-case edge count exceeds 2^31");
    }
    L.row_tiles = (L.max_rows + kTile - 1) / kTile;
    // the batch hash map addresses its slots with 32 bits at a load factor of at most 1/2
    if (2 * (uint64_t) L.rows[cfg->num_layers] > (uint64_t) 1 << 31) GNS_BAD("worst-case frontier too large for the batch hash map (more than 2^30 nodes)");
    L.hash_cap = pow2_at_least(2 * (uint64_t) L.rows[cfg->num_layers]);

    L.draw_chunk = C;
    if (L.draw_chunk < 65536) L.draw_chunk = 65536;
    if (L.draw_chunk > (int64_t) 1 << 22) L.draw_chunk = (int64_t) 1 << 22;
    L.draw_tiles = (L.draw_chunk + kTile - 1) / kTile;
    L.draw_hash_cap = pow2_at_least(2 * (uint64_t) (C + L.draw_chunk));

    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    // per-batch scratch (every forked context has its own copy of these sections)
    L.state = take(sizeof(DeviceState) + 64);
    L.mark_bitmap = take((size_t) L.words * 8);
    // A graph with millions of nodes gets a summary of the mark bitmap (one bit per word), so that the union
    // step reads the words that carry marks instead of walking n / 8 bytes per layer.
    {
        int64_t min_words = 65536;
        if (const char* e = getenv("GNS_MARK_SUMMARY_MIN_WORDS")) min_words = atoll(e);
        L.summary_words = L.words >= min_words ? (L.words + 63) / 64 : 0;
        L.mark_summary = take((size_t) (L.summary_words > 0 ? L.summary_words : 1) * 8);
    }
    L.seed_copy = take((size_t) cfg->max_seeds * 4);
    L.row_ext = take((size_t) L.rows[cfg->num_layers] * 16);
    L.hub_rows = take((size_t) L.rows[cfg->num_layers] * 4);
    L.slot_list[0] = take((size_t) L.rows[cfg->num_layers] * 4);
    L.slot_list[1] = take((size_t) L.rows[cfg->num_layers] * 4);
    L.hash_slots[0] = take((size_t) L.hash_cap * 8);
    L.hash_slots[1] = take((size_t) L.hash_cap * 8);
    for (int par = 0; par < 2; ++par) {
        L.s_nbr[par] = take((size_t) L.max_edges * 4);
        L.s_w[par] = take((size_t) L.max_edges * 4);
        L.s_cnt[par] = take((size_t) L.max_rows * 4);
    }
    L.sums_rows = take((size_t) (L.row_tiles + 1) * 4);
    const int64_t word_or_draw_tiles = L.word_tiles > L.draw_tiles ? L.word_tiles : L.draw_tiles;
    L.sums_words = take((size_t) (word_or_draw_tiles + 1) * 4);
    L.sums_marks = take((size_t) (L.mark_tiles + 1) * 4);
    L.sums_plan = take((size_t) (L.max_rows / kBlock + 2) * 4);
    if (uses_cache) {
        // a dst row of deg entries touches at most deg/64 + 2 aligned chunks; dst rows are distinct
        L.max_chunks = g->num_entries / 64 + 2 * L.max_rows + 64;
        if (L.max_chunks >= (int64_t) 1 << 31) GNS_BAD("graph too large for 32-bit chunk ids");
        L.plan_cnt = take((size_t) L.max_rows * 4);
        L.plan_g0 = take((size_t) L.max_rows * 4);
        L.plan_desc = take((size_t) L.max_chunks * 4);
    }
    // shared: the cache and everything that is a pure function of (graph, cache)
    L.shared_begin = off;
    if (uses_cache) {
        L.draw_keys = take((size_t) L.draw_hash_cap * 4);
        L.draw_vals = take((size_t) L.draw_hash_cap * 4);
        L.draw_node = take((size_t) L.draw_chunk * 4);
        L.draw_slot = take((size_t) L.draw_chunk * 4);
        if (cfg->cache_probability == GNS_PROB_WALK) {
            L.walk_a = take((size_t) n * 8);
            L.walk_b = take((size_t) n * 8);
            L.prob_prefix = take((size_t) (n + 1) * 8);
            const size_t tiles = (size_t) ((n + kTile - 1) / kTile);
            L.walk_tiles = take((tiles + 1) * 8);
            L.walk_tiles_nz = take((tiles + 1) * 4);
        }
    }
    if (uses_cache && cfg->flag_mode == GNS_FLAGS_PER_CACHE) {
        if (g->num_entries >= (int64_t) 1 << 32) GNS_BAD("GNS_FLAGS_PER_CACHE counts cached entries in 32 bits: num_entries must be < 2^32");
        L.chunk_tiles = (g->num_entries / 64 + 1 + kTile - 1) / kTile;
        L.sums_chunks = take((size_t) (L.chunk_tiles + 1) * 4);
    }
    // The cache block: everything a cache draw writes and the mini-batches read.  There are two copies
    // (generations): a draw fills the one that is not in use, so it can run while batches that were
    // enqueued before it still read the other.
    L.cache_block_begin = off;
    L.cache_bitmap = take((size_t) L.words * 8);
    L.cache_prefix = take((size_t) L.words * 4);
    // A cache bitmap too big for LDS gets a coarse companion that does fit: one bit per 2^shift ids.  With a
    // cache of about 1 % of the nodes it answers "not cached" for most entries without leaving the CU as long as
    // the groups stay small.
    L.coarse_shift = 0;
    L.coarse_words = 0;
    L.coarse_bitmap = 0;
    if (uses_cache && (size_t) L.words * 8 > kLdsBitmapBytes) {
        int sh = 1;
        while (sh <= 4 && (size_t) (((n >> sh) + 63) / 64 + 1) * 8 > kLdsBitmapBytes) ++sh;
        // Too big for LDS even at one bit per 16 ids: the coarse bitmap then stays in global memory, where it
        // is small enough for every XCD's L2 (n / 128 bytes at one bit per 16 ids), and still spares most entries
        // the read of the exact bitmap, which costs a 64-byte fetch over the fabric each time.
        if (sh > 4) {
            sh = 4;
            if (const char* e = getenv("GNS_COARSE_SHIFT")) { const int v = atoi(e); if (v >= 1 && v <= 6) sh = v; }
        }
        L.coarse_shift = sh;
        L.coarse_words = ((n >> sh) + 63) / 64 + 1;
        L.coarse_bitmap = take((size_t) (L.coarse_words + 1) * 8);
    }
    L.cache_nodes = take((size_t) (C > 0 ? C : 1) * 4);
    L.cache_feat = take((size_t) (C > 0 ? C : 1) * (size_t) (g->feat_dim > 0 ? g->feat_dim : 1) * 4);
    if (uses_cache) {
        L.edge_flags = take((size_t) (g->num_entries / 64 + 1) * 8);
        L.node_pc = take((size_t) n * 4);
        if (cfg->flag_mode == GNS_FLAGS_PER_CACHE) {
            L.srec = take((size_t) (g->num_entries / 64 + 2) * 16);
            L.s_nodes = take((size_t) g->num_entries * 4);
        }
    }
    L.cache_block_bytes = off - L.cache_block_begin;
    if (uses_cache) off += L.cache_block_bytes;            // the second generation
    L.total = off;
    *out = L;
    return true;
#undef GNS_BAD
}

gns_status ctx_fail(gns_ctx* c, gns_status st, const char* what, hipError_t e)
{
    if (e != hipSuccess) snprintf(c->err, sizeof(c->err), "%s: %s", what, hipGetErrorString(e));
    else snprintf(c->err, sizeof(c->err), "%s", what);
    return st;
}

}  // namespace gns

using namespace gns;

// Every launch of one mini-batch, in order, on stream s (also the body that is captured).
namespace gns {
// Every launch of one group of mini-batches, in order, on stream s (also the body that is captured).
gns_status enqueue_batch(const Group& g, const BeginDyn& d, hipStream_t s)
{
    gns_ctx* c = g.ctx[0];
    const int nl = c->config.num_layers;
    hipError_t e = launch_batch_begin(g, d, s);
    if (e != hipSuccess) return ctx_fail(c, GNS_EHIP, "batch begin", e);
    // the batch's kernels read the seeds from the context's own copy (made by the first kernel), so
    // the captured launch sequence does not depend on where the caller keeps them
    for (int i = 0; i < nl; ++i) {
        {
            StageTimer t(c, GNS_STAGE_SAMPLE + i, s);
            e = launch_sample_layer(g, i, s);
        }
        if (e != hipSuccess) return ctx_fail(c, GNS_EHIP, "sample layer", e);
        {
            StageTimer t(c, GNS_STAGE_FINISH + i, s);
            e = launch_finish_layer(g, i, s);
            if (e == hipSuccess && i == nl - 1) e = launch_relabel(g, i, s);
        }
        if (e != hipSuccess) return ctx_fail(c, GNS_EHIP, "finish layer", e);
    }
    return GNS_OK;
}

// The first kernel's per-call arguments: seeds, Philox keys, batch ids, and for every batch which hash map
// it uses and which copy of the cache structures it reads (the current one).
void fill_begin_dyn(const Group& g, const uint64_t* seeds, const int32_t* const* seeds_dev, const int32_t* num_seeds,
                    BeginDyn* out)
{
    memset(out, 0, sizeof(*out));
    for (int b = 0; b < g.count; ++b) {
        gns_ctx* c = g.ctx[b];
        out->seeds[b] = seeds_dev[b];
        out->num_seeds[b] = num_seeds[b];
        out->key0[b] = (uint32_t) seeds[b];
        out->key1[b] = (uint32_t) (seeds[b] >> 32);
        out->batch_id[b] = c->batch_id + 1;
        out->parity[b] = c->hash_parity;
        out->cache_gen[b] = active_gen(c);
    }
}

// Host-side checks of one mini-batch's arguments (no device work).
gns_status check_batch_args(gns_ctx* c, const int32_t* seeds_dev, int32_t num_seeds, const gns_block* blocks)
{
    if (!seeds_dev || !blocks) return ctx_fail(c, GNS_EINVAL, "null seeds or blocks");
    if (num_seeds < 1 || num_seeds > c->config.max_seeds) return ctx_fail(c, GNS_EINVAL, "num_seeds out of range");
    if (c->uses_cache && !c->root->cache_valid) return ctx_fail(c, GNS_ESTATE, "gns_sample_cache must run before gns_sample_blocks");
    const Layout& L = c->lay;
    for (int i = 0; i < c->config.num_layers; ++i) {
        const gns_block* b = &blocks[i];
        if (!b->indptr || !b->indices || !b->src_nodes || !b->row_eligible || !b->weights)
            return ctx_fail(c, GNS_EINVAL, "a block has a null buffer");
        if (b->cap_dst < L.rows[i] || b->cap_src < L.rows[i + 1] || b->cap_edges < L.edges[i]) {
            snprintf(c->err, sizeof(c->err), "block %d too small: need cap_dst %lld cap_src %lld cap_edges %lld", i,
                     (long long) L.rows[i], (long long) L.rows[i + 1], (long long) L.edges[i]);
            return GNS_ECAPACITY;
        }
    }
    return GNS_OK;
}
}  // namespace gns

static hipError_t events_create(gns_ctx* c)
{
    memset(c->gen_event, 0, sizeof(c->gen_event));
    c->ready_event[0] = c->ready_event[1] = nullptr;
    c->pending = false;
    c->cache_version = 0;
    c->seen_version = 0;
    c->gen_event_used[0] = c->gen_event_used[1] = 0;
    c->reader_stream_count = 0;
    hipError_t e = hipSuccess;
    for (int g = 0; g < 2; ++g)
        for (int i = 0; i < kReaderStreams && e == hipSuccess; ++i)
            e = hipEventCreateWithFlags(&c->gen_event[g][i], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ready_event[0], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ready_event[1], hipEventDisableTiming);
    return e;
}

static void events_destroy(gns_ctx* c)
{
    for (int g = 0; g < 2; ++g)
    {
        for (int i = 0; i < kReaderStreams; ++i)
            if (c->gen_event[g][i]) { (void) hipEventDestroy(c->gen_event[g][i]); c->gen_event[g][i] = nullptr; }
        if (c->ready_event[g]) { (void) hipEventDestroy(c->ready_event[g]); c->ready_event[g] = nullptr; }
    }
}

static void graph_release(BatchGraph& g)
{
    if (g.exec) (void) hipGraphExecDestroy(g.exec);
    if (g.graph) (void) hipGraphDestroy(g.graph);
    g.exec = nullptr;
    g.graph = nullptr;
    g.first = nullptr;
    g.valid = false;
}

// A group's launch sequence does not depend on the data (grids are sized for the worst case; counts, the
// hash-map parity and the cache generation stay on the device), so it is captured once per set of contexts
// and caller block buffers and replayed with hipGraphLaunch; only the first kernel's arguments (seeds
// pointers, seeds, seed counts, batch ids, parities, cache generation) change between replays.  The graphs
// are kept by the group's first context.
static gns_status launch_batch_graph(const Group& grp, const BeginDyn& dyn, hipStream_t s)
{
    gns_ctx* c = grp.ctx[0];
    const int nl = c->config.num_layers;
    BatchGraph* hit = nullptr;
    BatchGraph* victim = &c->bg[0];
    for (int k = 0; k < kGraphsPerContext; ++k) {
        BatchGraph& g = c->bg[k];
        if (!g.valid) { victim = &g; continue; }
        bool same = g.count == grp.count;
        for (int b = 0; same && b < grp.count; ++b) {
            same = g.ctx[b] == grp.ctx[b];
            for (int i = 0; same && i < nl; ++i) {
                const gns_block& x = g.blocks[b][i];
                const gns_block& y = grp.blocks[b][i];
                same = x.indptr == y.indptr && x.indices == y.indices && x.src_nodes == y.src_nodes &&
                       x.row_eligible == y.row_eligible && x.weights == y.weights;
            }
        }
        if (same) { hit = &g; break; }
        if (victim->valid && g.last_use < victim->last_use) victim = &g;
    }
    hipError_t e;
    if (!hit) {
        BatchGraph& g = *victim;
        graph_release(g);
        e = hipStreamBeginCapture(c->cap_stream, hipStreamCaptureModeRelaxed);
        if (e != hipSuccess) return ctx_fail(c, GNS_EHIP, "begin capture", e);
        const gns_status st = enqueue_batch(grp, dyn, c->cap_stream);
        e = hipStreamEndCapture(c->cap_stream, &g.graph);
        if (st != GNS_OK) { graph_release(g); return st; }
        if (e != hipSuccess) { graph_release(g); return ctx_fail(c, GNS_EHIP, "end capture", e); }
        e = hipGraphInstantiate(&g.exec, g.graph, nullptr, nullptr, 0);
        if (e != hipSuccess) { graph_release(g); return ctx_fail(c, GNS_EHIP, "graph instantiate", e); }
        // find the first kernel's node
        size_t count = 0;
        e = hipGraphGetNodes(g.graph, nullptr, &count);
        if (e != hipSuccess || count == 0 || count > 256) { graph_release(g); return ctx_fail(c, GNS_EHIP, "graph nodes", e); }
        hipGraphNode_t nodes[256];
        e = hipGraphGetNodes(g.graph, nodes, &count);
        if (e != hipSuccess) { graph_release(g); return ctx_fail(c, GNS_EHIP, "graph nodes", e); }
        for (size_t i = 0; i < count && !g.first; ++i) {
            hipGraphNodeType type;
            if (hipGraphNodeGetType(nodes[i], &type) != hipSuccess || type != hipGraphNodeTypeKernel) continue;
            hipKernelNodeParams kp;
            if (hipGraphKernelNodeGetParams(nodes[i], &kp) != hipSuccess) continue;
            if (kp.func == batch_first_kernel()) g.first = nodes[i];
        }
        if (!g.first) { graph_release(g); return ctx_fail(c, GNS_EHIP, "first kernel node not found in the captured graph"); }
        g.count = grp.count;
        for (int b = 0; b < grp.count; ++b) {
            g.ctx[b] = grp.ctx[b];
            for (int i = 0; i < nl; ++i) g.blocks[b][i] = grp.blocks[b][i];
        }
        // the first kernel's fixed argument block: the same for every replay of this graph
        static_assert(sizeof(LayerArgs) <= sizeof(g.args.fixed), "BeginArgsHost::fixed too small");
        static_assert(sizeof(BeginDyn) <= sizeof(g.args.dyn), "BeginArgsHost::dyn too small");
        LayerArgs* fixed = reinterpret_cast<LayerArgs*>(g.args.fixed);
        fill_group_args(grp, fixed);
        fill_finish_template(c, 0, &fixed->f);
        g.valid = true;
        hit = &g;
    }
    BatchGraph& g = *hit;
    g.last_use = ++c->graph_clock;
    // new scalars for this group of batches
    hipKernelNodeParams kp;
    e = hipGraphKernelNodeGetParams(g.first, &kp);
    if (e != hipSuccess) return ctx_fail(c, GNS_EHIP, "get first kernel params", e);
    memcpy(g.args.dyn, &dyn, sizeof(dyn));
    g.arg_ptrs[0] = g.args.fixed;
    g.arg_ptrs[1] = g.args.dyn;
    kp.kernelParams = g.arg_ptrs;
    kp.extra = nullptr;
    e = hipGraphExecKernelNodeSetParams(g.exec, g.first, &kp);
    if (e != hipSuccess) return ctx_fail(c, GNS_EHIP, "set first kernel params", e);
    e = hipGraphLaunch(g.exec, s);
    if (e != hipSuccess) return ctx_fail(c, GNS_EHIP, "graph launch", e);
    return GNS_OK;
}

namespace gns {
// What a context's per-batch scratch must hold before its first mini-batch: zeroed device state, an empty
// frontier mark bitmap, two empty hash maps.  Enqueue only.
hipError_t init_batch_scratch(gns_ctx* c, hipStream_t s)
{
    const Layout& L = c->lay;
    hipError_t e = launch_fill_u32(reinterpret_cast<uint32_t*>(c->d_state), (sizeof(DeviceState) + 64) / 4, 0u, s);
    if (e == hipSuccess) e = launch_fill_u64(ws_ptr<unsigned long long>(c, L.mark_bitmap), (size_t) L.words, 0ull, s);
    if (e == hipSuccess && L.summary_words > 0)
        e = launch_fill_u64(ws_ptr<unsigned long long>(c, L.mark_summary), (size_t) L.summary_words, 0ull, s);
    for (int par = 0; par < 2 && e == hipSuccess; ++par)
        e = launch_fill_u64(ws_ptr<unsigned long long>(c, L.hash_slots[par]), (size_t) L.hash_cap, ~0ull, s);
    return e;
}

// A context that shares root's graph, config and cache and keeps its per-batch scratch at `workspace`
// (not initialised here).  Joins root's family.
gns_status make_child(gns_ctx* root, void* workspace, bool with_capture_stream, gns_ctx** out)
{
    *out = nullptr;
    if (root->family_count >= (int) (sizeof(root->family) / sizeof(root->family[0])))
        return ctx_fail(root, GNS_ECAPACITY, "too many live forks of one context");
    gns_ctx* c = new (std::nothrow) gns_ctx;
    if (!c) return ctx_fail(root, GNS_ENOMEM, "host allocation failed");
    memcpy(c, root, sizeof(*c));
    c->ws = static_cast<char*>(workspace);
    c->shared_ws = root->ws;
    c->root = root;
    c->d_state = ws_ptr<DeviceState>(c, c->lay.state);
    c->h_state = nullptr;
    c->prof = nullptr;
    c->prof_capacity = c->prof_count = 0;
    c->prof_mask = 0;
    c->err[0] = 0;
    c->bg = nullptr;
    c->graph_clock = 0;
    c->hash_parity = 0;
    c->batch_id = 0;
    c->bad_reported = 0;
    c->cap_stream = nullptr;
    c->family_count = 0;
    c->static_child = nullptr;
    memset(c->gen_event, 0, sizeof(c->gen_event));
    c->ready_event[0] = c->ready_event[1] = nullptr;
    hipError_t e = hipSuccess;
    if (with_capture_stream) {
        e = hipStreamCreateWithFlags(&c->cap_stream, hipStreamNonBlocking);
        if (e != hipSuccess) c->cap_stream = nullptr;
        c->bg = static_cast<BatchGraph*>(calloc(kGraphsPerContext, sizeof(BatchGraph)));
        if (e == hipSuccess && !c->bg) e = hipErrorOutOfMemory;
    }
    if (e == hipSuccess) {
        e = hipHostMalloc(reinterpret_cast<void**>(&c->h_state), sizeof(DeviceState), hipHostMallocDefault);
        if (e != hipSuccess) c->h_state = nullptr;
    }
    if (e == hipSuccess) e = events_create(c);
    if (e != hipSuccess) {
        free(c->bg);
        if (c->h_state) (void) hipHostFree(c->h_state);
        if (c->cap_stream) (void) hipStreamDestroy(c->cap_stream);
        events_destroy(c);
        delete c;
        return ctx_fail(root, GNS_EHIP, "child context", e);
    }
    root->family[root->family_count++] = c;
    *out = c;
    return GNS_OK;
}
}  // namespace gns

extern "C" {

size_t gns_workspace_bytes(const gns_graph* graph, const gns_config* config)
{
    Layout L;
    if (!compute_layout(graph, config, &L, g_create_err, sizeof(g_create_err))) return 0;
    return L.total;
}

gns_status gns_block_capacity(const gns_graph* graph, const gns_config* config, int32_t layer_index,
                              int32_t* cap_dst, int32_t* cap_src, int32_t* cap_edges)
{
    Layout L;
    if (!compute_layout(graph, config, &L, g_create_err, sizeof(g_create_err))) return GNS_EINVAL;
    if (layer_index < 0 || layer_index >= config->num_layers) {
        snprintf(g_create_err, sizeof(g_create_err), "layer_index out of range");
        return GNS_EINVAL;
    }
    if (cap_dst) *cap_dst = (int32_t) L.rows[layer_index];
    if (cap_src) *cap_src = (int32_t) L.rows[layer_index + 1];
    if (cap_edges) *cap_edges = (int32_t) L.edges[layer_index];
    return GNS_OK;
}

gns_status gns_create(gns_ctx** out_ctx, const gns_graph* graph, const gns_config* config, void* workspace,
                      size_t workspace_bytes, void* hip_stream)
{
    if (!out_ctx) { snprintf(g_create_err, sizeof(g_create_err), "null out_ctx"); return GNS_EINVAL; }
    *out_ctx = nullptr;
    Layout L;
    if (!compute_layout(graph, config, &L, g_create_err, sizeof(g_create_err))) return GNS_EINVAL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) {
        snprintf(g_create_err, sizeof(g_create_err), "workspace must be a 256-byte aligned device pointer");
        return GNS_EINVAL;
    }
    if (workspace_bytes < L.total) {
        snprintf(g_create_err, sizeof(g_create_err), "workspace too small: need %zu bytes", L.total);
        return GNS_ECAPACITY;
    }
    gns_ctx* c = new (std::nothrow) gns_ctx;
    if (!c) { snprintf(g_create_err, sizeof(g_create_err), "host allocation failed"); return GNS_ENOMEM; }
    memset(c, 0, sizeof(*c));
    c->graph = *graph;
    c->config = *config;
    c->lay = L;
    c->ws = static_cast<char*>(workspace);
    c->shared_ws = c->ws;
    c->root = c;
    c->d_state = ws_ptr<DeviceState>(c, L.state);
    c->uses_cache = config_uses_cache(config);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    auto bail = [&](gns_status st, const char* what, hipError_t e) {
        if (e != hipSuccess) snprintf(g_create_err, sizeof(g_create_err), "%s: %s", what, hipGetErrorString(e));
        else snprintf(g_create_err, sizeof(g_create_err), "%s", what);
        if (c->h_state) (void) hipHostFree(c->h_state);
        if (c->cap_stream) (void) hipStreamDestroy(c->cap_stream);
        free(c->bg);
        events_destroy(c);
        delete c;
        return st;
    };

    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return bail(GNS_EHIP, "hipGetDevice", e);
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return bail(GNS_EHIP, "hipGetDeviceProperties", e);
    c->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    // the flag kernel may keep the whole cache bitmap in LDS (one 1024-thread block per CU)
    c->lds_bitmap_limit = prop.sharedMemPerBlock >= kLdsBitmapBytes + 1024 ? kLdsBitmapBytes : 0;
    e = hipHostMalloc(reinterpret_cast<void**>(&c->h_state), sizeof(DeviceState), hipHostMallocDefault);
    if (e != hipSuccess) { c->h_state = nullptr; return bail(GNS_EHIP, "hipHostMalloc", e); }
    e = events_create(c);
    if (e != hipSuccess) return bail(GNS_EHIP, "hipEventCreate", e);
    c->family[0] = c;
    c->family_count = 1;
    if (!getenv("GNS_NO_GRAPH")) {
        e = hipStreamCreateWithFlags(&c->cap_stream, hipStreamNonBlocking);
        if (e != hipSuccess) { c->cap_stream = nullptr; return bail(GNS_EHIP, "hipStreamCreate", e); }
        c->bg = static_cast<BatchGraph*>(calloc(kGraphsPerContext, sizeof(BatchGraph)));
        if (!c->bg) return bail(GNS_ENOMEM, "host allocation failed", hipSuccess);
    }

    // zero the state, the mark bitmap and the cache bitmap; validate the graph
    e = init_batch_scratch(c, s);
    if (e == hipSuccess) e = launch_fill_u64(cache_ptr<unsigned long long>(c, L.cache_bitmap, 0), (size_t) L.words, 0ull, s);
    if (e != hipSuccess) return bail(GNS_EHIP, "workspace init", e);
    int32_t* d_info = ws_ptr<int32_t>(c, L.sums_words);   // scratch, 4 ints
    e = launch_count_nonzero_rows(c, s, d_info);
    if (e != hipSuccess) return bail(GNS_EHIP, "graph validation launch", e);
    int32_t info[4] = {0, 0, 0, 0};
    e = hipMemcpyAsync(info, d_info, sizeof(info), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return bail(GNS_EHIP, "graph validation", e);
    if (info[1]) return bail(GNS_EINVAL, "indptr is not a non-decreasing offset array from 0 to num_entries", hipSuccess);
    if (info[2]) return bail(GNS_EINVAL, "indices holds an id outside [0, num_nodes)", hipSuccess);
    if (info[3]) return bail(GNS_EINVAL, "CSR rows must be sorted ascending without duplicates", hipSuccess);
    c->nonzero_degree_nodes = info[0];
    if (c->uses_cache && config->cache_size > c->nonzero_degree_nodes)
        return bail(GNS_EINVAL, "cache_size exceeds the number of nodes that have a neighbor", hipSuccess);
    // the hidden context gns_sample_blocks_static runs on (none if the per-batch scratch does not fit)
    {
        const gns_status st = static_scratch_setup(c);
        if (st != GNS_OK) {
            snprintf(g_create_err, sizeof(g_create_err), "%s", c->err);
            (void) gns_destroy(c);
            return st;
        }
    }
    *out_ctx = c;
    return GNS_OK;
}

static void profile_release(gns_ctx* c)
{
    for (int32_t i = 0; i < c->prof_capacity; ++i) {
        (void) hipEventDestroy(c->prof[i].start);
        (void) hipEventDestroy(c->prof[i].stop);
    }
    free(c->prof);
    c->prof = nullptr;
    c->prof_capacity = 0;
    c->prof_count = 0;
    c->prof_mask = 0;
}

gns_status gns_profile_begin(gns_ctx* ctx, uint32_t stage_mask, int32_t capacity)
{
    if (!ctx) return GNS_EINVAL;
    profile_release(ctx);
    if (stage_mask == 0) return GNS_OK;
    if (capacity < 1 || capacity > (1 << 20)) return ctx_fail(ctx, GNS_EINVAL, "profile capacity out of range");
    ctx->prof = static_cast<ProfileRecord*>(calloc((size_t) capacity, sizeof(ProfileRecord)));
    if (!ctx->prof) return ctx_fail(ctx, GNS_ENOMEM, "profile records");
    for (int32_t i = 0; i < capacity; ++i) {
        hipError_t e = hipEventCreate(&ctx->prof[i].start);
        if (e == hipSuccess) e = hipEventCreate(&ctx->prof[i].stop);
        if (e != hipSuccess) {
            ctx->prof_capacity = i;
            profile_release(ctx);
            return ctx_fail(ctx, GNS_EHIP, "hipEventCreate", e);
        }
    }
    ctx->prof_capacity = capacity;
    ctx->prof_mask = stage_mask;
    return GNS_OK;
}

gns_status gns_profile_collect(gns_ctx* ctx, int32_t stage, double* total_ms, int32_t* launches)
{
    if (!ctx || !total_ms || !launches) return GNS_EINVAL;
    double sum = 0.0;
    int32_t n = 0, kept = 0;
    for (int32_t i = 0; i < ctx->prof_count; ++i) {
        ProfileRecord r = ctx->prof[i];
        if (r.stage != stage) {                 // keep records of other stages, compacted to the front
            ProfileRecord tmp = ctx->prof[kept];
            ctx->prof[kept] = r;
            ctx->prof[i] = tmp;
            ++kept;
            continue;
        }
        hipError_t e = hipEventSynchronize(r.stop);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
        if (e != hipSuccess) return ctx_fail(ctx, GNS_EHIP, "profile collect", e);
        sum += (double) ms;
        ++n;
    }
    // the collected records' events now sit behind `kept`; reuse them
    ctx->prof_count = kept;
    *total_ms = sum;
    *launches = n;
    return GNS_OK;
}

size_t gns_fork_workspace_bytes(const gns_ctx* parent)
{
    return parent ? parent->lay.shared_begin : 0;
}

gns_status gns_fork(gns_ctx* parent, void* workspace, size_t workspace_bytes, void* hip_stream, gns_ctx** out_child)
{
    if (!parent || !out_child) return GNS_EINVAL;
    *out_child = nullptr;
    gns_ctx* root = parent->root;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return ctx_fail(parent, GNS_EINVAL, "workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < root->lay.shared_begin) return ctx_fail(parent, GNS_ECAPACITY, "fork workspace too small");
    gns_ctx* c = nullptr;
    const gns_status st = make_child(root, workspace, root->cap_stream != nullptr, &c);
    if (st != GNS_OK) { snprintf(parent->err, sizeof(parent->err), "%s", root->err); return st; }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e = init_batch_scratch(c, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        (void) gns_destroy(c);
        return ctx_fail(parent, GNS_EHIP, "fork init", e);
    }
    *out_child = c;
    return GNS_OK;
}

gns_status gns_destroy(gns_ctx* ctx)
{
    if (!ctx) return GNS_OK;
    if (ctx->static_child) { (void) gns_destroy(ctx->static_child); ctx->static_child = nullptr; }
    profile_release(ctx);
    // captured launch sequences that name this context: its own, and those of groups it was a member of
    gns_ctx* fam_root = ctx->root;
    for (int i = 0; i < fam_root->family_count; ++i) {
        gns_ctx* m = fam_root->family[i];
        if (!m->bg) continue;
        for (int k = 0; k < kGraphsPerContext; ++k) {
            BatchGraph& g = m->bg[k];
            bool names = m == ctx;
            for (int b = 0; !names && b < g.count; ++b) names = g.ctx[b] == ctx;
            if (names) graph_release(g);
        }
    }
    free(ctx->bg);
    ctx->bg = nullptr;
    if (ctx->cap_stream) (void) hipStreamDestroy(ctx->cap_stream);
    if (ctx->h_state) (void) hipHostFree(ctx->h_state);
    events_destroy(ctx);
    if (ctx->root != ctx) {                               // a fork leaves its family
        gns_ctx* root = ctx->root;
        for (int i = 0; i < root->family_count; ++i)
            if (root->family[i] == ctx) { root->family[i] = root->family[--root->family_count]; break; }
    }
    delete ctx;
    return GNS_OK;
}

gns_status gns_sample_cache(gns_ctx* ctx, uint64_t seed, uint64_t epoch, void* hip_stream)
{
    if (!ctx) return GNS_EINVAL;
    if (!ctx->uses_cache) return ctx_fail(ctx, GNS_ESTATE, "no layer of this config uses the cache");
    if (ctx->root != ctx) return ctx_fail(ctx, GNS_EINVAL, "draw the cache on the context made by gns_create, not on a fork");
    if (epoch >> 32) return ctx_fail(ctx, GNS_EINVAL, "epoch must be < 2^32");
    if (ctx->config.cache_probability == GNS_PROB_WALK) {
        if (!ctx->prob_valid) return ctx_fail(ctx, GNS_ESTATE, "gns_cache_walk_probability must run before gns_sample_cache");
        if (ctx->config.cache_size > ctx->prob_support)
            return ctx_fail(ctx, GNS_EINVAL, "cache_size exceeds the number of nodes the walk probability reaches");
    }
    return run_sample_cache(ctx, seed, epoch, true, static_cast<hipStream_t>(hip_stream));
}

gns_status gns_sample_cache_async(gns_ctx* ctx, uint64_t seed, uint64_t epoch, void* hip_stream)
{
    if (!ctx) return GNS_EINVAL;
    if (!ctx->uses_cache) return ctx_fail(ctx, GNS_ESTATE, "no layer of this config uses the cache");
    if (ctx->root != ctx) return ctx_fail(ctx, GNS_EINVAL, "draw the cache on the context made by gns_create, not on a fork");
    if (epoch >> 32) return ctx_fail(ctx, GNS_EINVAL, "epoch must be < 2^32");
    if (ctx->config.cache_probability == GNS_PROB_WALK) {
        if (!ctx->prob_valid) return ctx_fail(ctx, GNS_ESTATE, "gns_cache_walk_probability must run before gns_sample_cache");
        if (ctx->config.cache_size > ctx->prob_support)
            return ctx_fail(ctx, GNS_EINVAL, "cache_size exceeds the number of nodes the walk probability reaches");
    }
    return run_sample_cache(ctx, seed, epoch, false, static_cast<hipStream_t>(hip_stream));
}

gns_status gns_activate_cache(gns_ctx* ctx)
{
    if (!ctx) return GNS_EINVAL;
    if (ctx->root != ctx) return ctx_fail(ctx, GNS_EINVAL, "activate the cache on the context made by gns_create, not on a fork");
    if (!ctx->pending) return ctx_fail(ctx, GNS_ESTATE, "no cache draw is waiting to be made current");
    return activate_cache(ctx);
}

gns_status gns_cache_walk_probability(gns_ctx* ctx, const int32_t* train_nodes_dev, int64_t num_train,
                                      int32_t scale_log2, void* hip_stream)
{
    if (!ctx) return GNS_EINVAL;
    if (ctx->root != ctx) return ctx_fail(ctx, GNS_EINVAL, "set the cache probability on the context made by gns_create, not on a fork");
    if (!ctx->uses_cache || ctx->config.cache_probability != GNS_PROB_WALK)
        return ctx_fail(ctx, GNS_ESTATE, "the config does not ask for GNS_PROB_WALK");
    if (!train_nodes_dev || num_train < 1) return ctx_fail(ctx, GNS_EINVAL, "no training nodes");
    if (scale_log2 < 0 || scale_log2 > 40) return ctx_fail(ctx, GNS_EINVAL, "scale_log2 must be in [0, 40]");
    // Mini-batches still in flight keep reading the current copy of the cache structures: record where they
    // end, as a draw does when it replaces a cache, so that the draw after next does not overwrite that copy
    // under them; the next draw goes into the other copy.
    if (ctx->cache_valid) {
        const gns_status st = retire_cache(ctx);
        if (st != GNS_OK) return st;
    }
    return run_walk_probability(ctx, train_nodes_dev, num_train, scale_log2, static_cast<hipStream_t>(hip_stream));
}

gns_status gns_cache_probability_view(gns_ctx* ctx, const uint64_t** weights, const int64_t** prefix,
                                      uint64_t* total, int64_t* support)
{
    if (!ctx) return GNS_EINVAL;
    gns_ctx* root = ctx->root;
    if (!root->prob_valid) return ctx_fail(ctx, GNS_ESTATE, "no cache probability has been computed");
    if (weights) *weights = reinterpret_cast<const uint64_t*>(root->prob_weights);
    if (prefix) *prefix = ws_ptr<int64_t>(root, root->lay.prob_prefix);
    if (total) *total = root->prob_total;
    if (support) *support = root->prob_support;
    return GNS_OK;
}

gns_status gns_cache_view(gns_ctx* ctx, const int32_t** cache_nodes, int64_t* cache_size, const uint64_t** bitmap,
                          int64_t* num_draws)
{
    if (!ctx) return GNS_EINVAL;
    if (!ctx->uses_cache || !ctx->root->cache_valid) return ctx_fail(ctx, GNS_ESTATE, "no cache has been drawn");
    if (cache_nodes) *cache_nodes = cache_ptr<int32_t>(ctx, ctx->lay.cache_nodes, active_gen(ctx));
    if (cache_size) *cache_size = ctx->config.cache_size;
    if (bitmap) *bitmap = cache_ptr<uint64_t>(ctx, ctx->lay.cache_bitmap, active_gen(ctx));
    if (ctx->root->cache_draws < 0) {                     // drawn asynchronously: look at the outcome now
        const gns_status st = finish_pending_draw(ctx->root);
        if (st != GNS_OK) { snprintf(ctx->err, sizeof(ctx->err), "%s", ctx->root->err); return st; }
    }
    if (num_draws) *num_draws = ctx->root->cache_draws;
    return GNS_OK;
}

// Checks a group: 1..GNS_MAX_GROUP distinct contexts of one family.  Errors are reported on ctxs[0].
static gns_status check_group(gns_ctx* const* ctxs, int32_t count)
{
    if (!ctxs || count < 1 || !ctxs[0]) return GNS_EINVAL;
    gns_ctx* lead = ctxs[0];
    if (count > GNS_MAX_GROUP) return ctx_fail(lead, GNS_EINVAL, "a group holds at most GNS_MAX_GROUP mini-batches");
    for (int b = 0; b < count; ++b) {
        if (!ctxs[b]) return ctx_fail(lead, GNS_EINVAL, "null context in the group");
        if (ctxs[b]->root != lead->root) return ctx_fail(lead, GNS_EINVAL, "the contexts of a group must be one context and its forks");
        for (int q = 0; q < b; ++q)
            if (ctxs[q] == ctxs[b]) return ctx_fail(lead, GNS_EINVAL, "a context appears twice in the group");
    }
    return GNS_OK;
}

static gns_status group_before_cache_readers(gns_ctx* const* ctxs, int32_t count, hipStream_t s)
{
    for (int b = 0; b < count; ++b) {
        const hipError_t er = before_cache_readers(ctxs[b], s);
        if (er == hipErrorInvalidValue) return ctx_fail(ctxs[0], GNS_ESTATE, "a context may use at most 4 streams between two cache draws");
        if (er != hipSuccess) return ctx_fail(ctxs[0], GNS_EHIP, "wait for the cache draw", er);
    }
    return GNS_OK;
}

gns_status gns_sample_blocks_group(gns_ctx* const* ctxs, int32_t count, const uint64_t* seeds,
                                   const int32_t* const* seeds_dev, const int32_t* num_seeds,
                                   gns_block* const* blocks, void* hip_stream)
{
    gns_status st = check_group(ctxs, count);
    if (st != GNS_OK) return st;
    gns_ctx* lead = ctxs[0];
    if (!seeds || !seeds_dev || !num_seeds || !blocks) return ctx_fail(lead, GNS_EINVAL, "null argument array");
    Group g;
    memset(&g, 0, sizeof(g));
    g.count = count;
    for (int b = 0; b < count; ++b) {
        st = check_batch_args(ctxs[b], seeds_dev[b], num_seeds[b], blocks[b]);
        if (st != GNS_OK) {
            if (ctxs[b] != lead) snprintf(lead->err, sizeof(lead->err), "%s", ctxs[b]->err);
            return st;
        }
        g.ctx[b] = ctxs[b];
        g.blocks[b] = blocks[b];
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    st = group_before_cache_readers(ctxs, count, s);
    if (st != GNS_OK) return st;
    BeginDyn dyn;
    fill_begin_dyn(g, seeds, seeds_dev, num_seeds, &dyn);
    if (lead->prof_mask == 0 && lead->cap_stream) st = launch_batch_graph(g, dyn, s);
    else                                           st = enqueue_batch(g, dyn, s);
    if (st != GNS_OK) return st;
    const int nl = lead->config.num_layers;
    for (int b = 0; b < count; ++b) {
        ctxs[b]->batch_id += 1;
        ctxs[b]->hash_parity ^= 1;             // this batch has left the other map empty
        for (int i = 0; i < nl; ++i) {
            blocks[b][i].num_dst = GNS_DEVICE_COUNTS(i);
            blocks[b][i].num_src = -1;
            blocks[b][i].num_edges = -1;
        }
    }
    return GNS_OK;
}

gns_status gns_sample_blocks_group_wait(gns_ctx* const* ctxs, int32_t count, gns_block* const* blocks, void* hip_stream)
{
    gns_status st = check_group(ctxs, count);
    if (st != GNS_OK) return st;
    gns_ctx* lead = ctxs[0];
    if (!blocks) return ctx_fail(lead, GNS_EINVAL, "null blocks");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipSuccess;
    for (int b = 0; b < count && e == hipSuccess; ++b)
        e = hipMemcpyAsync(ctxs[b]->h_state, ctxs[b]->d_state, sizeof(DeviceState), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return ctx_fail(lead, GNS_EHIP, "sample_blocks wait", e);
    st = GNS_OK;
    for (int b = 0; b < count; ++b) {
        gns_ctx* c = ctxs[b];
        if (!blocks[b]) return ctx_fail(lead, GNS_EINVAL, "null blocks");
        for (int i = 0; i < c->config.num_layers; ++i) {
            blocks[b][i].num_dst = c->h_state->num_dst[i];
            blocks[b][i].num_src = c->h_state->num_dst[i + 1];
            blocks[b][i].num_edges = c->h_state->num_edges[i];
        }
        // bad_seed holds the id of the latest mini-batch that had a bad seed: anything newer than the last one
        // reported means that a batch enqueued since the previous wait (not necessarily the last one) was bad
        if (c->h_state->bad_seed != c->bad_reported) {
            c->bad_reported = c->h_state->bad_seed;
            st = ctx_fail(lead, GNS_EINVAL, "seeds must be distinct node ids in [0, num_nodes) (a mini-batch enqueued since the last wait had a bad seed)");
        }
    }
    return st;
}

gns_status gns_sample_blocks_async(gns_ctx* ctx, uint64_t seed, const int32_t* seeds_dev, int32_t num_seeds,
                                   gns_block* blocks, void* hip_stream)
{
    if (!ctx) return GNS_EINVAL;
    return gns_sample_blocks_group(&ctx, 1, &seed, &seeds_dev, &num_seeds, &blocks, hip_stream);
}

gns_status gns_sample_blocks_wait(gns_ctx* ctx, gns_block* blocks, void* hip_stream)
{
    if (!ctx) return GNS_EINVAL;
    return gns_sample_blocks_group_wait(&ctx, 1, &blocks, hip_stream);
}

gns_status gns_sample_blocks(gns_ctx* ctx, uint64_t seed, const int32_t* seeds_dev, int32_t num_seeds,
                             gns_block* blocks, void* hip_stream)
{
    const gns_status st = gns_sample_blocks_async(ctx, seed, seeds_dev, num_seeds, blocks, hip_stream);
    if (st != GNS_OK) return st;
    return gns_sample_blocks_wait(ctx, blocks, hip_stream);
}

gns_status gns_gather_features_group(gns_ctx* const* ctxs, int32_t count, const int32_t* const* nodes_dev,
                                     const int32_t* num_nodes, float* const* out_dev, void* hip_stream)
{
    gns_status st = check_group(ctxs, count);
    if (st != GNS_OK) return st;
    gns_ctx* lead = ctxs[0];
    if (lead->graph.feat_dim <= 0) return ctx_fail(lead, GNS_ESTATE, "the graph was created without features");
    if (!nodes_dev || !num_nodes || !out_dev) return ctx_fail(lead, GNS_EINVAL, "null argument array");
    bool any = false;
    for (int b = 0; b < count; ++b) {
        if (num_nodes[b] == 0) continue;
        any = true;
        if (!nodes_dev[b] || !out_dev[b]) return ctx_fail(lead, GNS_EINVAL, "null nodes or output");
    }
    if (!any) return GNS_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    st = group_before_cache_readers(ctxs, count, s);
    if (st != GNS_OK) return st;
    StageTimer t(lead, GNS_STAGE_GATHER, s);
    hipError_t e = launch_gather(ctxs, count, nodes_dev, num_nodes, out_dev, active_gen(lead), s);
    if (e != hipSuccess) return ctx_fail(lead, GNS_EHIP, "gather launch", e);
    return GNS_OK;
}

gns_status gns_gather_features(gns_ctx* ctx, const int32_t* nodes_dev, int32_t num_nodes, float* out_dev,
                               void* hip_stream)
{
    if (!ctx) return GNS_EINVAL;
    return gns_gather_features_group(&ctx, 1, &nodes_dev, &num_nodes, &out_dev, hip_stream);
}

gns_status gns_aggregate_group(gns_ctx* const* ctxs, int32_t count, const gns_block* const* blocks,
                               const float* const* x_src_dev, int32_t feat_dim, float* const* out_dev, void* hip_stream)
{
    gns_status st = check_group(ctxs, count);
    if (st != GNS_OK) return st;
    gns_ctx* lead = ctxs[0];
    if (!blocks || !x_src_dev || !out_dev) return ctx_fail(lead, GNS_EINVAL, "null argument array");
    if (feat_dim < 1) return ctx_fail(lead, GNS_EINVAL, "feat_dim must be >= 1");
    for (int b = 0; b < count; ++b) {
        const gns_block* block = blocks[b];
        if (!block || !x_src_dev[b] || !out_dev[b]) return ctx_fail(lead, GNS_EINVAL, "null block, input or output");
        if (block->num_dst < 0) {
            if (-1 - block->num_dst >= lead->config.num_layers) return ctx_fail(lead, GNS_EINVAL, "bad device-count placeholder");
        } else if (block->num_src < block->num_dst || block->num_edges < 0) {
            return ctx_fail(lead, GNS_EINVAL, "block counts are inconsistent");
        }
        if (!block->indptr || !block->indices || !block->weights) return ctx_fail(lead, GNS_EINVAL, "block has a null buffer");
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    StageTimer t(lead, GNS_STAGE_AGGREGATE, s);
    hipError_t e = launch_aggregate(ctxs, count, blocks, x_src_dev, feat_dim, out_dev, s);
    if (e != hipSuccess) return ctx_fail(lead, GNS_EHIP, "aggregate launch", e);
    return GNS_OK;
}

gns_status gns_aggregate(gns_ctx* ctx, const gns_block* block, const float* x_src_dev, int32_t feat_dim,
                         float* out_dev, void* hip_stream)
{
    if (!ctx) return GNS_EINVAL;
    return gns_aggregate_group(&ctx, 1, &block, &x_src_dev, feat_dim, &out_dev, hip_stream);
}

gns_status gns_sage_dense(gns_ctx* ctx, const float* h_self_dev, int32_t f1, const float* h_neigh_dev, int32_t f2,
                          const float* w_dev, const float* bias_dev, int32_t hdim, int32_t relu, float* out_dev,
                          int32_t num_rows, void* hip_stream)
{
    if (!ctx) return GNS_EINVAL;
    if (!h_self_dev || !h_neigh_dev || !w_dev || !out_dev) return ctx_fail(ctx, GNS_EINVAL, "null input, weight or output");
    if (f1 < 4 || f2 < 4 || hdim < 4 || (f1 & 3) || (f2 & 3) || (hdim & 3))
        return ctx_fail(ctx, GNS_EINVAL, "f1, f2 and hdim must be positive multiples of 4");
    const uintptr_t bits = reinterpret_cast<uintptr_t>(h_self_dev) | reinterpret_cast<uintptr_t>(h_neigh_dev) |
                           reinterpret_cast<uintptr_t>(w_dev) | reinterpret_cast<uintptr_t>(out_dev);
    if (bits & 15u) return ctx_fail(ctx, GNS_EINVAL, "inputs, weights and output must be 16-byte aligned");
    if (num_rows < 0 && -1 - num_rows >= ctx->config.num_layers) return ctx_fail(ctx, GNS_EINVAL, "bad device-count placeholder");
    StageTimer t(ctx, GNS_STAGE_DENSE, static_cast<hipStream_t>(hip_stream));
    hipError_t e = launch_sage_dense(ctx, h_self_dev, f1, h_neigh_dev, f2, w_dev, bias_dev, hdim, relu, out_dev, num_rows,
                                     static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return ctx_fail(ctx, GNS_EHIP, "dense launch", e);
    return GNS_OK;
}

const char* gns_last_error(const gns_ctx* ctx)
{
    return ctx ? ctx->err : g_create_err;
}

}  // extern "C"
