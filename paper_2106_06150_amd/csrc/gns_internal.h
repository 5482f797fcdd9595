// Host-side internals of the GNS library: context, workspace layout and the
// launch functions each kernel file exports to the API layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/gns.h"

namespace gns {

// Device-resident scalars the kernels of one call communicate through.  The
// whole struct is copied to a pinned host mirror when a call has to report
// counts.
struct DeviceState {
    int32_t num_dst[GNS_MAX_LAYERS + 1];  // rows of layer index i (num_dst[i+1] = num_src of layer i)
    int32_t num_edges[GNS_MAX_LAYERS];
    uint32_t key0, key1;                  // Philox key of the current batch (lo32(seed), hi32(seed))
    uint32_t bad_seed;                    // id of the last batch that had a seed out of range or repeated
    int32_t map_nodes[2];                 // entries of each of the two hash maps (what its next clear has to undo)
    int32_t hub_count;                    // entries of the batch's hub-row list (reset by the batch's last kernel)
    int32_t chunk_distinct;               // cache draw: first occurrences found in the current chunk
    int32_t chunk_limit;                  //   how many of them enter the cache
    int32_t chunk_final;                  //   1 if they complete it
    int32_t draw_distinct;                //   nodes in the cache before the current chunk
    int32_t draw_done_chunk;              //   index of the chunk that completed the cache, -1 while incomplete
    int32_t plan_chunks;                  // CACHE_ONLY sampler: aligned chunks in the current work list
    int32_t hash_parity;                  // which of the two hash maps the current batch uses (set by its first kernel)
    int32_t cache_gen;                    // which copy of the cache structures it reads (set by its first kernel)
    unsigned long long cut_draw;          // cache draw: stream index of the draw that completed the cache
    unsigned long long walk_total;        // random-walk probability: sum of the weights
    int32_t walk_support;                 //   number of nodes with a non-zero weight
    int32_t walk_error;                   //   1: bad training node, 2: does not fit in 62 bits
};

// LDS a flag-kernel block may fill with a membership bitmap (the chip's 160 KB minus the block's own needs)
constexpr size_t kLdsBitmapBytes = 160 * 1024 - 1024;

struct Layout {
    // persistent cache structures
    size_t cache_bitmap, cache_prefix, cache_nodes, cache_feat;
    size_t coarse_bitmap;     // one bit per 2^coarse_shift node ids: "some node of the group is cached" (0: unused)
    int32_t coarse_shift;
    int64_t coarse_words;
    // random-walk cache probability (only with GNS_PROB_WALK): two weight vectors, their prefix, scan partials
    size_t walk_a, walk_b, prob_prefix, walk_tiles, walk_tiles_nz;
    size_t node_pc;           // [n] floats: 1 / p^C_u (Section 3.4), filled for the nodes of the current cache
    // cache-draw scratch
    size_t draw_keys, draw_vals, draw_node, draw_slot;
    // frontier structures
    size_t mark_bitmap;
    size_t mark_summary;      // one bit per word of the mark bitmap: "this word has a mark" (large graphs only)
    int64_t summary_words;    // 0: no summary
    size_t seed_copy;         // [max_seeds] the batch's seeds, copied by its first kernel
    size_t hub_rows;          // [max nodes of a batch] rows whose CSR segment spans more than kHubChunks chunks
    size_t row_ext;           // [max nodes of a batch] CSR extent of every node of the batch's list (append-only)
    size_t slot_list[2];      // [max nodes of a batch] per hash map: the slot each of the batch's nodes went into
    size_t hash_slots[2];     // consecutive batches alternate: each one leaves the other map empty for the next
    // per-layer sampler scratch (fixed stride fanout)
    size_t s_nbr[2], s_w[2], s_cnt[2];     // double-buffered by layer parity
    // CACHE_ONLY sampler: per-row chunk counts, chunk work list, CSR-aligned membership flags
    size_t plan_cnt, plan_g0, plan_desc, edge_flags;
    // GNS_FLAGS_PER_CACHE: the induced subgraph S of Section 3.3 in compact form.  s_nodes lists, in CSR order,
    // the entries that point into the cache; srec[g] = {flags of chunk g, number of such entries before chunk g},
    // so a row's cached neighbors are s_nodes[P(start) .. P(end)) with P(e) = off[e >> 6] + popcount(flags below e).
    size_t srec, s_nodes, sums_chunks;

    int64_t chunk_tiles;
    int64_t max_chunks;
    // scan partials
    size_t sums_rows, sums_words, sums_marks, sums_plan;
    size_t state;
    size_t shared_begin;      // sections at or past this offset are shared with forked contexts
    size_t cache_block_begin; // first of the two copies of what a cache draw writes (bitmap ... 1/p^C table)
    size_t cache_block_bytes; // the second copy lies this many bytes further
    size_t total;
    // sizes
    int64_t words;            // ceil(n / 64)
    int64_t word_tiles;       // ceil(words / kTile)
    int32_t mark_tile_words;  // bitmap words per frontier tile (kMarkTileMin .. kMarkTileMax, a power of two)
    int64_t mark_tiles;       // ceil(words / mark_tile_words)
    int64_t row_tiles;        // ceil(max rows / kTile)
    int64_t draw_chunk;       // stream draws processed per round of the cache draw
    int64_t draw_tiles;
    uint32_t draw_hash_cap;   // power of two
    uint32_t hash_cap;        // power of two
    int64_t max_rows;         // worst-case dst rows of any layer
    int64_t max_edges;        // worst-case edges of any layer
    int64_t rows[GNS_MAX_LAYERS + 1];
    int64_t edges[GNS_MAX_LAYERS];
};

}  // namespace gns

namespace gns {
// Streams one context may enqueue mini-batches on between two cache draws (each gets an event the
// draw after next waits for).
constexpr int kReaderStreams = 4;
struct Group;       // gns_kernels.hpp: the mini-batches one launch sequence serves
struct BeginDyn;    //   the first kernel's per-replay arguments
// Opaque host-side storage for the first kernel's two argument blocks (LayerArgs, BeginDyn).
struct BeginArgsHost {
    alignas(8) unsigned char fixed[3072];
    alignas(8) unsigned char dyn[768];
};
// One captured launch sequence of a group of mini-batches, kept by the group's first context.
struct BatchGraph {
    hipGraph_t graph;
    hipGraphExec_t exec;
    hipGraphNode_t first;            // the k_batch_begin node
    bool valid;
    uint64_t last_use;
    // capture key: the contexts of the group and the caller's block buffers
    int count;
    gns_ctx* ctx[GNS_MAX_GROUP];
    gns_block blocks[GNS_MAX_GROUP][GNS_MAX_LAYERS];
    BeginArgsHost args;              // the first kernel's arguments (the node's parameter list points here)
    void* arg_ptrs[2];
};
constexpr int kGraphsPerContext = 2;
struct ProfileRecord {
    int32_t stage;
    hipEvent_t start, stop;
};
}  // namespace gns

struct gns_ctx {
    gns_graph graph;
    gns_config config;
    gns::Layout lay;
    char* ws;                        // device workspace base (per-batch scratch sections)
    char* shared_ws;                 // base for the shared sections (the root context's workspace)
    gns_ctx* root;                   // owner of the cache; this for a context made by gns_create
    gns::DeviceState* d_state;       // device
    gns::DeviceState* h_state;       // pinned host mirror
    bool uses_cache;
    bool cache_valid;
    int cache_gen;                   // root only: which copy of the cache block the mini-batches read
    // Who may still read the copy a draw is about to overwrite: work enqueued before the previous draw.
    // Every draw records an event on the stream each context of the family last used (all that was
    // enqueued there so far) and waits, on the device, for the events the previous draw recorded.
    hipEvent_t gen_event[2][gns::kReaderStreams];   // alternate from draw to draw; one per stream used
    int gen_event_used[2];           // how many of them the draw that overwrites that copy has to wait for
    hipStream_t reader_streams[gns::kReaderStreams];   // where this context enqueued readers of the cache block
    int reader_stream_count;         //   since the last draw became current
    bool had_cache;                  // root only: some draw has been made current (cache_gen is meaningful)
    int64_t refresh_count;           // root only
    // root only: a draw enqueued by gns_sample_cache_async and not yet made current
    bool pending;
    int pending_gen;
    hipEvent_t ready_event[2];       // recorded behind the draw that filled the copy
    uint64_t cache_version;          // bumped when a copy becomes current
    uint64_t seen_version;           // per context: the version its stream has been made to wait for
    gns_ctx* family[64];             // root only: the root itself and its live forks
    int family_count;
    int64_t cache_draws;
    // cache probability other than Eq. (1): set by gns_cache_walk_probability on the root context
    bool prob_valid;
    const unsigned long long* prob_weights;   // device, [n]
    unsigned long long prob_total;
    int64_t prob_support;            // nodes with non-zero weight
    int64_t nonzero_degree_nodes;
    int num_cus;
    size_t lds_bitmap_limit;         // largest cache bitmap (bytes) the flag kernel stages in LDS
    // The launch sequence of one mini-batch, captured once per (seeds pointer, block buffers) and
    // replayed; only the first kernel's arguments (seed, number of seeds) change between replays.
    hipStream_t cap_stream;          // used for capture only, never for execution
    gns::BatchGraph* bg;             // [kGraphsPerContext] captured launch sequences (least recently used is replaced)
    uint64_t graph_clock;
    int hash_parity;                 // which hash map the next mini-batch uses
    uint32_t batch_id;               // id of the last mini-batch enqueued on this context (from 1)
    uint32_t bad_reported;           // DeviceState::bad_seed as of the last report to the caller
    gns_ctx* static_child;           // root only: the context of gns_sample_blocks_static (scratch in the library's array)
    char static_err[160];            // root only: why the library's scratch array is unavailable on this device, if it is
    // optional stage timing (benchmarks only)
    uint32_t prof_mask;
    int32_t prof_capacity;
    int32_t prof_count;
    gns::ProfileRecord* prof;
    char err[256];
};

namespace gns {

template <typename T>
static inline T* ws_ptr(const gns_ctx* c, size_t off)
{
    return reinterpret_cast<T*>((off >= c->lay.shared_begin ? c->shared_ws : c->ws) + off);
}

// A section of the cache block in the given generation (off is the section's offset in generation 0).
template <typename T>
static inline T* cache_ptr(const gns_ctx* c, size_t off, int gen)
{
    return reinterpret_cast<T*>(c->shared_ws + off + (gen ? c->lay.cache_block_bytes : 0));
}

// The generation the mini-batches enqueued now read.
static inline int active_gen(const gns_ctx* c) { return c->root->cache_gen; }

// Called before a context enqueues kernels that read the cache block on stream s: remembers the stream and,
// the first time after another copy became current, makes the stream wait for the draw that filled it.
static inline hipError_t before_cache_readers(gns_ctx* c, hipStream_t s)
{
    int known = 0;
    while (known < c->reader_stream_count && c->reader_streams[known] != s) ++known;
    if (known == c->reader_stream_count) {
        if (known == kReaderStreams) return hipErrorInvalidValue;     // reported as GNS_ESTATE
        c->reader_streams[c->reader_stream_count++] = s;
    }
    gns_ctx* root = c->root;
    if (!c->uses_cache || !root->cache_valid || c->seen_version == root->cache_version) return hipSuccess;
    c->seen_version = root->cache_version;
    return hipStreamWaitEvent(s, root->ready_event[root->cache_gen], 0);
}

gns_status ctx_fail(gns_ctx* c, gns_status st, const char* what, hipError_t e = hipSuccess);
// gns_api.hip
gns_status enqueue_batch(const Group& g, const BeginDyn& d, hipStream_t s);
void fill_begin_dyn(const Group& g, const uint64_t* seeds, const int32_t* const* seeds_dev, const int32_t* num_seeds,
                    BeginDyn* out);
gns_status check_batch_args(gns_ctx* c, const int32_t* seeds_dev, int32_t num_seeds, const gns_block* blocks);
hipError_t init_batch_scratch(gns_ctx* c, hipStream_t s);
gns_status make_child(gns_ctx* root, void* workspace, bool with_capture_stream, gns_ctx** out);
// gns_static.hip
gns_status static_scratch_setup(gns_ctx* root);
bool compute_layout(const gns_graph* g, const gns_config* cfg, Layout* out, char* err, size_t errlen);

// Brackets a stage's launches with events when that stage is being timed.
struct StageTimer {
    gns_ctx* c;
    hipStream_t s;
    int32_t slot;
    StageTimer(gns_ctx* ctx, int32_t stage, hipStream_t stream, bool enabled = true) : c(ctx), s(stream), slot(-1)
    {
        if (!enabled || !(c->prof_mask & (1u << stage)) || c->prof_count >= c->prof_capacity) return;
        slot = c->prof_count++;
        c->prof[slot].stage = stage;
        (void) hipEventRecord(c->prof[slot].start, s);
    }
    ~StageTimer()
    {
        if (slot >= 0) (void) hipEventRecord(c->prof[slot].stop, s);
    }
};

// gns_dense.hip
hipError_t launch_sage_dense(gns_ctx* c, const float* h_self, int32_t f1, const float* h_neigh, int32_t f2,
                             const float* w, const float* bias, int32_t hdim, int32_t relu, float* out,
                             int32_t num_rows, hipStream_t s);

// gns_walk.hip
gns_status run_walk_probability(gns_ctx* c, const int32_t* train_nodes, int64_t num_train, int32_t scale_log2,
                                hipStream_t s);

// gns_cache.hip
hipError_t launch_count_nonzero_rows(gns_ctx* c, hipStream_t s, int32_t* d_out);
// wait_for_it: run the chunk loop with a read-back per chunk and synchronise (exact error reporting); otherwise
// enqueue a fixed number of chunks (later ones stand down once the cache is complete) and return.
gns_status run_sample_cache(gns_ctx* c, uint64_t seed, uint64_t epoch, bool wait_for_it, hipStream_t s);
gns_status activate_cache(gns_ctx* c);
gns_status retire_cache(gns_ctx* c);
gns_status finish_pending_draw(gns_ctx* c);

// gns_induced.hip
hipError_t launch_build_induced(gns_ctx* c, int cache_gen, hipStream_t s);

// gns_sampler.hip
// the previous layer's relabel shares this layer's first launch
hipError_t launch_sample_layer(const Group& g, int layer_index, hipStream_t s);
hipError_t launch_flag_all_entries(gns_ctx* c, int cache_gen, hipStream_t s);

// gns_frontier.hip
hipError_t launch_batch_begin(const Group& g, const BeginDyn& d, hipStream_t s);
const void* batch_first_kernel();
hipError_t launch_relabel(const Group& g, int layer_index, hipStream_t s);
hipError_t launch_finish_layer(const Group& g, int layer_index, hipStream_t s);
hipError_t launch_fill_u64(unsigned long long* p, size_t n, unsigned long long v, hipStream_t s);
hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s);

// gns_feature.hip
// use_cache_gen < 0: every row comes from the full store (used while a cache's own table is being filled)
hipError_t launch_gather(gns_ctx* const* ctxs, int count, const int32_t* const* nodes, const int32_t* num_nodes,
                         float* const* out, int use_cache_gen, hipStream_t s);
hipError_t launch_aggregate(gns_ctx* const* ctxs, int count, const gns_block* const* blks, const float* const* x_src,
                            int32_t feat_dim, float* const* out, hipStream_t s);

}  // namespace gns
