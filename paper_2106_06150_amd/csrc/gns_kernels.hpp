// Kernel argument blocks and device bodies shared between the sampler and the frontier kernels.
//
// One launch serves a *group* of up to kMaxGroup independent mini-batches (mini-batches are independent
// given the cache: the paper's sampling workers, Section 3.3): blockIdx.y is the batch's index in the
// group.  A launch's arguments are one LayerArgs: templates of the per-batch argument structs holding
// everything the batches have in common (graph, cache, layer constants), the offsets of the sections of a
// context's per-batch scratch, and one BatchSlot per batch (where its scratch lies, its block buffers).
// Every kernel first binds the templates to its own batch.
#pragma once
#include "gns_internal.h"
#include "gns_device.hpp"

namespace gns {

constexpr int kMaxGroup = GNS_MAX_GROUP;

// One record per aligned 64-entry chunk of the CSR entry array (GNS_FLAGS_PER_CACHE).
struct alignas(16) ChunkRec {
    uint64_t flags;            // bit e & 63: entry e points into the cache
    uint32_t before;           // number of such entries in all earlier chunks
    uint32_t pad;
};

struct SampleArgs {
    DeviceState* st;
    int layer_index;
    uint32_t layer_number;     // the paper's l = L - layer_index
    int fanout;
    int wmode;
    int policy;                // GNS_CACHE_ONLY or GNS_CACHE_FIRST for the select kernel
    int64_t num_nodes;
    const void* indptr;
    const int32_t* indices;
    const int32_t* dst_nodes;
    const RowExtent* row_ext;  // CSR extent of every dst row's node (written when the node joined the batch)
    const float* node_inv_pc;  // 1 / p^C_u for the nodes of the cache
    const int32_t* hub_rows;   // rows of the batch whose CSR segment spans more than kHubChunks chunks
    const uint64_t* cache_bitmap;
    const int32_t* cache_prefix;
    int64_t cache_size;
    int32_t* s_nbr;
    float* s_w;
    int32_t* s_cnt;
    int32_t* row_eligible;
    uint64_t* mark;
    uint64_t* mark_summary;    // one bit per word of mark, or null (small graphs)
    const unsigned long long* slots;   // batch hash map node -> local id (holds this layer's dst nodes)
    uint32_t hmask, hshift;
    // CACHE_ONLY: per-batch plan and the CSR-aligned membership flags
    int64_t num_entries;
    int32_t* plan_cnt;         // [rows] aligned 64-entry chunks touched by each dst row
    int32_t* plan_g0;          // [rows] id of the first of them
    int32_t* plan_sums;        // [row tiles + 1]
    int32_t* plan_desc;        // [chunks] ids of the aligned chunks to flag
    uint64_t* flags;           // [ceil(nnz / 64)] bit e & 63 of word e >> 6: entry e points into the cache
    int64_t bitmap_words;
    const uint64_t* coarse_bitmap;   // one bit per 2^coarse_shift ids (flag kernel, mode 2)
    int64_t coarse_words;
    int coarse_shift;
    const ChunkRec* srec;      // induced subgraph (GNS_FLAGS_PER_CACHE): chunk records and the cached entries' node ids
    const int32_t* s_nodes;
};

struct FinishArgs {
    DeviceState* st;
    int layer_index;
    int fanout;
    const int32_t* dst_nodes;      // [R]
    const int32_t* s_nbr;          // [R x fanout]
    const float* s_w;              // [R x fanout]
    const int32_t* s_cnt;          // [R]
    uint64_t* mark;                // [words]
    uint64_t* mark_summary;        // [ceil(words / 64)] or null: bit w & 63 of word w >> 6 says mark[w] != 0
    int64_t words;
    unsigned long long* slots;
    uint32_t hmask, hshift;
    int32_t* sums_rows;            // [row_tiles + 1]
    int32_t* sums_marks;           // [mark_tiles + 1]
    int32_t row_tiles_max;         // grid split point: blocks [0, row_tiles_max) work on rows
    int32_t mark_tiles;            // tiles of mark_tile_words bitmap words
    int32_t mark_tile_words;
    int32_t* indptr;               // block outputs
    int32_t* indices;
    float* weights;
    int32_t* src_nodes;
    int64_t max_slots;             // worst-case rows * fanout of this layer
    RowExtent* row_ext;            // [nodes of the batch] phase 3 appends the new nodes' CSR extents
    const void* g_indptr;          // the graph's offsets
    int g_i64;
    int32_t* hub_rows;             // phase 3 appends the new nodes that are hubs
    uint32_t* slot_list;           // phase 3 records the hash slot of every new node (for the sparse clear)
    int parity;                    // which of the two hash maps this batch uses
    unsigned long long* other_slots;       // the other hash map and its slot list (emptied by the batch's last kernel)
    const uint32_t* other_slot_list;
    int64_t num_nodes;
};

// Byte offsets of the sections of a context's per-batch scratch (the same for every context of a family).
struct WsOffsets {
    uint64_t state, mark, mark_summary, seed_copy, row_ext, hub_rows;
    uint64_t slot_list[2], hash_slots[2];
    uint64_t s_nbr[2], s_w[2], s_cnt[2];
    uint64_t plan_cnt, plan_g0, plan_desc;
    uint64_t sums_rows, sums_marks, sums_plan;
    uint64_t cache_block_bytes;    // distance between the two copies of what a cache draw writes
    int32_t uses_cache;
    int32_t has_summary;
};

struct BlockPtrs {
    int32_t* indptr;
    int32_t* indices;
    int32_t* src_nodes;
    int32_t* row_eligible;
    float* weights;
};

// What differs between the mini-batches of a group.
struct BatchSlot {
    char* ws;                  // the batch's context: its per-batch scratch
    const int32_t* dst;        // dst nodes of the layer being sampled / finished
    const int32_t* prev_dst;   // dst nodes of the layer before it
    BlockPtrs cur, prev;       // block buffers of that layer and of the one before it
};

struct LayerArgs {
    SampleArgs s;              // template: cache pointers are those of cache generation 0
    FinishArgs f;              // template for the layer the launch finishes or relabels
    WsOffsets off;
    BatchSlot b[kMaxGroup];
};

// What changes from one replay of a group's launch sequence to the next (arguments of the first kernel).
struct BeginDyn {
    const int32_t* seeds[kMaxGroup];
    int32_t num_seeds[kMaxGroup];
    uint32_t key0[kMaxGroup], key1[kMaxGroup];
    uint32_t batch_id[kMaxGroup];
    int32_t parity[kMaxGroup];     // which hash map the batch uses
    int32_t cache_gen[kMaxGroup];  // which copy of the cache structures it reads
};

template <typename T>
__device__ __forceinline__ T* at(char* base, uint64_t off) { return reinterpret_cast<T*>(base + off); }

__device__ __forceinline__ DeviceState* bind_state(const LayerArgs& g, int b)
{
    return at<DeviceState>(g.b[b].ws, g.off.state);
}

// The sampler's arguments for batch b of the group.  The hash-map parity and the cache generation were
// left in the batch's device state by its first kernel.
__device__ __forceinline__ SampleArgs bind_sample(const LayerArgs& g, int b)
{
    SampleArgs a = g.s;
    const BatchSlot& q = g.b[b];
    char* ws = q.ws;
    a.st = at<DeviceState>(ws, g.off.state);
    const int parity = a.st->hash_parity;
    const uint64_t gen_shift = a.st->cache_gen ? g.off.cache_block_bytes : 0;
    const int par = g.s.layer_index & 1;             // sampler scratch is double-buffered by layer parity
    a.dst_nodes = q.dst;
    a.row_ext = at<RowExtent>(ws, g.off.row_ext);
    a.hub_rows = g.off.uses_cache ? at<int32_t>(ws, g.off.hub_rows) : nullptr;
    a.s_nbr = at<int32_t>(ws, g.off.s_nbr[par]);
    a.s_w = at<float>(ws, g.off.s_w[par]);
    a.s_cnt = at<int32_t>(ws, g.off.s_cnt[par]);
    a.row_eligible = q.cur.row_eligible;
    a.mark = at<uint64_t>(ws, g.off.mark);
    a.mark_summary = g.off.has_summary ? at<uint64_t>(ws, g.off.mark_summary) : nullptr;
    a.slots = at<unsigned long long>(ws, g.off.hash_slots[parity]);
    a.plan_cnt = at<int32_t>(ws, g.off.plan_cnt);
    a.plan_g0 = at<int32_t>(ws, g.off.plan_g0);
    a.plan_sums = at<int32_t>(ws, g.off.sums_plan);
    a.plan_desc = at<int32_t>(ws, g.off.plan_desc);
    if (g.off.uses_cache) {
        a.node_inv_pc = reinterpret_cast<const float*>(reinterpret_cast<const char*>(g.s.node_inv_pc) + gen_shift);
        a.cache_bitmap = reinterpret_cast<const uint64_t*>(reinterpret_cast<const char*>(g.s.cache_bitmap) + gen_shift);
        a.cache_prefix = reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(g.s.cache_prefix) + gen_shift);
        a.flags = reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(g.s.flags) + gen_shift);
        if (g.s.coarse_bitmap)
            a.coarse_bitmap = reinterpret_cast<const uint64_t*>(reinterpret_cast<const char*>(g.s.coarse_bitmap) + gen_shift);
        if (g.s.srec) {
            a.srec = reinterpret_cast<const ChunkRec*>(reinterpret_cast<const char*>(g.s.srec) + gen_shift);
            a.s_nodes = reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(g.s.s_nodes) + gen_shift);
        }
    }
    return a;
}

// The union / relabel arguments of batch b for the layer the template describes: the launch's own layer
// (own_layer) or the one before it (a relabel riding in the next layer's sampler launch).
__device__ __forceinline__ FinishArgs bind_finish(const LayerArgs& g, int b, bool own_layer)
{
    FinishArgs a = g.f;
    const BatchSlot& q = g.b[b];
    char* ws = q.ws;
    a.st = at<DeviceState>(ws, g.off.state);
    const int parity = a.st->hash_parity;
    const int par = g.f.layer_index & 1;
    const BlockPtrs& blk = own_layer ? q.cur : q.prev;
    a.dst_nodes = own_layer ? q.dst : q.prev_dst;
    a.s_nbr = at<int32_t>(ws, g.off.s_nbr[par]);
    a.s_w = at<float>(ws, g.off.s_w[par]);
    a.s_cnt = at<int32_t>(ws, g.off.s_cnt[par]);
    a.mark = at<uint64_t>(ws, g.off.mark);
    a.mark_summary = g.off.has_summary ? at<uint64_t>(ws, g.off.mark_summary) : nullptr;
    a.slots = at<unsigned long long>(ws, g.off.hash_slots[parity]);
    a.sums_rows = at<int32_t>(ws, g.off.sums_rows);
    a.sums_marks = at<int32_t>(ws, g.off.sums_marks);
    a.indptr = blk.indptr;
    a.indices = blk.indices;
    a.weights = blk.weights;
    a.src_nodes = blk.src_nodes;
    a.row_ext = at<RowExtent>(ws, g.off.row_ext);
    a.hub_rows = g.off.uses_cache ? at<int32_t>(ws, g.off.hub_rows) : nullptr;
    a.slot_list = at<uint32_t>(ws, g.off.slot_list[parity]);
    a.parity = parity;
    a.other_slots = at<unsigned long long>(ws, g.off.hash_slots[parity ^ 1]);
    a.other_slot_list = at<uint32_t>(ws, g.off.slot_list[parity ^ 1]);
    return a;
}

// Relabel: every sampled edge of a finished layer gets its neighbor's local id (from the scratch slot if
// the sampler already found one, else from the batch's hash map) and is compacted to its CSR position.  `block` of `nblocks` blocks of kBlock threads.
// It only needs that layer's phase 3, so it shares a launch with the next layer's first kernel.
__device__ __forceinline__ void relabel_body(const FinishArgs& a, int64_t block, int64_t nblocks)
{
    const int32_t R = a.st->num_dst[a.layer_index];
    const int64_t limit = (int64_t) R * a.fanout;
    int64_t t = block * kBlock + threadIdx.x;
    const int64_t stride = nblocks * kBlock;
    for (; t < limit && t < a.max_slots; t += stride) {
        const int32_t row = (int32_t) (t / a.fanout);
        const int32_t s = (int32_t) (t - (int64_t) row * a.fanout);
        if (s < a.s_cnt[row]) {
            const int32_t u = a.s_nbr[t];          // -(local id + 1) if the sampler already knew it, else the global id
            const int32_t o = a.indptr[row] + s;
            a.indices[o] = u < 0 ? -1 - u : hash_lookup(a.slots, a.hmask, a.hshift, (uint32_t) u);
            a.weights[o] = a.s_w[t];
        }
    }
}

// A node whose CSR segment touches more than kHubChunks aligned 64-entry chunks is a hub: the
// CACHE_ONLY sampler gives such rows a whole wave each.  Nodes are classified when they join the
// batch's node list; the list of hub rows is append-only like the node list itself.
constexpr int kHubChunks = 32;

__device__ __forceinline__ bool is_hub_extent(int64_t start, int64_t end)
{
    return end > start && ((end - 1) >> 6) - (start >> 6) + 1 > kHubChunks;
}

// Appends `row` for the calling lanes that have is_hub set: one atomic per wave.
__device__ __forceinline__ void append_hub_rows(DeviceState* st, int32_t* hub_rows, bool is_hub, int32_t row)
{
    const uint64_t m = __ballot(is_hub && hub_rows != nullptr);      // no list without a cache layer
    if (m == 0) return;
    const int lane = lane_id();
    const int leader = __builtin_ctzll(m);
    int32_t base = 0;
    if (lane == leader) base = atomicAdd(&st->hub_count, (int32_t) __popcll(m));
    base = __shfl(base, leader, kWave);
    if (is_hub && hub_rows) hub_rows[base + __popcll(m & ((1ull << lane) - 1ull))] = row;
}

// ---------------------------------------------------------------------------
// Host side: a group of mini-batches and the argument block of one of its launches.
struct Group {
    int count;
    gns_ctx* ctx[kMaxGroup];
    gns_block* blocks[kMaxGroup];    // each: the caller's array of num_layers blocks
};

// Fills the parts of a LayerArgs that do not depend on the layer: offsets and the per-batch scratch bases.
void fill_group_args(const Group& g, LayerArgs* out);
// Points the slots at layer `layer_index` (dst lists and block buffers of that layer and the one before).
void set_group_layer(const Group& g, int layer_index, LayerArgs* out);
// The templates for one layer (sampler side: own layer; finish side: `finish_layer`).
void fill_sample_template(gns_ctx* c, int layer_index, SampleArgs* out);
void fill_finish_template(gns_ctx* c, int finish_layer, FinishArgs* out);
int relabel_grid(const gns_ctx* c, int layer_index);

}  // namespace gns
