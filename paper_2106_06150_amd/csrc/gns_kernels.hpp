// Kernel argument blocks and device bodies shared between the sampler and the frontier kernels.
#pragma once
#include "gns_internal.h"
#include "gns_device.hpp"

namespace gns {

struct FinishArgs {
    DeviceState* st;
    int layer_index;
    int fanout;
    const int32_t* dst_nodes;      // [R]
    const int32_t* s_nbr;          // [R x fanout]
    const float* s_w;              // [R x fanout]
    const int32_t* s_cnt;          // [R]
    uint64_t* mark;                // [words]
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
};

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

void fill_finish_args(gns_ctx* c, int layer_index, const int32_t* dst_nodes, const gns_block* blk, FinishArgs* out);
int relabel_grid(const gns_ctx* c, int layer_index);

}  // namespace gns
