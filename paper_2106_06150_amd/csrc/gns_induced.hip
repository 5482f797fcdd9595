// The induced subgraph S of the cache (paper Section 3.3: "we construct an induced subgraph S that contains
// the nodes in the cache and their neighbor nodes.  This is done once right after we sample nodes in the
// cache.") in compact form, built from the per-entry membership flags of GNS_FLAGS_PER_CACHE:
//
//   s_nodes   the CSR entries that point into the cache, in CSR order (node ids)
//   srec[g]   for every aligned 64-entry chunk g of the CSR entry array: its 64 flags and the number of
//             flagged entries in all earlier chunks
//
// The cached neighbors of a row with CSR extent [start, end) are then s_nodes[P(start) .. P(end)),
// P(e) = srec[e >> 6].before + popcount(srec[e >> 6].flags below bit e & 63): a mini-batch reads two
// records and the few entries it draws, never the row.  Three streaming passes per cache draw: count the
// flags per tile of chunks, scan, then compact the flagged entries.
#include "gns_kernels.hpp"

namespace gns {

struct InducedArgs {
    const uint64_t* flags;     // [num_chunks] (words past the last entry's chunk are not read)
    const int32_t* indices;
    int64_t num_entries;
    int64_t num_chunks;        // ceil(nnz / 64)
    int32_t* sums;             // [tiles + 1]
    int32_t tiles;
    ChunkRec* srec;            // [num_chunks + 1]: the last record only carries the total
    int32_t* s_nodes;
};

__global__ void __launch_bounds__(kBlock) k_induced_phase1(InducedArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const int64_t base = (int64_t) blockIdx.x * kTile;
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int64_t g = base + (int64_t) i * kBlock + threadIdx.x;
        if (g < a.num_chunks) sum += __popcll(a.flags[g]);
    }
    sum = block_sum(sum, smem);
    if (threadIdx.x == 0) a.sums[blockIdx.x] = sum;
}

// exclusive scan of the tile sums by one block (counts are kept as unsigned 32-bit values)
__global__ void __launch_bounds__(kBlock) k_induced_phase2(InducedArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    int32_t carry = 0;
    for (int32_t base = 0; base < a.tiles; base += kBlock) {
        const int32_t i = base + (int32_t) threadIdx.x;
        const int32_t v = (i < a.tiles) ? a.sums[i] : 0;
        int32_t total;
        const int32_t ex = block_exclusive_scan(v, smem, &total);
        if (i < a.tiles) a.sums[i] = (int32_t) ((uint32_t) carry + (uint32_t) ex);
        carry = (int32_t) ((uint32_t) carry + (uint32_t) total);
    }
    if (threadIdx.x == 0) a.sums[a.tiles] = carry;
}

__global__ void __launch_bounds__(kBlock) k_induced_phase3(InducedArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const int64_t g0 = (int64_t) blockIdx.x * kTile + (int64_t) threadIdx.x * kItems;
    uint64_t w[kItems];
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        w[i] = (g0 + i < a.num_chunks) ? a.flags[g0 + i] : 0ull;
        sum += __popcll(w[i]);
    }
    int32_t total;
    uint32_t before = (uint32_t) a.sums[blockIdx.x] + (uint32_t) block_exclusive_scan(sum, smem, &total);
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        if (g0 + i < a.num_chunks) {
            ChunkRec r;
            r.flags = w[i];
            r.before = before;
            r.pad = 0;
            a.srec[g0 + i] = r;
        }
        before += (uint32_t) __popcll(w[i]);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ChunkRec r;
        r.flags = 0ull;
        r.before = (uint32_t) a.sums[a.tiles];
        r.pad = 0;
        a.srec[a.num_chunks] = r;          // P(nnz) when nnz is a multiple of 64
    }
}

constexpr int kFillUnroll = 8;

// Compaction: lane l of a wave holds entry l of a chunk; flagged entries go to s_nodes in order.  Every
// wave takes an equal contiguous share of the chunks, kFillUnroll chunks in flight.
__global__ void __launch_bounds__(kBlock) k_induced_fill(InducedArgs a)
{
    const int lane = opaque_lane_id();
    const int64_t wave_global = (int64_t) blockIdx.x * (kBlock / kWave) +
                                __builtin_amdgcn_readfirstlane((int) (threadIdx.x >> 6));
    const int64_t num_waves = (int64_t) gridDim.x * (kBlock / kWave);
    const int64_t share = (a.num_chunks + num_waves - 1) / num_waves;
    const int64_t begin = wave_global * share;
    const int64_t end = begin + share < a.num_chunks ? begin + share : a.num_chunks;
    const uint64_t below = (1ull << lane) - 1ull;
    for (int64_t g = begin; g < end; g += kFillUnroll) {
        uint64_t w[kFillUnroll];
        uint32_t off[kFillUnroll];
        int32_t u[kFillUnroll];
#pragma unroll
        for (int i = 0; i < kFillUnroll; ++i) {
            const int64_t gi = g + i < end ? g + i : end - 1;            // wave-uniform, a valid chunk
            const ChunkRec r = a.srec[gi];
            w[i] = g + i < end ? r.flags : 0ull;
            off[i] = r.before;
            const int64_t e = (gi << 6) + lane;
            u[i] = a.indices[e < a.num_entries ? e : a.num_entries - 1];
        }
#pragma unroll
        for (int i = 0; i < kFillUnroll; ++i)
            if ((w[i] >> lane) & 1ull) a.s_nodes[(int64_t) off[i] + __popcll(w[i] & below)] = u[i];
    }
}

hipError_t launch_build_induced(gns_ctx* c, int cache_gen, hipStream_t s)
{
    const Layout& L = c->lay;
    InducedArgs a;
    a.flags = cache_ptr<uint64_t>(c, L.edge_flags, cache_gen);
    a.indices = c->graph.indices;
    a.num_entries = c->graph.num_entries;
    a.num_chunks = (c->graph.num_entries + 63) / 64;
    a.sums = ws_ptr<int32_t>(c, L.sums_chunks);
    a.tiles = (int32_t) ((a.num_chunks + kTile - 1) / kTile);
    a.srec = cache_ptr<ChunkRec>(c, L.srec, cache_gen);
    a.s_nodes = cache_ptr<int32_t>(c, L.s_nodes, cache_gen);
    hipLaunchKernelGGL(k_induced_phase1, dim3((unsigned) a.tiles), dim3(kBlock), 0, s, a);
    hipLaunchKernelGGL(k_induced_phase2, dim3(1), dim3(kBlock), 0, s, a);
    hipLaunchKernelGGL(k_induced_phase3, dim3((unsigned) a.tiles), dim3(kBlock), 0, s, a);
    int64_t blocks = (a.num_chunks + (kBlock / kWave) * kFillUnroll - 1) / ((kBlock / kWave) * kFillUnroll);
    const int64_t cap = (int64_t) c->num_cus * 16;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_induced_fill, dim3((unsigned) blocks), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

}  // namespace gns
