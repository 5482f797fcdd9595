// Frontier union and relabelling (paper Algorithm 1, top-down loop:
// B^{l-1} <- B^{l-1} U N_l(u)), turned into a block CSR per layer.
//
// The sampler leaves, per dst row, up to k global neighbor ids at a fixed
// stride and has set one bit per sampled id in a node-indexed mark bitmap.
// Here:
//   begin    the batch's first kernel: scalars, seeds with their local ids into the batch's
//            hash map, the seeds' CSR extents and hub entries
//   phase 1  per-tile sums of the row counts and of the mark bitmap's
//            population (the sampler marks only ids without a local id)
//   phase 3  every block adds up the sums of the tiles before its own, scans
//            its tile and writes: indptr for row tiles; for bitmap tiles the
//            marked ids in ascending order behind the dst prefix, one thread
//            per new id, each inserted into the hash map with its local id, its
//            CSR extent recorded; the bitmap words are cleared for the next layer
//   relabel  every sampled edge looks its neighbor's local id up and is
//            compacted to its CSR position (inside the next layer's first sampler
//            launch; the last layer's own launch also empties the hash map the
//            next batch will use)
// Sorted order comes from walking the bitmap, so the result does not depend on
// the order in which threads ran.
#include "gns_kernels.hpp"

namespace gns {

__global__ void k_fill_u64(unsigned long long* p, size_t n, unsigned long long v)
{
    size_t i = (size_t) blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t) gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

__global__ void k_fill_u32(uint32_t* p, size_t n, uint32_t v)
{
    size_t i = (size_t) blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t) gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

static inline unsigned fill_grid(size_t n)
{
    size_t b = (n + kBlock - 1) / kBlock;
    if (b > 4096) b = 4096;
    if (b < 1) b = 1;
    return (unsigned) b;
}

hipError_t launch_fill_u64(unsigned long long* p, size_t n, unsigned long long v, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_u64, dim3(fill_grid(n)), dim3(kBlock), 0, s, p, n, v);
    return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_u32, dim3(fill_grid(n)), dim3(kBlock), 0, s, p, n, v);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// First kernel of a mini-batch: publishes the batch's scalars (number of seeds, Philox key) in
// the device state, copies the seeds into the context and inserts them, with their local ids, into
// this batch's hash map.  The
// map is already empty: the context keeps two, and every batch empties the other one for its
// successor (see k_relabel_last).  A bad seed is reported by stamping the batch id, so no flag
// needs resetting while other blocks may be setting it.
struct BeginArgs {
    unsigned long long* slots;
    DeviceState* st;
    const int32_t* seeds;
    int64_t num_nodes;
    uint32_t hmask, hshift;
    RowExtent* row_ext;
    const void* g_indptr;
    int g_i64;
    int32_t* hub_rows;
    int32_t* seed_copy;
    uint32_t* slot_list;
};

__global__ void __launch_bounds__(kBlock) k_batch_begin(BeginArgs a, int32_t num_seeds, uint32_t key0, uint32_t key1,
                                                        uint32_t batch_id)
{
    const int64_t t = (int64_t) blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0) {
        a.st->num_dst[0] = num_seeds;
        for (int l = 0; l < GNS_MAX_LAYERS; ++l) { a.st->num_edges[l] = 0; a.st->num_dst[l + 1] = 0; }
        a.st->key0 = key0;
        a.st->key1 = key1;
    }
    for (int64_t q = t; q < num_seeds; q += (int64_t) gridDim.x * blockDim.x) {
        const int32_t u = a.seeds[q];
        const bool in_range = u >= 0 && (int64_t) u < a.num_nodes;
        RowExtent ext = {0, 0};
        if (in_range) {
            ext.start = load_off_rt(a.g_indptr, a.g_i64, u);
            ext.end = load_off_rt(a.g_indptr, a.g_i64, (int64_t) u + 1);
        }
        a.seed_copy[q] = u;
        a.row_ext[q] = ext;
        append_hub_rows(a.st, a.hub_rows, is_hub_extent(ext.start, ext.end), (int32_t) q);
        const int64_t slot = in_range ? hash_insert(a.slots, a.hmask, a.hshift, (uint32_t) u, (uint32_t) q) : -1;
        a.slot_list[q] = slot >= 0 ? (uint32_t) slot : 0xFFFFFFFFu;
        if (slot < 0) a.st->bad_seed = batch_id;
    }
}

const void* batch_first_kernel() { return reinterpret_cast<const void*>(&k_batch_begin); }

static inline unsigned long long* batch_hash(gns_ctx* c) { return ws_ptr<unsigned long long>(c, c->lay.hash_slots[c->hash_parity]); }

void fill_begin_args(gns_ctx* c, const int32_t* seeds, BeginArgsHost* out)
{
    const Layout& L = c->lay;
    BeginArgs* a = reinterpret_cast<BeginArgs*>(out->bytes);
    static_assert(sizeof(BeginArgs) <= sizeof(out->bytes), "BeginArgsHost too small");
    a->slots = batch_hash(c);
    a->st = c->d_state;
    a->seeds = seeds;
    a->num_nodes = c->graph.num_nodes;
    a->hmask = L.hash_cap - 1;
    a->hshift = 32u - (uint32_t) __builtin_ctz(L.hash_cap);
    a->row_ext = ws_ptr<RowExtent>(c, L.row_ext);
    a->g_indptr = c->graph.indptr;
    a->g_i64 = c->graph.indptr_is_i64;
    a->hub_rows = c->uses_cache ? ws_ptr<int32_t>(c, L.hub_rows) : nullptr;
    a->seed_copy = ws_ptr<int32_t>(c, L.seed_copy);
    a->slot_list = ws_ptr<uint32_t>(c, L.slot_list[c->hash_parity]);
}

hipError_t launch_batch_begin(gns_ctx* c, uint64_t seed, const int32_t* seeds, int32_t num_seeds, uint32_t batch_id,
                              hipStream_t s)
{
    BeginArgsHost h;
    fill_begin_args(c, seeds, &h);
    const BeginArgs a = *reinterpret_cast<const BeginArgs*>(h.bytes);
    // the grid is sized for the largest batch: the same launch serves every replay
    const unsigned grid = (unsigned) ((c->config.max_seeds + kBlock - 1) / kBlock);
    hipLaunchKernelGGL(k_batch_begin, dim3(grid), dim3(kBlock), 0, s, a, num_seeds, (uint32_t) seed,
                       (uint32_t) (seed >> 32), batch_id);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlock) k_finish_phase1(FinishArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const int32_t R = a.st->num_dst[a.layer_index];
    if ((int32_t) blockIdx.x < a.row_tiles_max) {
        const int64_t base = (int64_t) blockIdx.x * kTile;
        if (base >= R) return;
        int32_t sum = 0;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const int64_t r = base + (int64_t) i * kBlock + threadIdx.x;
            if (r < R) sum += a.s_cnt[r];
        }
        sum = block_sum(sum, smem);
        if (threadIdx.x == 0) a.sums_rows[blockIdx.x] = sum;
    } else {
        const int32_t tile = (int32_t) blockIdx.x - a.row_tiles_max;
        const int64_t base = (int64_t) tile * a.mark_tile_words;
        int32_t sum = 0;
        for (int i = (int) threadIdx.x; i < a.mark_tile_words; i += kBlock)
            if (base + i < a.words) sum += __popcll(a.mark[base + i]);
        sum = block_sum(sum, smem);
        if (threadIdx.x == 0) a.sums_marks[tile] = sum;
    }
}

// sum of vals[0..count) by the whole block
__device__ __forceinline__ int32_t block_sum_array(const int32_t* vals, int32_t count, int32_t* smem)
{
    int32_t v = 0;
    for (int32_t t = (int32_t) threadIdx.x; t < count; t += kBlock) v += vals[t];
    return block_sum(v, smem);
}

// Phase 3 needs each tile's offset = the sum of the earlier tiles' sums.  Every block adds
// those up itself (at most a few thousand values), which saves a single-block scan kernel.
__global__ void __launch_bounds__(kBlock) k_finish_phase3(FinishArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    __shared__ int32_t s_off[kMarkTileMax + 1];
    __shared__ uint64_t s_word[kMarkTileMax];
    const int32_t R = a.st->num_dst[a.layer_index];
    const int32_t row_tiles = (R + kTile - 1) / kTile;
    if ((int32_t) blockIdx.x < a.row_tiles_max) {
        const int64_t base = (int64_t) blockIdx.x * kTile;
        if (base >= R) return;
        const int32_t before = block_sum_array(a.sums_rows, (int32_t) blockIdx.x, smem);
        // blocked arrangement: thread t owns rows base + t*kItems .. +kItems
        int32_t c[kItems];
        int32_t sum = 0;
        const int64_t r0 = base + (int64_t) threadIdx.x * kItems;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            c[i] = (r0 + i < R) ? a.s_cnt[r0 + i] : 0;
            sum += c[i];
        }
        int32_t total;
        int32_t off = before + block_exclusive_scan(sum, smem, &total);
        if ((int32_t) blockIdx.x == row_tiles - 1 && threadIdx.x == 0) {
            a.st->num_edges[a.layer_index] = before + total;
            a.indptr[R] = before + total;
        }
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            if (r0 + i < R) {
                a.indptr[r0 + i] = off;
                a.src_nodes[r0 + i] = a.dst_nodes[r0 + i];
            }
            off += c[i];
        }
    } else {
        const int32_t tile = (int32_t) blockIdx.x - a.row_tiles_max;
        const int T = a.mark_tile_words;
        const int64_t base = (int64_t) tile * T;
        const int32_t before = block_sum_array(a.sums_marks, tile, smem);
        const int32_t here = a.sums_marks[tile];
        if (tile == a.mark_tiles - 1 && threadIdx.x == 0) a.st->num_dst[a.layer_index + 1] = R + before + here;
        if (here == 0) return;
        // thread t owns words t*per .. t*per+per-1 of the tile (per = 1 for tiles of up to kBlock words);
        // exclusive offsets of the tile's words into LDS
        constexpr int kPerMax = kMarkTileMax / kBlock;
        const int per = T > kBlock ? T / kBlock : 1;
        const int first = (int) threadIdx.x * per;
        uint64_t word[kPerMax];
        int32_t cnt = 0;
#pragma unroll
        for (int i = 0; i < kPerMax; ++i) {
            const int64_t w = base + first + i;
            word[i] = (i < per && first + i < T && w < a.words) ? a.mark[w] : 0ull;
            cnt += __popcll(word[i]);
        }
        int32_t total;
        int32_t off = block_exclusive_scan(cnt, smem, &total);
#pragma unroll
        for (int i = 0; i < kPerMax; ++i) {
            if (i < per && first + i < T) {
                s_off[first + i] = off;
                s_word[first + i] = word[i];
                off += __popcll(word[i]);
                if (word[i]) a.mark[base + first + i] = 0ull;        // ready for the next layer
            }
        }
        if (threadIdx.x == 0) s_off[T] = total;
        __syncthreads();
        // one thread per new node: locate its word (last word whose offset is <= j), then its bit
        for (int32_t j = (int32_t) threadIdx.x; j < total; j += kBlock) {
            int32_t lo = 0, hi = T;                                  // answer in [lo, hi)
            while (hi - lo > 1) {
                const int32_t mid = (lo + hi) >> 1;
                if (s_off[mid] <= j) lo = mid; else hi = mid;
            }
            const int bit = select_bit64(s_word[lo], j - s_off[lo]);
            const uint32_t node = (uint32_t) ((base + lo) * 64 + bit);
            const int32_t pos = R + before + j;
            RowExtent ext;
            ext.start = load_off_rt(a.g_indptr, a.g_i64, node);
            ext.end = load_off_rt(a.g_indptr, a.g_i64, (int64_t) node + 1);
            a.src_nodes[pos] = (int32_t) node;
            a.row_ext[pos] = ext;
            append_hub_rows(a.st, a.hub_rows, is_hub_extent(ext.start, ext.end), pos);
            const int64_t slot = hash_insert(a.slots, a.hmask, a.hshift, node, (uint32_t) pos);
            a.slot_list[pos] = slot >= 0 ? (uint32_t) slot : 0xFFFFFFFFu;
        }
    }
}

void fill_finish_args(gns_ctx* c, int layer_index, const int32_t* dst_nodes, const gns_block* blk, FinishArgs* out)
{
    const Layout& L = c->lay;
    FinishArgs& a = *out;
    const int par = layer_index & 1;                 // sampler scratch is double-buffered by layer parity
    a.st = c->d_state;
    a.layer_index = layer_index;
    a.fanout = c->config.fanout[layer_index];
    a.dst_nodes = dst_nodes;
    a.s_nbr = ws_ptr<int32_t>(c, L.s_nbr[par]);
    a.s_w = ws_ptr<float>(c, L.s_w[par]);
    a.s_cnt = ws_ptr<int32_t>(c, L.s_cnt[par]);
    a.mark = ws_ptr<uint64_t>(c, L.mark_bitmap);
    a.words = L.words;
    a.slots = batch_hash(c);
    a.hmask = L.hash_cap - 1;
    a.hshift = 32u - (uint32_t) __builtin_ctz(L.hash_cap);
    a.sums_rows = ws_ptr<int32_t>(c, L.sums_rows);
    a.sums_marks = ws_ptr<int32_t>(c, L.sums_marks);
    a.row_tiles_max = (int32_t) ((L.rows[layer_index] + kTile - 1) / kTile);
    a.mark_tiles = (int32_t) L.mark_tiles;
    a.mark_tile_words = L.mark_tile_words;
    a.indptr = blk->indptr;
    a.indices = blk->indices;
    a.weights = blk->weights;
    a.src_nodes = blk->src_nodes;
    a.max_slots = L.rows[layer_index] * (int64_t) a.fanout;
    a.row_ext = ws_ptr<RowExtent>(c, L.row_ext);
    a.g_indptr = c->graph.indptr;
    a.g_i64 = c->graph.indptr_is_i64;
    a.hub_rows = c->uses_cache ? ws_ptr<int32_t>(c, L.hub_rows) : nullptr;
    a.slot_list = ws_ptr<uint32_t>(c, L.slot_list[c->hash_parity]);
    a.parity = c->hash_parity;
}

int relabel_grid(const gns_ctx* c, int layer_index)
{
    const int64_t max_slots = c->lay.rows[layer_index] * (int64_t) c->config.fanout[layer_index];
    int64_t rb = (max_slots + kBlock - 1) / kBlock;
    if (rb > (int64_t) c->num_cus * 16) rb = (int64_t) c->num_cus * 16;
    if (rb < 1) rb = 1;
    return (int) rb;
}

// Phases 1 and 3 of a layer (the relabel rides with the next layer's first kernel).
hipError_t launch_finish_layer(gns_ctx* c, int layer_index, const int32_t* dst_nodes, gns_block* blk, hipStream_t s)
{
    FinishArgs a;
    fill_finish_args(c, layer_index, dst_nodes, blk, &a);
    const unsigned grid = (unsigned) (a.row_tiles_max + a.mark_tiles);
    hipLaunchKernelGGL(k_finish_phase1, dim3(grid), dim3(kBlock), 0, s, a);
    hipLaunchKernelGGL(k_finish_phase3, dim3(grid), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

// The last layer's relabel has no following sampler to ride with; its launch also leaves the context's
// other hash map empty for the next mini-batch (nothing in this batch touches that map).  The map was
// filled by the batch before this one; every insertion recorded its slot, so emptying it means
// resetting exactly those slots -- a few hundred KB instead of the whole table.
__global__ void __launch_bounds__(kBlock) k_relabel_last(FinishArgs a, unsigned long long* other_slots,
                                                         const uint32_t* other_slot_list, int total_layers)
{
    relabel_body(a, blockIdx.x, gridDim.x);
    const int32_t stale = a.st->map_nodes[a.parity ^ 1];
    const size_t stride = (size_t) gridDim.x * kBlock;
    for (size_t i = (size_t) blockIdx.x * kBlock + threadIdx.x; i < (size_t) stale; i += stride) {
        const uint32_t slot = other_slot_list[i];
        if (slot != 0xFFFFFFFFu) other_slots[slot] = kEmptySlot;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        a.st->hub_count = 0;                                     // the next batch starts a new hub list
        a.st->map_nodes[a.parity] = a.st->num_dst[total_layers]; // what the clear of this batch's map will have to undo
    }
}

hipError_t launch_relabel(gns_ctx* c, int layer_index, const int32_t* dst_nodes, gns_block* blk, hipStream_t s)
{
    FinishArgs a;
    fill_finish_args(c, layer_index, dst_nodes, blk, &a);
    const int other = c->hash_parity ^ 1;
    hipLaunchKernelGGL(k_relabel_last, dim3((unsigned) relabel_grid(c, layer_index)), dim3(kBlock), 0, s, a,
                       ws_ptr<unsigned long long>(c, c->lay.hash_slots[other]),
                       ws_ptr<uint32_t>(c, c->lay.slot_list[other]), (int) c->config.num_layers);
    return hipGetLastError();
}

}  // namespace gns
