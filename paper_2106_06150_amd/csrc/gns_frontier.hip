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
#include <string.h>
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
// First kernel of a mini-batch: publishes the batch's scalars (number of seeds, Philox key, which hash map
// it uses, which copy of the cache structures it reads) in the device state, copies the seeds into the
// context and inserts them, with their local ids, into this batch's hash map.  The
// map is already empty: the context keeps two, and every batch empties the other one for its
// successor (see k_relabel_last).  A bad seed is reported by stamping the batch id, so no flag
// needs resetting while other blocks may be setting it.
__global__ void __launch_bounds__(kBlock) k_batch_begin(LayerArgs g, BeginDyn d)
{
    const int b = (int) blockIdx.y;
    char* ws = g.b[b].ws;
    DeviceState* st = at<DeviceState>(ws, g.off.state);
    const int parity = d.parity[b];
    const int32_t num_seeds = d.num_seeds[b];
    const int32_t* seeds = d.seeds[b];
    const uint32_t batch_id = d.batch_id[b];
    unsigned long long* slots = at<unsigned long long>(ws, g.off.hash_slots[parity]);
    uint32_t* slot_list = at<uint32_t>(ws, g.off.slot_list[parity]);
    RowExtent* row_ext = at<RowExtent>(ws, g.off.row_ext);
    int32_t* hub_rows = g.off.uses_cache ? at<int32_t>(ws, g.off.hub_rows) : nullptr;
    int32_t* seed_copy = at<int32_t>(ws, g.off.seed_copy);
    const int64_t t = (int64_t) blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0) {
        st->num_dst[0] = num_seeds;
        for (int l = 0; l < GNS_MAX_LAYERS; ++l) { st->num_edges[l] = 0; st->num_dst[l + 1] = 0; }
        st->key0 = d.key0[b];
        st->key1 = d.key1[b];
        st->hash_parity = parity;
        st->cache_gen = d.cache_gen[b];
    }
    for (int64_t q = t; q < num_seeds; q += (int64_t) gridDim.x * blockDim.x) {
        const int32_t u = seeds[q];
        const bool in_range = u >= 0 && (int64_t) u < g.f.num_nodes;
        RowExtent ext = {0, 0};
        if (in_range) {
            ext.start = load_off_rt(g.f.g_indptr, g.f.g_i64, u);
            ext.end = load_off_rt(g.f.g_indptr, g.f.g_i64, (int64_t) u + 1);
        }
        seed_copy[q] = u;
        row_ext[q] = ext;
        append_hub_rows(st, hub_rows, is_hub_extent(ext.start, ext.end), (int32_t) q);
        const int64_t slot = in_range ? hash_insert(slots, g.f.hmask, g.f.hshift, (uint32_t) u, (uint32_t) q) : -1;
        slot_list[q] = slot >= 0 ? (uint32_t) slot : 0xFFFFFFFFu;
        if (slot < 0) st->bad_seed = batch_id;
    }
}

const void* batch_first_kernel() { return reinterpret_cast<const void*>(&k_batch_begin); }

void fill_group_args(const Group& g, LayerArgs* out)
{
    gns_ctx* c = g.ctx[0];
    const Layout& L = c->lay;
    memset(out, 0, sizeof(*out));
    WsOffsets& o = out->off;
    o.mark_summary = L.mark_summary;
    o.has_summary = L.summary_words > 0 ? 1 : 0;
    o.state = L.state; o.mark = L.mark_bitmap; o.seed_copy = L.seed_copy; o.row_ext = L.row_ext; o.hub_rows = L.hub_rows;
    for (int p = 0; p < 2; ++p) {
        o.slot_list[p] = L.slot_list[p]; o.hash_slots[p] = L.hash_slots[p];
        o.s_nbr[p] = L.s_nbr[p]; o.s_w[p] = L.s_w[p]; o.s_cnt[p] = L.s_cnt[p];
    }
    o.plan_cnt = L.plan_cnt; o.plan_g0 = L.plan_g0; o.plan_desc = L.plan_desc;
    o.sums_rows = L.sums_rows; o.sums_marks = L.sums_marks; o.sums_plan = L.sums_plan;
    o.cache_block_bytes = L.cache_block_bytes;
    o.uses_cache = c->uses_cache ? 1 : 0;
    for (int b = 0; b < kMaxGroup; ++b) out->b[b].ws = g.ctx[b < g.count ? b : 0]->ws;
}

static inline BlockPtrs block_ptrs(const gns_block& k)
{
    BlockPtrs p;
    p.indptr = k.indptr; p.indices = k.indices; p.src_nodes = k.src_nodes; p.row_eligible = k.row_eligible; p.weights = k.weights;
    return p;
}

void set_group_layer(const Group& g, int layer_index, LayerArgs* out)
{
    for (int b = 0; b < g.count; ++b) {
        gns_ctx* c = g.ctx[b];
        BatchSlot& q = out->b[b];
        const int32_t* seed_copy = ws_ptr<int32_t>(c, c->lay.seed_copy);
        const gns_block* blk = g.blocks[b];
        q.dst = layer_index == 0 ? seed_copy : blk[layer_index - 1].src_nodes;
        q.prev_dst = layer_index <= 1 ? seed_copy : blk[layer_index - 2].src_nodes;
        q.cur = block_ptrs(blk[layer_index]);
        q.prev = block_ptrs(blk[layer_index > 0 ? layer_index - 1 : 0]);
    }
}

// Enqueues the first kernel of a group of mini-batches.
hipError_t launch_batch_begin(const Group& g, const BeginDyn& d, hipStream_t s)
{
    gns_ctx* c = g.ctx[0];
    LayerArgs a;
    fill_group_args(g, &a);
    fill_finish_template(c, 0, &a.f);
    // the grid is sized for the largest batch: the same launch serves every replay
    const unsigned grid = (unsigned) ((c->config.max_seeds + kBlock - 1) / kBlock);
    hipLaunchKernelGGL(k_batch_begin, dim3(grid, (unsigned) g.count), dim3(kBlock), 0, s, a, d);
    return hipGetLastError();
}

// Words first .. first + per - 1 of a tile that starts at word `base` (per <= kPerMax consecutive words of one
// thread; they never straddle a summary word because per divides 64 and first is a multiple of per).  With a
// summary only the words it reports as marked are read; the reads are issued together, behind one read of
// the summary word.
template <int kPerMax>
__device__ __forceinline__ void load_marks(const FinishArgs& a, int64_t base, int first, int per, int T, uint64_t* word)
{
    uint64_t has = ~0ull;
    const int64_t w0 = base + first;
    if (a.mark_summary && first < T && w0 < a.words) has = a.mark_summary[w0 >> 6] >> (w0 & 63);
#pragma unroll
    for (int i = 0; i < kPerMax; ++i) {
        const int64_t w = w0 + i;
        const bool live = i < per && first + i < T && w < a.words && ((has >> i) & 1ull);
        word[i] = live ? a.mark[w] : 0ull;
    }
}

// ---------------------------------------------------------------------------
template <int kPerMax>
__global__ void __launch_bounds__(kBlock) k_finish_phase1(LayerArgs g)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const FinishArgs a = bind_finish(g, (int) blockIdx.y, true);
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
        const int T = a.mark_tile_words;
        const int per = T > kBlock ? T / kBlock : 1;
        uint64_t word[kPerMax];
        load_marks<kPerMax>(a, base, (int) threadIdx.x * per, per, T, word);
        int32_t sum = 0;
#pragma unroll
        for (int i = 0; i < kPerMax; ++i) sum += __popcll(word[i]);
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
template <int kPerMax>
__global__ void __launch_bounds__(kBlock) k_finish_phase3(LayerArgs g)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const FinishArgs a = bind_finish(g, (int) blockIdx.y, true);
    // the tile's marked words, kMarkCap at a time: the word, its index in the tile, the number of marks before it
    __shared__ uint64_t s_word[kMarkCap];
    __shared__ int32_t s_widx[kMarkCap];
    __shared__ int32_t s_off[kMarkCap];
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
        const int per = T > kBlock ? T / kBlock : 1;
        const int first = (int) threadIdx.x * per;
        uint64_t word[kPerMax];
        load_marks<kPerMax>(a, base, first, per, T, word);
        int32_t cnt = 0, nz = 0;
#pragma unroll
        for (int i = 0; i < kPerMax; ++i) {
            cnt += __popcll(word[i]);
            nz += word[i] ? 1 : 0;
            if (word[i]) a.mark[base + first + i] = 0ull;            // ready for the next layer
        }
        int32_t total, total_nz;
        const int32_t off = block_exclusive_scan(cnt, smem, &total);        // marks before this thread's words
        const int32_t widx = block_exclusive_scan(nz, smem, &total_nz);     // marked words before them
        __syncthreads();
        // every thread has read its summary words: clear them (a tile is a whole number of summary words)
        if (a.mark_summary)
            for (int i = (int) threadIdx.x; i < T / 64; i += kBlock)
                if (base / 64 + i < (a.words + 63) / 64) a.mark_summary[base / 64 + i] = 0ull;
        // The marked words go through LDS in order, kMarkCap at a time (most tiles need one pass).
        for (int32_t p0 = 0; p0 < total_nz; p0 += kMarkCap) {
            int32_t my = widx, my_off = off;
#pragma unroll
            for (int i = 0; i < kPerMax; ++i) {
                if (word[i]) {
                    if (my >= p0 && my < p0 + kMarkCap) {
                        s_word[my - p0] = word[i];
                        s_widx[my - p0] = first + i;
                        s_off[my - p0] = my_off;
                    }
                    ++my;
                    my_off += __popcll(word[i]);
                }
            }
            __syncthreads();
            const int32_t in_pass = total_nz - p0 < kMarkCap ? total_nz - p0 : kMarkCap;
            const int32_t node_lo = s_off[0];
            const int32_t node_hi = s_off[in_pass - 1] + __popcll(s_word[in_pass - 1]);
            // one thread per new node: locate its word (last word whose offset is <= j), then its bit
            for (int32_t j = node_lo + (int32_t) threadIdx.x; j < node_hi; j += kBlock) {
                int32_t lo = 0, hi = in_pass;                            // answer in [lo, hi)
                while (hi - lo > 1) {
                    const int32_t mid = (lo + hi) >> 1;
                    if (s_off[mid] <= j) lo = mid; else hi = mid;
                }
                const int bit = select_bit64(s_word[lo], j - s_off[lo]);
                const uint32_t node = (uint32_t) ((base + s_widx[lo]) * 64 + bit);
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
            __syncthreads();
        }
    }
}

void fill_finish_template(gns_ctx* c, int layer_index, FinishArgs* out)
{
    const Layout& L = c->lay;
    FinishArgs& a = *out;
    memset(&a, 0, sizeof(a));
    a.layer_index = layer_index;
    a.fanout = c->config.fanout[layer_index];
    a.words = L.words;
    a.hmask = L.hash_cap - 1;
    a.hshift = 32u - (uint32_t) __builtin_ctz(L.hash_cap);
    a.row_tiles_max = (int32_t) ((L.rows[layer_index] + kTile - 1) / kTile);
    a.mark_tiles = (int32_t) L.mark_tiles;
    a.mark_tile_words = L.mark_tile_words;
    a.max_slots = L.rows[layer_index] * (int64_t) a.fanout;
    a.g_indptr = c->graph.indptr;
    a.g_i64 = c->graph.indptr_is_i64;
    a.num_nodes = c->graph.num_nodes;
}

int relabel_grid(const gns_ctx* c, int layer_index)
{
    const int64_t max_slots = c->lay.rows[layer_index] * (int64_t) c->config.fanout[layer_index];
    int64_t rb = (max_slots + kBlock - 1) / kBlock;
    if (rb > (int64_t) c->num_cus * 8) rb = (int64_t) c->num_cus * 8;
    if (rb < 1) rb = 1;
    return (int) rb;
}

// Phases 1 and 3 of a layer (the relabel rides with the next layer's first kernel).
hipError_t launch_finish_layer(const Group& g, int layer_index, hipStream_t s)
{
    gns_ctx* c = g.ctx[0];
    LayerArgs a;
    fill_group_args(g, &a);
    set_group_layer(g, layer_index, &a);
    fill_finish_template(c, layer_index, &a.f);
    const dim3 grid((unsigned) (a.f.row_tiles_max + a.f.mark_tiles), (unsigned) g.count);
    // words of a tile per thread: the kernels' loops over them are unrolled for 1, 4 or 32
    const int per = a.f.mark_tile_words / kBlock;
    if (per <= 1) {
        hipLaunchKernelGGL(k_finish_phase1<1>, grid, dim3(kBlock), 0, s, a);
        hipLaunchKernelGGL(k_finish_phase3<1>, grid, dim3(kBlock), 0, s, a);
    } else if (per <= 4) {
        hipLaunchKernelGGL(k_finish_phase1<4>, grid, dim3(kBlock), 0, s, a);
        hipLaunchKernelGGL(k_finish_phase3<4>, grid, dim3(kBlock), 0, s, a);
    } else {
        hipLaunchKernelGGL((k_finish_phase1<kMarkTileMax / kBlock>), grid, dim3(kBlock), 0, s, a);
        hipLaunchKernelGGL((k_finish_phase3<kMarkTileMax / kBlock>), grid, dim3(kBlock), 0, s, a);
    }
    return hipGetLastError();
}

// The last layer's relabel has no following sampler to ride with; its launch also leaves the context's
// other hash map empty for the next mini-batch (nothing in this batch touches that map).  The map was
// filled by the batch before this one; every insertion recorded its slot, so emptying it means
// resetting exactly those slots -- a few hundred KB instead of the whole table.
__global__ void __launch_bounds__(kBlock) k_relabel_last(LayerArgs g, int total_layers)
{
    const FinishArgs a = bind_finish(g, (int) blockIdx.y, true);
    relabel_body(a, blockIdx.x, gridDim.x);
    const int32_t stale = a.st->map_nodes[a.parity ^ 1];
    const size_t stride = (size_t) gridDim.x * kBlock;
    for (size_t i = (size_t) blockIdx.x * kBlock + threadIdx.x; i < (size_t) stale; i += stride) {
        const uint32_t slot = a.other_slot_list[i];
        if (slot != 0xFFFFFFFFu) a.other_slots[slot] = kEmptySlot;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        a.st->hub_count = 0;                                     // the next batch starts a new hub list
        a.st->map_nodes[a.parity] = a.st->num_dst[total_layers]; // what the clear of this batch's map will have to undo
    }
}

hipError_t launch_relabel(const Group& g, int layer_index, hipStream_t s)
{
    gns_ctx* c = g.ctx[0];
    LayerArgs a;
    fill_group_args(g, &a);
    set_group_layer(g, layer_index, &a);
    fill_finish_template(c, layer_index, &a.f);
    hipLaunchKernelGGL(k_relabel_last, dim3((unsigned) relabel_grid(c, layer_index), (unsigned) g.count), dim3(kBlock), 0, s, a,
                       (int) c->config.num_layers);
    return hipGetLastError();
}

}  // namespace gns
