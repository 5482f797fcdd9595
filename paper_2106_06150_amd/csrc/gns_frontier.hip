// Frontier union and relabelling (paper Algorithm 1, top-down loop:
// B^{l-1} <- B^{l-1} U N_l(u)), turned into a block CSR per layer.
//
// The sampler leaves, per dst row, up to k global neighbor ids at a fixed
// stride and has set one bit per sampled id in a node-indexed mark bitmap.
// Here:
//   phase 1  per-tile sums of the row counts, and of the mark bitmap's
//            population after removing ids that already have a local id
//            (the dst nodes, found through the batch's hash map)
//   phase 2  one block scans both arrays of tile sums and publishes the
//            layer's edge and src counts
//   phase 3  tiles are scanned again with their offsets: indptr is written,
//            the marked ids are emitted in ascending order behind the dst
//            prefix, inserted into the hash map with their local ids, and the
//            bitmap words are cleared for the next layer
//   relabel  every sampled edge looks its neighbor's local id up and is
//            compacted to its CSR position
// Sorted order comes from walking the bitmap, so the result does not depend on
// the order in which threads ran.
#include "gns_internal.h"
#include "gns_device.hpp"

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
__global__ void k_batch_clear(unsigned long long* slots, size_t cap, DeviceState* st, int32_t num_seeds)
{
    size_t i = (size_t) blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t) gridDim.x * blockDim.x;
    if (i == 0) {
        st->num_dst[0] = num_seeds;
        for (int l = 0; l < GNS_MAX_LAYERS; ++l) { st->queue[l] = 0; st->num_edges[l] = 0; st->num_dst[l + 1] = 0; }
        st->bad_seed = 0;
    }
    for (; i < cap; i += stride) slots[i] = kEmptySlot;
}

__global__ void k_seed_insert(unsigned long long* slots, uint32_t mask, uint32_t shift, const int32_t* seeds,
                              int32_t num_seeds, int64_t n, DeviceState* st)
{
    const int32_t i = (int32_t) (blockIdx.x * blockDim.x + threadIdx.x);
    if (i >= num_seeds) return;
    const int32_t u = seeds[i];
    if (u < 0 || (int64_t) u >= n) { st->bad_seed = 1; return; }
    if (!hash_insert(slots, mask, shift, (uint32_t) u, (uint32_t) i)) st->bad_seed = 1;
}

hipError_t launch_batch_begin(gns_ctx* c, const int32_t* seeds, int32_t num_seeds, hipStream_t s)
{
    const Layout& L = c->lay;
    unsigned long long* slots = ws_ptr<unsigned long long>(c, L.hash_slots);
    hipLaunchKernelGGL(k_batch_clear, dim3(fill_grid(L.hash_cap)), dim3(kBlock), 0, s, slots, (size_t) L.hash_cap,
                       c->d_state, num_seeds);
    const uint32_t mask = L.hash_cap - 1;
    const uint32_t shift = 32u - (uint32_t) __builtin_ctz(L.hash_cap);
    hipLaunchKernelGGL(k_seed_insert, dim3((num_seeds + kBlock - 1) / kBlock), dim3(kBlock), 0, s, slots, mask, shift,
                       seeds, num_seeds, c->graph.num_nodes, c->d_state);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
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
    int32_t* sums_words;           // [word_tiles + 1]
    int32_t row_tiles_max;         // grid split point: blocks [0, row_tiles_max) work on rows
    int32_t word_tiles;
    int32_t* indptr;               // block outputs
    int32_t* indices;
    float* weights;
    int32_t* src_nodes;
};

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
        const int64_t base = (int64_t) tile * kTile;
        int32_t sum = 0;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const int64_t w = base + (int64_t) i * kBlock + threadIdx.x;
            if (w < a.words) {
                uint64_t word = a.mark[w];
                if (word) {
                    // drop ids that already own a local id (they are dst nodes of this layer)
                    uint64_t rest = word;
                    while (rest) {
                        const int bit = __builtin_ctzll(rest);
                        rest &= rest - 1;
                        const uint32_t node = (uint32_t) (w * 64 + bit);
                        if (hash_lookup(a.slots, a.hmask, a.hshift, node) >= 0) word &= ~(1ull << bit);
                    }
                    a.mark[w] = word;
                    sum += __popcll(word);
                }
            }
        }
        sum = block_sum(sum, smem);
        if (threadIdx.x == 0) a.sums_words[tile] = sum;
    }
}

// exclusive scan of vals[0..count) in place by one block; returns the total in every thread
__device__ int32_t scan_in_place(int32_t* vals, int32_t count, int32_t* smem)
{
    int32_t carry = 0;
    for (int32_t base = 0; base < count; base += kBlock) {
        const int32_t i = base + (int32_t) threadIdx.x;
        const int32_t v = (i < count) ? vals[i] : 0;
        int32_t total;
        const int32_t ex = block_exclusive_scan(v, smem, &total);
        if (i < count) vals[i] = carry + ex;
        carry += total;
    }
    return carry;
}

__global__ void __launch_bounds__(kBlock) k_finish_phase2(FinishArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const int32_t R = a.st->num_dst[a.layer_index];
    const int32_t row_tiles = (R + kTile - 1) / kTile;
    const int32_t edges = scan_in_place(a.sums_rows, row_tiles, smem);
    const int32_t fresh = scan_in_place(a.sums_words, a.word_tiles, smem);
    if (threadIdx.x == 0) {
        a.st->num_edges[a.layer_index] = edges;
        a.st->num_dst[a.layer_index + 1] = R + fresh;
        a.indptr[R] = edges;
    }
}

__global__ void __launch_bounds__(kBlock) k_finish_phase3(FinishArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const int32_t R = a.st->num_dst[a.layer_index];
    if ((int32_t) blockIdx.x < a.row_tiles_max) {
        const int64_t base = (int64_t) blockIdx.x * kTile;
        if (base >= R) return;
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
        int32_t off = a.sums_rows[blockIdx.x] + block_exclusive_scan(sum, smem, &total);
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
        const int64_t base = (int64_t) tile * kTile;
        uint64_t word[kItems];
        int32_t sum = 0;
        const int64_t w0 = base + (int64_t) threadIdx.x * kItems;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            word[i] = (w0 + i < a.words) ? a.mark[w0 + i] : 0ull;
            sum += __popcll(word[i]);
        }
        int32_t total;
        int32_t pos = R + a.sums_words[tile] + block_exclusive_scan(sum, smem, &total);
        if (total == 0) return;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            uint64_t rest = word[i];
            if (rest) {
                while (rest) {
                    const int bit = __builtin_ctzll(rest);
                    rest &= rest - 1;
                    const uint32_t node = (uint32_t) ((w0 + i) * 64 + bit);
                    a.src_nodes[pos] = (int32_t) node;
                    hash_insert(a.slots, a.hmask, a.hshift, node, (uint32_t) pos);
                    ++pos;
                }
                a.mark[w0 + i] = 0ull;
            }
        }
    }
}

__global__ void __launch_bounds__(kBlock) k_relabel(FinishArgs a, int64_t max_slots)
{
    const int32_t R = a.st->num_dst[a.layer_index];
    const int64_t limit = (int64_t) R * a.fanout;
    int64_t t = (int64_t) blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t) gridDim.x * blockDim.x;
    for (; t < limit && t < max_slots; t += stride) {
        const int32_t row = (int32_t) (t / a.fanout);
        const int32_t s = (int32_t) (t - (int64_t) row * a.fanout);
        if (s < a.s_cnt[row]) {
            const int32_t u = a.s_nbr[t];
            const int32_t o = a.indptr[row] + s;
            a.indices[o] = hash_lookup(a.slots, a.hmask, a.hshift, (uint32_t) u);
            a.weights[o] = a.s_w[t];
        }
    }
}

hipError_t launch_finish_layer(gns_ctx* c, int layer_index, const int32_t* dst_nodes, gns_block* blk, hipStream_t s)
{
    const Layout& L = c->lay;
    FinishArgs a;
    a.st = c->d_state;
    a.layer_index = layer_index;
    a.fanout = c->config.fanout[layer_index];
    a.dst_nodes = dst_nodes;
    a.s_nbr = ws_ptr<int32_t>(c, L.s_nbr);
    a.s_w = ws_ptr<float>(c, L.s_w);
    a.s_cnt = ws_ptr<int32_t>(c, L.s_cnt);
    a.mark = ws_ptr<uint64_t>(c, L.mark_bitmap);
    a.words = L.words;
    a.slots = ws_ptr<unsigned long long>(c, L.hash_slots);
    a.hmask = L.hash_cap - 1;
    a.hshift = 32u - (uint32_t) __builtin_ctz(L.hash_cap);
    a.sums_rows = ws_ptr<int32_t>(c, L.sums_rows);
    a.sums_words = ws_ptr<int32_t>(c, L.sums_words);
    a.row_tiles_max = (int32_t) ((L.rows[layer_index] + kTile - 1) / kTile);
    a.word_tiles = (int32_t) L.word_tiles;
    a.indptr = blk->indptr;
    a.indices = blk->indices;
    a.weights = blk->weights;
    a.src_nodes = blk->src_nodes;

    const unsigned grid = (unsigned) (a.row_tiles_max + a.word_tiles);
    hipLaunchKernelGGL(k_finish_phase1, dim3(grid), dim3(kBlock), 0, s, a);
    hipLaunchKernelGGL(k_finish_phase2, dim3(1), dim3(kBlock), 0, s, a);
    hipLaunchKernelGGL(k_finish_phase3, dim3(grid), dim3(kBlock), 0, s, a);
    const int64_t max_slots = L.rows[layer_index] * (int64_t) a.fanout;
    int64_t rb = (max_slots + kBlock - 1) / kBlock;
    if (rb > (int64_t) c->num_cus * 16) rb = (int64_t) c->num_cus * 16;
    if (rb < 1) rb = 1;
    hipLaunchKernelGGL(k_relabel, dim3((unsigned) rb), dim3(kBlock), 0, s, a, max_slots);
    return hipGetLastError();
}

}  // namespace gns
