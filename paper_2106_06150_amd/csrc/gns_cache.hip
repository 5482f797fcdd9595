// The periodic global node cache (paper Section 3.2, Eq. (1); Theorem 1: the
// cache is drawn without replacement and has |C| nodes).
//
// The cache is the set of the first |C| distinct nodes of an i.i.d. stream in
// which node i appears with probability deg(i)/nnz: draw j picks a CSR entry
// uniformly with a Philox word pair and takes the row that owns it.  The
// stream is processed in chunks; a small hash map keeps, per drawn node, the
// smallest stream index at which it appeared (atomicMin), which makes "draw j
// is the first occurrence of its node" a pure function of the stream and
// independent of thread order.  First occurrences are counted with a prefix
// scan; the chunk in which the count reaches |C| is cut at exactly that draw.
#include "gns_internal.h"
#include "gns_device.hpp"

namespace gns {

// ---------------------------------------------------------------------------
// Graph validation at create time: offsets non-decreasing, ids in range, rows
// strictly ascending; also counts the rows with at least one neighbor.
struct ValidateOut {
    int32_t nonzero_rows;
    int32_t bad_offsets;
    int32_t bad_index;
    int32_t unsorted;
};

template <typename OffT>
__global__ void __launch_bounds__(kBlock) k_validate_graph(const void* indptr, const int32_t* indices, int64_t n,
                                                           int64_t nnz, ValidateOut* out)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    int32_t nonzero = 0;
    for (int64_t v = (int64_t) blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (int64_t) gridDim.x * blockDim.x) {
        const int64_t b = load_off<OffT>(indptr, v), e = load_off<OffT>(indptr, v + 1);
        if (b < 0 || e < b || e > nnz || (v == 0 && b != 0) || (v == n - 1 && e != nnz)) { out->bad_offsets = 1; continue; }
        if (e > b) ++nonzero;
        int32_t prev = -1;
        for (int64_t q = b; q < e; ++q) {
            const int32_t u = indices[q];
            if (u < 0 || (int64_t) u >= n) out->bad_index = 1;
            if (u <= prev) out->unsorted = 1;
            prev = u;
        }
    }
    nonzero = block_sum(nonzero, smem);
    if (threadIdx.x == 0 && nonzero) atomicAdd(&out->nonzero_rows, nonzero);
}

hipError_t launch_count_nonzero_rows(gns_ctx* c, hipStream_t s, int32_t* d_out)
{
    const int64_t n = c->graph.num_nodes;
    int64_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > (int64_t) c->num_cus * 32) blocks = (int64_t) c->num_cus * 32;
    hipError_t e = launch_fill_u32(reinterpret_cast<uint32_t*>(d_out), 4, 0u, s);
    if (e != hipSuccess) return e;
    ValidateOut* out = reinterpret_cast<ValidateOut*>(d_out);
    if (c->graph.indptr_is_i64)
        hipLaunchKernelGGL((k_validate_graph<int64_t>), dim3((unsigned) blocks), dim3(kBlock), 0, s, c->graph.indptr,
                           c->graph.indices, n, c->graph.num_entries, out);
    else
        hipLaunchKernelGGL((k_validate_graph<int32_t>), dim3((unsigned) blocks), dim3(kBlock), 0, s, c->graph.indptr,
                           c->graph.indices, n, c->graph.num_entries, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
struct DrawArgs {
    DeviceState* st;
    const void* indptr;
    int64_t n;
    uint64_t nnz;
    uint32_t key0, key1, epoch;
    uint64_t j0;               // stream index of the chunk's first draw
    int32_t count;             // draws in this chunk
    uint32_t* keys;            // draw hash: node ids (0xFFFFFFFF = empty)
    uint32_t* first;           // draw hash: smallest stream index seen for the node
    uint32_t hmask, hshift;
    int32_t* draw_node;        // [chunk]
    int32_t* draw_slot;        // [chunk] slot of the node in the draw hash
    int32_t* sums;             // [tiles + 1]
    int32_t tiles;
    uint64_t* cache_bitmap;
    int64_t cache_size;
    int32_t chunk_index;       // chunks of one draw are numbered from 0
};

// A draw enqueues its chunks without knowing how many it needs: the chunk that completes the cache says
// so in the device state and every later chunk stands down.
__device__ __forceinline__ bool chunk_stands_down(const DrawArgs& a)
{
    const int32_t done = a.st->draw_done_chunk;
    return done >= 0 && done < a.chunk_index;
}

__global__ void k_cache_draw_reset(DeviceState* st)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        st->draw_distinct = 0;
        st->draw_done_chunk = -1;
        st->chunk_distinct = 0;
        st->chunk_limit = 0;
        st->chunk_final = 0;
    }
}

// the unique row i with indptr[i] <= e < indptr[i+1]
template <typename OffT>
__device__ __forceinline__ int64_t owner_row(const void* indptr, int64_t n, int64_t e)
{
    int64_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (load_off<OffT>(indptr, mid) <= e) lo = mid; else hi = mid;
    }
    return lo;
}

template <typename OffT>
__global__ void __launch_bounds__(kBlock) k_cache_draw(DrawArgs a)
{
    const int32_t t = (int32_t) (blockIdx.x * blockDim.x + threadIdx.x);
    if (t >= a.count || chunk_stands_down(a)) return;
    const uint64_t j = a.j0 + (uint64_t) t;
    const Philox4 r = philox4x32_10((uint32_t) j, (uint32_t) (j >> 32), a.epoch, kTagCache, a.key0, a.key1);
    const uint64_t r64 = ((uint64_t) r.w[1] << 32) | (uint64_t) r.w[0];
    const uint64_t e = __umul64hi(r64, a.nnz);                      // uniform CSR entry
    const uint32_t node = (uint32_t) owner_row<OffT>(a.indptr, a.n, (int64_t) e);
    uint32_t h = hash_start(node, a.hshift);
    for (uint32_t probe = 0; probe <= a.hmask; ++probe) {
        const uint32_t old = atomicCAS(&a.keys[h], 0xFFFFFFFFu, node);
        if (old == 0xFFFFFFFFu || old == node) break;
        h = (h + 1) & a.hmask;
    }
    atomicMin(&a.first[h], (uint32_t) j);
    a.draw_node[t] = (int32_t) node;
    a.draw_slot[t] = (int32_t) h;
}

__device__ __forceinline__ int32_t is_first_occurrence(const DrawArgs& a, int32_t t)
{
    if (t >= a.count) return 0;
    return a.first[a.draw_slot[t]] == (uint32_t) (a.j0 + (uint64_t) t) ? 1 : 0;
}

__global__ void __launch_bounds__(kBlock) k_cache_flags_phase1(DrawArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    if (chunk_stands_down(a)) return;
    const int32_t base = (int32_t) blockIdx.x * kTile;
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) sum += is_first_occurrence(a, base + i * kBlock + (int32_t) threadIdx.x);
    sum = block_sum(sum, smem);
    if (threadIdx.x == 0) a.sums[blockIdx.x] = sum;
}

__global__ void __launch_bounds__(kBlock) k_cache_flags_phase2(DrawArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    if (chunk_stands_down(a)) return;
    int32_t carry = 0;
    for (int32_t base = 0; base < a.tiles; base += kBlock) {
        const int32_t i = base + (int32_t) threadIdx.x;
        const int32_t v = (i < a.tiles) ? a.sums[i] : 0;
        int32_t total;
        const int32_t ex = block_exclusive_scan(v, smem, &total);
        if (i < a.tiles) a.sums[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) {
        // how many of this chunk's first occurrences the cache still takes, and whether that completes it
        const int64_t need = a.cache_size - (int64_t) a.st->draw_distinct;
        const int32_t limit = (int32_t) ((int64_t) carry < need ? (int64_t) carry : need);
        const int32_t final = (int64_t) carry >= need ? 1 : 0;
        a.st->chunk_distinct = carry;
        a.st->chunk_limit = limit;
        a.st->chunk_final = final;
        a.st->draw_distinct += limit;
        if (final) a.st->draw_done_chunk = a.chunk_index;
    }
}

__global__ void __launch_bounds__(kBlock) k_cache_commit(DrawArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    if (chunk_stands_down(a)) return;
    const int32_t limit = a.st->chunk_limit, is_final = a.st->chunk_final;
    const int32_t base = (int32_t) blockIdx.x * kTile;
    const int32_t t0 = base + (int32_t) threadIdx.x * kItems;
    int32_t f[kItems];
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) { f[i] = is_first_occurrence(a, t0 + i); sum += f[i]; }
    int32_t total;
    int32_t g = a.sums[blockIdx.x] + block_exclusive_scan(sum, smem, &total);
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        if (f[i]) {
            if (g < limit) {
                const uint32_t node = (uint32_t) a.draw_node[t0 + i];
                atomicOr(reinterpret_cast<unsigned long long*>(&a.cache_bitmap[node >> 6]), 1ull << (node & 63u));
                if (is_final && g == limit - 1) a.st->cut_draw = a.j0 + (uint64_t) (t0 + i);
            }
            ++g;
        }
    }
}

// ---------------------------------------------------------------------------
// Rank index and ascending node list from the finished bitmap.
struct IndexArgs {
    const uint64_t* bitmap;
    int64_t words;
    int32_t* sums;
    int32_t tiles;
    int32_t* word_prefix;
    int32_t* cache_nodes;
};

__global__ void __launch_bounds__(kBlock) k_cache_index_phase1(IndexArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const int64_t base = (int64_t) blockIdx.x * kTile;
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int64_t w = base + (int64_t) i * kBlock + threadIdx.x;
        if (w < a.words) sum += __popcll(a.bitmap[w]);
    }
    sum = block_sum(sum, smem);
    if (threadIdx.x == 0) a.sums[blockIdx.x] = sum;
}

__global__ void __launch_bounds__(kBlock) k_cache_index_phase2(IndexArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    int32_t carry = 0;
    for (int32_t base = 0; base < a.tiles; base += kBlock) {
        const int32_t i = base + (int32_t) threadIdx.x;
        const int32_t v = (i < a.tiles) ? a.sums[i] : 0;
        int32_t total;
        const int32_t ex = block_exclusive_scan(v, smem, &total);
        if (i < a.tiles) a.sums[i] = carry + ex;
        carry += total;
    }
}

__global__ void __launch_bounds__(kBlock) k_cache_index_phase3(IndexArgs a)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const int64_t base = (int64_t) blockIdx.x * kTile;
    const int64_t w0 = base + (int64_t) threadIdx.x * kItems;
    uint64_t word[kItems];
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        word[i] = (w0 + i < a.words) ? a.bitmap[w0 + i] : 0ull;
        sum += __popcll(word[i]);
    }
    int32_t total;
    int32_t pos = a.sums[blockIdx.x] + block_exclusive_scan(sum, smem, &total);
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        if (w0 + i < a.words) {
            a.word_prefix[w0 + i] = pos;
            uint64_t rest = word[i];
            while (rest) {
                const int bit = __builtin_ctzll(rest);
                rest &= rest - 1;
                a.cache_nodes[pos++] = (int32_t) ((w0 + i) * 64 + bit);
            }
        }
    }
}

// Section 3.4 for every node of the cache: p_u = deg(u)/nnz, p^C_u = 1 - (1 - p_u)^|C|
// (expm1/log1p keep a tiny p_u exact), stored as 1/p^C_u in fp32.  The table is indexed by node id; entries of nodes
// outside the current cache are stale and never read.
template <typename OffT>
__global__ void __launch_bounds__(kBlock) k_cache_pc(const int32_t* cache_nodes, int64_t C, const void* indptr,
                                                     int64_t nnz, float* node_inv_pc)
{
    const int64_t i = (int64_t) blockIdx.x * kBlock + threadIdx.x;
    if (i >= C) return;
    const int32_t u = cache_nodes[i];
    const int64_t deg = load_off<OffT>(indptr, (int64_t) u + 1) - load_off<OffT>(indptr, u);
    const double p = (double) deg / (double) nnz;
    const double pc = (p >= 1.0) ? 1.0 : -expm1((double) C * log1p(-p));
    node_inv_pc[u] = (float) (1.0 / pc);
}

// Coarse companion of the cache bitmap: bit g of the result is set iff some node of
// [g << shift, (g + 1) << shift) is cached.  One thread per 64-bit coarse word.
__global__ void __launch_bounds__(kBlock) k_cache_coarse(const uint64_t* bitmap, int64_t words, int shift,
                                                         uint64_t* coarse, int64_t coarse_words)
{
    const int64_t cw = (int64_t) blockIdx.x * kBlock + threadIdx.x;
    if (cw >= coarse_words) return;
    const int fine_per_coarse = 1 << shift;                    // fine words folded into one coarse word
    const int groups_per_fine = 64 >> shift;                   // coarse bits one fine word yields
    const uint64_t group_mask = (shift == 6) ? ~0ull : ((1ull << (1 << shift)) - 1ull);
    uint64_t out = 0;
    for (int f = 0; f < fine_per_coarse; ++f) {
        const int64_t w = cw * fine_per_coarse + f;
        const uint64_t x = (w < words) ? bitmap[w] : 0ull;
        for (int g = 0; g < groups_per_fine; ++g)
            if ((x >> (g << shift)) & group_mask) out |= 1ull << (f * groups_per_fine + g);
    }
    coarse[cw] = out;
}

// ---------------------------------------------------------------------------
static gns_status fail(gns_ctx* c, gns_status st, const char* what, hipError_t e)
{
    if (e != hipSuccess) snprintf(c->err, sizeof(c->err), "%s: %s", what, hipGetErrorString(e));
    else snprintf(c->err, sizeof(c->err), "%s", what);
    return st;
}

#define GNS_HIP_TRY(expr, what)                                        \
    do {                                                               \
        hipError_t e__ = (expr);                                       \
        if (e__ != hipSuccess) return fail(c, GNS_EHIP, what, e__);    \
    } while (0)

constexpr int kAsyncChunks = 8;     // chunks an asynchronous draw enqueues (a typical cache needs one or two)

// Records, on the stream every context of the family last used, the end of what may still read the copy
// of the cache block that stops being current now.
static gns_status mark_last_readers(gns_ctx* c, int old_gen)
{
    for (int i = 0; i < c->family_count; ++i) {
        gns_ctx* m = c->family[i];
        for (int i = 0; i < m->reader_stream_count; ++i)
            GNS_HIP_TRY(hipEventRecord(m->gen_event[old_gen][i], m->reader_streams[i]), "event record");
        m->gen_event_used[old_gen] = m->reader_stream_count;
        m->reader_stream_count = 0;          // streams used from now on read the next cache
    }
    return GNS_OK;
}

// The current cache stops being usable without a successor (the cache probability is about to change).
gns_status retire_cache(gns_ctx* c)
{
    const gns_status st = mark_last_readers(c, c->cache_gen);
    if (st != GNS_OK) return st;
    c->cache_valid = false;
    return GNS_OK;
}

// Makes the copy a finished or enqueued draw filled the current one.
gns_status activate_cache(gns_ctx* c)
{
    if (c->cache_valid) {
        const gns_status st = mark_last_readers(c, c->cache_gen);
        if (st != GNS_OK) return st;
    }
    c->cache_gen = c->pending_gen;
    c->cache_valid = true;
    c->had_cache = true;
    c->pending = false;
    c->cache_version += 1;
    return GNS_OK;
}

// Reads the outcome of the last draw back (synchronises behind it).
gns_status finish_pending_draw(gns_ctx* c)
{
    const int gen = c->pending ? c->pending_gen : c->cache_gen;
    GNS_HIP_TRY(hipEventSynchronize(c->ready_event[gen]), "cache draw wait");
    GNS_HIP_TRY(hipMemcpy(c->h_state, c->d_state, sizeof(DeviceState), hipMemcpyDeviceToHost), "cache readback");
    if (c->h_state->draw_done_chunk < 0)
        return fail(c, GNS_ECAPACITY, "cache draw: the stream did not yield cache_size distinct nodes within the chunks an asynchronous draw enqueues", hipSuccess);
    c->cache_draws = (int64_t) c->h_state->cut_draw + 1;
    return GNS_OK;
}

gns_status run_sample_cache(gns_ctx* c, uint64_t seed, uint64_t epoch, bool wait_for_it, hipStream_t s)
{
    const Layout& L = c->lay;
    const int64_t C = c->config.cache_size;
    // The draw fills the copy of the cache block the mini-batches are not reading.  Whatever was enqueued
    // while that copy was the current one ended with the events recorded when it stopped being current:
    // the device may not have reached all of it yet if the host runs far ahead, so the draw waits for them.
    const int gen = c->had_cache ? (c->cache_gen ^ 1) : 0;
    uint64_t* bitmap = cache_ptr<uint64_t>(c, L.cache_bitmap, gen);
    if (c->pending)                                  // a draw that was never made current: this one replaces it
        GNS_HIP_TRY(hipStreamWaitEvent(s, c->ready_event[c->pending_gen], 0), "wait for the replaced draw");
    for (int i = 0; i < c->family_count; ++i) {
        gns_ctx* m = c->family[i];
        for (int i = 0; i < m->gen_event_used[gen]; ++i)
            GNS_HIP_TRY(hipStreamWaitEvent(s, m->gen_event[gen][i], 0), "wait for the readers of the old cache");
        m->gen_event_used[gen] = 0;
    }
    hipLaunchKernelGGL(k_cache_draw_reset, dim3(1), dim3(kWave), 0, s, c->d_state);
    GNS_HIP_TRY(launch_fill_u64(reinterpret_cast<unsigned long long*>(bitmap), (size_t) L.words, 0ull, s), "clear cache bitmap");
    GNS_HIP_TRY(launch_fill_u32(ws_ptr<uint32_t>(c, L.draw_keys), L.draw_hash_cap, 0xFFFFFFFFu, s), "clear draw keys");
    GNS_HIP_TRY(launch_fill_u32(ws_ptr<uint32_t>(c, L.draw_vals), L.draw_hash_cap, 0xFFFFFFFFu, s), "clear draw vals");

    // The draw picks a uniform integer below the total mass and takes the node whose prefix interval
    // holds it: the CSR offsets for Eq. (1), the prefix of the walk weights for the other probability.
    const bool walk = c->config.cache_probability == GNS_PROB_WALK;
    const void* prob_prefix = walk ? static_cast<const void*>(ws_ptr<int64_t>(c, L.prob_prefix)) : c->graph.indptr;
    const uint64_t prob_total = walk ? (uint64_t) c->prob_total : (uint64_t) c->graph.num_entries;
    DrawArgs a;
    a.st = c->d_state;
    a.indptr = prob_prefix;
    a.n = c->graph.num_nodes;
    a.nnz = prob_total;
    a.key0 = (uint32_t) seed;
    a.key1 = (uint32_t) (seed >> 32);
    a.epoch = (uint32_t) epoch;
    a.keys = ws_ptr<uint32_t>(c, L.draw_keys);
    a.first = ws_ptr<uint32_t>(c, L.draw_vals);
    a.hmask = L.draw_hash_cap - 1;
    a.hshift = 32u - (uint32_t) __builtin_ctz(L.draw_hash_cap);
    a.draw_node = ws_ptr<int32_t>(c, L.draw_node);
    a.draw_slot = ws_ptr<int32_t>(c, L.draw_slot);
    a.sums = ws_ptr<int32_t>(c, L.sums_words);      // sized for max(word tiles, draw tiles)
    a.cache_bitmap = bitmap;
    a.cache_size = C;

    // The draw hash holds every distinct node seen so far: fewer than |C| before the final
    // chunk plus at most one chunk's worth, which is what it was sized for.  Stream indices
    // are kept in 32 bits; a cache that needs more draws than the limit is refused.  How many of a
    // chunk's first occurrences enter the cache, and whether they complete it, is decided on the device
    // (k_cache_flags_phase2); the host only needs to know when to stop enqueuing chunks.
    uint64_t draw_limit = 256ull * (uint64_t) C + 64ull * (uint64_t) L.draw_chunk;
    if (draw_limit > 0xFFFFFFFFull) draw_limit = 0xFFFFFFFFull;
    const bool i64 = walk || c->graph.indptr_is_i64 != 0;
    const int64_t count = L.draw_chunk;
    a.count = (int32_t) count;
    a.tiles = (int32_t) ((count + kTile - 1) / kTile);
    const unsigned draw_blocks = (unsigned) ((count + kBlock - 1) / kBlock);
    for (int chunk = 0;; ++chunk) {
        const uint64_t j0 = (uint64_t) chunk * (uint64_t) count;
        if (j0 + (uint64_t) count > draw_limit) {
            if (!wait_for_it) break;
            return fail(c, GNS_ECAPACITY, "cache draw: the stream did not yield cache_size distinct nodes within the draw limit (cache_size too close to the number of nodes with neighbors)", hipSuccess);
        }
        if (!wait_for_it && chunk >= kAsyncChunks) break;
        a.j0 = j0;
        a.chunk_index = chunk;
        if (i64) hipLaunchKernelGGL((k_cache_draw<int64_t>), dim3(draw_blocks), dim3(kBlock), 0, s, a);
        else     hipLaunchKernelGGL((k_cache_draw<int32_t>), dim3(draw_blocks), dim3(kBlock), 0, s, a);
        hipLaunchKernelGGL(k_cache_flags_phase1, dim3((unsigned) a.tiles), dim3(kBlock), 0, s, a);
        hipLaunchKernelGGL(k_cache_flags_phase2, dim3(1), dim3(kBlock), 0, s, a);
        hipLaunchKernelGGL(k_cache_commit, dim3((unsigned) a.tiles), dim3(kBlock), 0, s, a);
        GNS_HIP_TRY(hipGetLastError(), "cache draw launch");
        if (wait_for_it) {
            GNS_HIP_TRY(hipMemcpyAsync(c->h_state, c->d_state, sizeof(DeviceState), hipMemcpyDeviceToHost, s), "cache draw readback");
            GNS_HIP_TRY(hipStreamSynchronize(s), "cache draw sync");
            if (c->h_state->draw_done_chunk >= 0) break;
        }
    }

    IndexArgs x;
    x.bitmap = bitmap;
    x.words = L.words;
    x.sums = ws_ptr<int32_t>(c, L.sums_words);
    x.tiles = (int32_t) L.word_tiles;
    x.word_prefix = cache_ptr<int32_t>(c, L.cache_prefix, gen);
    x.cache_nodes = cache_ptr<int32_t>(c, L.cache_nodes, gen);
    hipLaunchKernelGGL(k_cache_index_phase1, dim3((unsigned) x.tiles), dim3(kBlock), 0, s, x);
    hipLaunchKernelGGL(k_cache_index_phase2, dim3(1), dim3(kBlock), 0, s, x);
    hipLaunchKernelGGL(k_cache_index_phase3, dim3((unsigned) x.tiles), dim3(kBlock), 0, s, x);
    GNS_HIP_TRY(hipGetLastError(), "cache index launch");

    {
        const unsigned pc_blocks = (unsigned) ((C + kBlock - 1) / kBlock);
        float* node_pc = cache_ptr<float>(c, L.node_pc, gen);
        if (i64) hipLaunchKernelGGL((k_cache_pc<int64_t>), dim3(pc_blocks), dim3(kBlock), 0, s, x.cache_nodes, C, prob_prefix, (int64_t) prob_total, node_pc);
        else     hipLaunchKernelGGL((k_cache_pc<int32_t>), dim3(pc_blocks), dim3(kBlock), 0, s, x.cache_nodes, C, prob_prefix, (int64_t) prob_total, node_pc);
        GNS_HIP_TRY(hipGetLastError(), "cache weight table launch");
    }
    if (L.coarse_shift > 0) {
        const unsigned cb = (unsigned) ((L.coarse_words + kBlock - 1) / kBlock);
        hipLaunchKernelGGL(k_cache_coarse, dim3(cb), dim3(kBlock), 0, s, bitmap, (int64_t) L.words, (int) L.coarse_shift,
                           cache_ptr<uint64_t>(c, L.coarse_bitmap, gen), (int64_t) L.coarse_words);
        GNS_HIP_TRY(hipGetLastError(), "coarse bitmap launch");
    }
    if (c->config.flag_mode == GNS_FLAGS_PER_CACHE) {
        GNS_HIP_TRY(launch_flag_all_entries(c, gen, s), "flag all entries");
        GNS_HIP_TRY(launch_build_induced(c, gen, s), "induced subgraph");
    }
    if (c->graph.feat_dim > 0) {
        // fill the device table of cached feature rows (slot order) straight from the full store
        const int32_t* fill_nodes = x.cache_nodes;
        const int32_t fill_count = (int32_t) C;
        float* fill_out = cache_ptr<float>(c, L.cache_feat, gen);
        GNS_HIP_TRY(launch_gather(&c, 1, &fill_nodes, &fill_count, &fill_out, -1, s), "cache feature fill");
    }
    GNS_HIP_TRY(hipEventRecord(c->ready_event[gen], s), "event record");
    c->pending = true;
    c->pending_gen = gen;
    c->cache_draws = -1;                           // read back on demand
    if (!wait_for_it) return GNS_OK;
    const gns_status st = finish_pending_draw(c);
    if (st != GNS_OK) { c->pending = false; return st; }
    return activate_cache(c);
}

}  // namespace gns
