// Layer sampler: for every dst row v independently, N_l(v) <- sample(N(v), C)
// (paper Algorithm 1, top-down loop).
//
//   UNIFORM     Section 2.1: min(k, deg(v)) neighbors uniformly without
//               replacement.  Only the k chosen CSR entries are read.
//   CACHE_ONLY  Sections 3.3 and 4.1: the eligible list is the row's entries
//               whose node is in the cache, in CSR order; min(k, N_C(v)) of
//               them are chosen; each carries the Section 3.4 weight.
//   CACHE_FIRST Section 3.3: as CACHE_ONLY; a row with N_C(v) < k then draws the
//               shortfall uniformly from its entries outside the cache.
//
// The without-replacement choice is Robert Floyd's subset algorithm on ranks
// of the eligible list, driven by k Philox words keyed by (seed, layer, node,
// slot); the chosen ranks are emitted in ascending order.  All decisions are
// integer arithmetic, so the sample does not depend on scheduling.
//
// Output per row r (fixed stride k): s_nbr[r*k + i] (the neighbor's local id as -(id+1) if it has
// one, else its global id), s_w[r*k + i] for
// i < s_cnt[r], row_eligible[r]; every emitted id that has no local id yet
// (it is not a dst node of this layer) also sets its bit in the node-indexed
// mark bitmap that the frontier stage turns into the src list.
#include <string.h>
#include <stdlib.h>
#include "gns_kernels.hpp"

namespace gns {

// Floyd's subset draw inside a group of G consecutive lanes (G a power of two
// <= 64).  Lane s < k ends up with one chosen rank of {0..m-1} in *val and that
// rank's position in ascending order in *pos.  Requires m > k.  k may differ from
// group to group; k_loop >= every group's k must be the same for the whole wave
// (it bounds the loops that exchange data between lanes).  The word of lane s is
// slot slot0 + s of (layer, node).  Every lane of the wave must call it.
template <int G>
__device__ __forceinline__ void floyd_in_group(uint32_t m, int k, int k_loop, uint32_t key0, uint32_t key1,
                                               uint32_t layer, uint32_t node, int s, uint32_t* val, int* pos,
                                               int slot0 = 0)
{
    s = opaque(s);
    // lane s draws t_s uniform in [0, m-k+s]
    const uint32_t slot = (uint32_t) (slot0 + s);
    const Philox4 r = philox4x32_10(node, slot >> 2, layer, kTagNeighbor, key0, key1);
    const int sel = (int) (slot & 3u);
    const uint32_t word = sel == 0 ? r.w[0] : sel == 1 ? r.w[1] : sel == 2 ? r.w[2] : r.w[3];
    const uint32_t j_own = m - (uint32_t) k + (uint32_t) s;
    const uint32_t t_own = __umulhi(word, j_own + 1u);
    uint32_t chosen = 0xFFFFFFFFu;              // not yet decided
    const int group_base = opaque_lane_id() & ~(G - 1);
    const uint64_t group_mask = (G == 64) ? ~0ull : (((1ull << (G & 63)) - 1ull) << group_base);
    for (int q = 0; q < k_loop; ++q) {
        const uint32_t t_q = __shfl(t_own, q, G);
        // is t_q already among the ranks decided by slots < q ?
        const uint64_t hit = __ballot(s < q && chosen == t_q) & group_mask;
        if (s == q) chosen = hit ? j_own : t_own;
    }
    int rank = 0;
    for (int q = 0; q < k_loop; ++q) {
        const uint32_t c_q = __shfl(chosen, q, G);
        rank += (q < k && c_q < chosen) ? 1 : 0;
    }
    *val = chosen;
    *pos = rank;
}

// A sampled id becomes a new src node unless it already owns a local id.  Returns what the relabel
// step should find in the scratch slot: the node's local id as -(id + 1) if it has one (no second
// lookup then), else the global id (>= 0), whose local id is assigned by the union step.
// Sets node u's bit in the frontier mark bitmap.  (Looking at the bit first, to spare popular nodes'
// words thousands of atomics per batch, measured slower: the extra dependent read costs more than the
// atomics it saves.)
__device__ __forceinline__ void mark_node(const SampleArgs& a, uint32_t u)
{
    atomicOr(reinterpret_cast<unsigned long long*>(&a.mark[u >> 6]), 1ull << (u & 63u));
    if (a.mark_summary)
        atomicOr(reinterpret_cast<unsigned long long*>(&a.mark_summary[u >> 12]), 1ull << ((u >> 6) & 63u));
}

__device__ __forceinline__ int32_t mark_if_new(const SampleArgs& a, uint32_t u)
{
    const int32_t local = hash_lookup(a.slots, a.hmask, a.hshift, u);
    if (local >= 0) return -1 - local;
    mark_node(a, u);
    return (int32_t) u;
}

// ---------------------------------------------------------------------------
// UNIFORM: G lanes per row, rows assigned round-robin to groups.
template <int G>
__global__ void __launch_bounds__(kBlock) k_sample_uniform(LayerArgs g, int relabel_blocks)
{
    // the last relabel_blocks blocks finish the previous layer's block instead (see relabel_body); they are
    // dispatched after this layer's rows, whose dependent loads set the length of the launch
    const int64_t nblocks = (int64_t) gridDim.x - relabel_blocks;
    if ((int64_t) blockIdx.x >= nblocks) {
        relabel_body(bind_finish(g, (int) blockIdx.y, false), (int64_t) blockIdx.x - nblocks, relabel_blocks);
        return;
    }
    const SampleArgs a = bind_sample(g, (int) blockIdx.y);
    const int64_t block = (int64_t) blockIdx.x;
    const int32_t R = a.st->num_dst[a.layer_index];
    const int k = a.fanout;
    constexpr int kRowsPerWave = kWave / G;
    // The loop bounds live in scalar registers (readfirstlane) so that the whole wave
    // provably iterates together: the draw below exchanges data between lanes.
    const int64_t wave_global = block * (kBlock / kWave) +
                                __builtin_amdgcn_readfirstlane((int) (threadIdx.x >> 6));
    const int64_t num_waves = nblocks * (kBlock / kWave);
    for (int64_t row0 = wave_global * kRowsPerWave; row0 < R; row0 += num_waves * kRowsPerWave) {
        const int lane = opaque_lane_id();
        const int s = lane & (G - 1);
        const int64_t row = row0 + (lane / G);
        const bool live = row < R;
        int64_t start = 0;
        uint32_t m = 0;
        uint32_t v = 0;
        if (live) {
            const RowExtent ext = a.row_ext[row];
            v = (uint32_t) a.dst_nodes[row];
            start = ext.start;
            m = (uint32_t) (ext.end - ext.start);
        }
        uint32_t val;
        int pos;
        // run the draw with a safe size in every lane, then keep it only where it applies
        floyd_in_group<G>(m > (uint32_t) k ? m : (uint32_t) k + 1u, k, k, a.st->key0, a.st->key1, a.layer_number, v, s, &val, &pos);
        const int cnt = (m > (uint32_t) k) ? k : (int) m;
        if (m <= (uint32_t) k) { val = (uint32_t) s; pos = s; }
        if (live && s < cnt) {
            const int32_t u = a.indices[start + val];
            a.s_w[row * k + pos] = 1.0f;
            a.s_nbr[row * k + pos] = mark_if_new(a, (uint32_t) u);
        }
        if (live && s == 0) {
            a.s_cnt[row] = cnt;
            a.row_eligible[row] = (int32_t) m;
        }
    }
}

// ---------------------------------------------------------------------------
// One dst row per lane (fan-outs up to 16).  The list a row draws from is either its CSR segment (UNIFORM)
// or, with the induced subgraph S of GNS_FLAGS_PER_CACHE, its cached neighbors s_nodes[P(start) .. P(end))
// (CACHE_ONLY): in both cases a contiguous list of m ids of which min(k, m) ranks are chosen, so a lane
// needs the row's extent, the k drawn entries and nothing else of the row.  Every lane runs Floyd's draw
// for its own row with the loops over the k slots unrolled (the chosen ranks stay in registers); the
// loads of all k entries, their weights and their hash slots are issued together.  A wave handles 64
// rows at once and consecutive lanes read consecutive rows' extents and ids.
__device__ __forceinline__ uint64_t bits_below(int64_t e)
{
    return (1ull << (e & 63)) - 1ull;
}

template <int KMAX, bool kInduced>
__global__ void __launch_bounds__(kBlock) k_sample_lane(LayerArgs g, int relabel_blocks)
{
    const int64_t nblocks = (int64_t) gridDim.x - relabel_blocks;
    if ((int64_t) blockIdx.x >= nblocks) {
        relabel_body(bind_finish(g, (int) blockIdx.y, false), (int64_t) blockIdx.x - nblocks, relabel_blocks);
        return;
    }
    const SampleArgs a = bind_sample(g, (int) blockIdx.y);
    const int32_t R = a.st->num_dst[a.layer_index];
    const int k = a.fanout;                         // <= KMAX
    const uint32_t key0 = a.st->key0, key1 = a.st->key1;
    const int32_t* list = kInduced ? a.s_nodes : a.indices;
    for (int64_t row = (int64_t) blockIdx.x * kBlock + threadIdx.x; row < R; row += nblocks * kBlock) {
        const RowExtent ext = a.row_ext[row];
        const uint32_t v = (uint32_t) a.dst_nodes[row];
        int64_t base = ext.start;
        uint32_t m = (uint32_t) (ext.end - ext.start);
        if (kInduced) {
            m = 0;
            if (ext.end > ext.start) {
                const ChunkRec rs = a.srec[ext.start >> 6];
                const ChunkRec re = a.srec[ext.end >> 6];
                const uint32_t p0 = rs.before + (uint32_t) __popcll(rs.flags & bits_below(ext.start));
                const uint32_t p1 = re.before + (uint32_t) __popcll(re.flags & bits_below(ext.end));
                base = (int64_t) p0;
                m = p1 - p0;
            }
        }
        const int cnt = m > (uint32_t) k ? k : (int) m;
        uint32_t chosen[KMAX];
#pragma unroll
        for (int s = 0; s < KMAX; ++s) chosen[s] = s < cnt ? (uint32_t) s : 0xFFFFFFFFu;     // m <= k: take all
        if (m > (uint32_t) k) {
            // slot s of (layer, node) is word s & 3 of the Philox block with counter word s >> 2
            uint32_t word[KMAX];
#pragma unroll
            for (int c = 0; c < KMAX / 4; ++c) {
                if (4 * c < k) {
                    const Philox4 r = philox4x32_10(v, (uint32_t) c, a.layer_number, kTagNeighbor, key0, key1);
                    word[4 * c] = r.w[0]; word[4 * c + 1] = r.w[1]; word[4 * c + 2] = r.w[2]; word[4 * c + 3] = r.w[3];
                } else {
                    word[4 * c] = word[4 * c + 1] = word[4 * c + 2] = word[4 * c + 3] = 0u;
                }
            }
#pragma unroll
            for (int s = 0; s < KMAX; ++s) {
                if (s < k) {
                    const uint32_t j = m - (uint32_t) k + (uint32_t) s;
                    const uint32_t t = __umulhi(word[s], j + 1u);
                    bool dup = false;
#pragma unroll
                    for (int q = 0; q < s; ++q) dup = dup || chosen[q] == t;
                    chosen[s] = dup ? j : t;
                }
            }
        }
        // entries of the chosen ranks, all in flight together
        uint32_t u[KMAX];
#pragma unroll
        for (int s = 0; s < KMAX; ++s) u[s] = s < cnt ? (uint32_t) list[base + (int64_t) chosen[s]] : 0u;
        float wgt[KMAX];
        unsigned long long first[KMAX];
#pragma unroll
        for (int s = 0; s < KMAX; ++s) {
            wgt[s] = 1.0f;
            first[s] = kEmptySlot;
            if (s < cnt) {
                if (kInduced) wgt[s] = a.node_inv_pc[u[s]];
                first[s] = a.slots[hash_start(u[s], a.hshift)];
            }
        }
        // Section 3.4: coefficient p^C_u * k / min(k, N_C(v)), weight = 1 / coefficient (fp32 from the table on)
        const float scale = !kInduced ? 1.0f
                          : (a.wmode == GNS_W_UNBIASED) ? ((float) m / (float) (cnt > 0 ? cnt : 1))
                                                        : ((float) cnt / (float) k);
#pragma unroll
        for (int s = 0; s < KMAX; ++s) {
            if (s < cnt) {
                int pos = 0;
#pragma unroll
                for (int q = 0; q < KMAX; ++q) pos += chosen[q] < chosen[s] ? 1 : 0;
                // local id if the node has one already (first probe in hand), else mark it as a new src node
                int32_t out;
                const unsigned long long f = first[s];
                if ((uint32_t) f == u[s] && f != kEmptySlot) {
                    out = -1 - (int32_t) (f >> 32);
                } else {
                    const int32_t local = f == kEmptySlot ? -1 : hash_lookup(a.slots, a.hmask, a.hshift, u[s]);
                    if (local >= 0) {
                        out = -1 - local;
                    } else {
                        mark_node(a, u[s]);
                        out = (int32_t) u[s];
                    }
                }
                a.s_nbr[row * k + pos] = out;
                a.s_w[row * k + pos] = kInduced ? wgt[s] * scale : 1.0f;
            }
        }
        a.s_cnt[row] = cnt;
        a.row_eligible[row] = (int32_t) m;
    }
}

// ---------------------------------------------------------------------------
// CACHE_ONLY in two balanced phases.
//
// The CSR entry array is cut into aligned chunks of 64 entries; flags[g] holds, for chunk g,
// one bit per entry: "this neighbor is in the cache".
//   plan     per dst row, the aligned chunks its segment touches; prefix sum; the chunk ids
//            are written out as a flat work list (k_plan_count, k_plan_expand)
//   flag     one wave step = a few chunks of the list: coalesced 256-byte index loads, one
//            cache-bitmap test per entry, a ballot per chunk stored as one 64-bit word.  Every
//            chunk costs the same, so the stream is balanced whatever the degree skew
//            (k_flag_chunks; the bitmap is staged in LDS when it fits)
//   select   per dst row (a group of lanes): read the row's flag words, trim the two boundary
//            words to the row, count N_C(v), draw, map the chosen ranks back to CSR positions,
//            emit ids and Section 3.4 weights (k_select_rows)
// A chunk shared by two dst rows is flagged twice with the same value.

__device__ __forceinline__ int32_t chunks_touched(int64_t start, int64_t end)
{
    return end > start ? (int32_t) (((end - 1) >> 6) - (start >> 6) + 1) : 0;
}

// Plan tiles are kPlanTile rows (one row per thread): many small blocks keep the expansion parallel.
constexpr int kPlanTile = kBlock;

__global__ void __launch_bounds__(kBlock) k_plan_count(LayerArgs g, int relabel_blocks)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const int64_t ntiles = (int64_t) gridDim.x - relabel_blocks;
    if ((int64_t) blockIdx.x >= ntiles) {
        relabel_body(bind_finish(g, (int) blockIdx.y, false), (int64_t) blockIdx.x - ntiles, relabel_blocks);
        return;
    }
    const SampleArgs a = bind_sample(g, (int) blockIdx.y);
    const int64_t tile = (int64_t) blockIdx.x;
    const int32_t R = a.st->num_dst[a.layer_index];
    const int64_t r = tile * kPlanTile + threadIdx.x;
    if (tile * kPlanTile >= R) return;
    int32_t c = 0;
    if (r < R) {
        const RowExtent ext = a.row_ext[r];
        const int64_t start = ext.start, end = ext.end;
        c = chunks_touched(start, end);
        a.plan_cnt[r] = c;
        a.plan_g0[r] = (int32_t) (start >> 6);
    }
    const int32_t sum = block_sum(c, smem);
    if (threadIdx.x == 0) a.plan_sums[tile] = sum;
}

__global__ void __launch_bounds__(kBlock) k_plan_expand(LayerArgs g)
{
    __shared__ int32_t smem[kBlock / kWave + 1];
    const SampleArgs a = bind_sample(g, (int) blockIdx.y);
    __shared__ int32_t s_off[kPlanTile + 1];
    __shared__ int32_t s_g0[kPlanTile];
    const int32_t R = a.st->num_dst[a.layer_index];
    const int64_t base = (int64_t) blockIdx.x * kPlanTile;
    if (base >= R) return;
    // chunks of all earlier tiles
    int32_t before = 0;
    for (int32_t t = (int32_t) threadIdx.x; t < (int32_t) blockIdx.x; t += kBlock) before += a.plan_sums[t];
    before = block_sum(before, smem);
    const int64_t r = base + threadIdx.x;
    const int32_t c = (r < R) ? a.plan_cnt[r] : 0;
    s_g0[threadIdx.x] = (r < R) ? a.plan_g0[r] : 0;
    int32_t total;
    s_off[threadIdx.x] = block_exclusive_scan(c, smem, &total);
    if (threadIdx.x == 0) s_off[kPlanTile] = total;
    const int32_t last_tile = (R - 1) / kPlanTile;
    if ((int32_t) blockIdx.x == last_tile && threadIdx.x == 0) a.st->plan_chunks = before + total;
    __syncthreads();
    // one thread per work-list entry: its row is the last one whose offset is <= j
    for (int32_t j = (int32_t) threadIdx.x; j < total; j += kBlock) {
        int32_t lo = 0, hi = kPlanTile;
        while (hi - lo > 1) {
            const int32_t mid = (lo + hi) >> 1;
            if (s_off[mid] <= j) lo = mid; else hi = mid;
        }
        a.plan_desc[before + j] = s_g0[lo] + (j - s_off[lo]);
    }
}

constexpr int kFlagUnroll = 32;     // chunks a wave keeps in flight
constexpr int kFlagBatch = 64;      // work-list entries a wave fetches at once (one per lane)

// Membership words of kFlagUnroll chunks, chunk ids in lanes sub .. sub+kFlagUnroll-1 of my_chunk
// (every one a valid chunk id).  Lane l tests entry l of each chunk; the ballot of chunk sub+i
// lands in lane sub+i of (*lo, *hi).  Three passes over the unrolled set -- all index loads, all
// bitmap reads, all tests -- so that the loads of the whole set are in flight together.
//   kCareful: the set may hold the last chunk of the entry array, whose tail lanes lie beyond
//   num_entries; those lanes re-read the last entry and are masked out of the ballot.
//   kMode 0: the bitmap is read from global memory; 1: from LDS; 2: LDS holds the coarse bitmap (one bit
//   per group of ids): only the entries whose group has a cached node go on to read the exact bitmap;
//   3: as 2 with the coarse bitmap in global memory (small enough to stay in every XCD's L2).
template <int kMode, bool kCareful>
__device__ __forceinline__ void flag_chunk_set(const SampleArgs& a, const uint32_t* lds32, int32_t my_chunk, int sub,
                                               int lane, uint32_t* lo, uint32_t* hi)
{
    const int64_t last_chunk = (a.num_entries - 1) >> 6;
    const int last_lanes = (int) (a.num_entries - (last_chunk << 6));          // 1..64 entries in the last chunk
    const int lane_clamped = lane < last_lanes ? lane : last_lanes - 1;
    const uint64_t last_mask = last_lanes == 64 ? ~0ull : ((1ull << last_lanes) - 1ull);
    uint32_t u[kFlagUnroll];
#pragma unroll
    for (int i = 0; i < kFlagUnroll; ++i) {
        const int32_t g = __builtin_amdgcn_readlane(my_chunk, sub + i);
        const int32_t* row = a.indices + ((int64_t) g << 6);                   // wave-uniform base
        const int off = (kCareful && g == last_chunk) ? lane_clamped : lane;
        u[i] = (uint32_t) row[off];
    }
    const uint32_t* exact32 = reinterpret_cast<const uint32_t*>(a.cache_bitmap);
    uint32_t w[kFlagUnroll];
#pragma unroll
    for (int i = 0; i < kFlagUnroll; ++i) {
        if (kMode == 1)      w[i] = lds32[u[i] >> 5];
        else if (kMode == 0) w[i] = exact32[u[i] >> 5];
        else if (kMode == 2) w[i] = lds32[(u[i] >> a.coarse_shift) >> 5];
        else                 w[i] = reinterpret_cast<const uint32_t*>(a.coarse_bitmap)[(u[i] >> a.coarse_shift) >> 5];
    }
    if (kMode >= 2) {
#pragma unroll
        for (int i = 0; i < kFlagUnroll; ++i) {
            const bool maybe = (w[i] >> ((u[i] >> a.coarse_shift) & 31u)) & 1u;
            w[i] = maybe ? exact32[u[i] >> 5] : 0u;
        }
    }
#pragma unroll
    for (int i = 0; i < kFlagUnroll; ++i) {
        uint64_t ballot = __ballot((w[i] >> (u[i] & 31u)) & 1u);
        if (kCareful && __builtin_amdgcn_readlane(my_chunk, sub + i) == last_chunk) ballot &= last_mask;
        if (lane == sub + i) { *lo = (uint32_t) ballot; *hi = (uint32_t) (ballot >> 32); }
    }
}

// kMode 1 / 2: the cache bitmap / its coarse companion is first copied into dynamic LDS (rounded up to
// 16 bytes).  Every wave takes an equal, contiguous share of the work list.
// One work list: every wave takes an equal, contiguous share of its Q chunks.
template <int kMode>
__device__ __forceinline__ void flag_work_list(const SampleArgs& a, const uint32_t* lds32, int64_t Q, int use_plan)
{
    if (Q <= 0 || a.num_entries <= 0) return;
    const int waves_per_block = (int) (blockDim.x >> 6);
    const int64_t wave_global = (int64_t) blockIdx.x * waves_per_block +
                                __builtin_amdgcn_readfirstlane((int) (threadIdx.x >> 6));
    const int64_t num_waves = (int64_t) gridDim.x * waves_per_block;
    const int64_t share = (Q + num_waves - 1) / num_waves;
    const int64_t begin = wave_global * share;
    const int64_t end = (begin + share < Q) ? begin + share : Q;
    const int64_t last_chunk = (a.num_entries - 1) >> 6;
    const bool last_is_partial = (a.num_entries & 63) != 0;
    for (int64_t c0 = begin; c0 < end; c0 += kFlagBatch) {
        const int lane = opaque_lane_id();
        const int here = (int) ((end - c0 < kFlagBatch) ? end - c0 : kFlagBatch);     // scalar, >= 1
        // Lane l holds the chunk id of work-list entry c0 + l; lanes past the share repeat its last
        // entry (their result is not stored), so that every unrolled set is made of valid chunks.
        const int64_t q = c0 + (lane < here ? lane : here - 1);
        const int32_t my_chunk = use_plan ? a.plan_desc[q] : (int32_t) q;
        const bool careful = last_is_partial && __ballot((int64_t) my_chunk == last_chunk) != 0ull;
        uint32_t lo = 0, hi = 0;
        for (int sub = 0; sub < here; sub += kFlagUnroll) {                            // scalar bounds
            if (careful) flag_chunk_set<kMode, true>(a, lds32, my_chunk, sub, lane, &lo, &hi);
            else         flag_chunk_set<kMode, false>(a, lds32, my_chunk, sub, lane, &lo, &hi);
        }
        if (lane < here) a.flags[my_chunk] = ((uint64_t) hi << 32) | lo;
    }
}

// kMode 1 / 2: the cache bitmap / its coarse companion is first copied into dynamic LDS (rounded up to
// 16 bytes).  count > 0: the work lists of the group's `count` mini-batches, one after the other (they read
// the same cache, so the bitmap is staged once); count == 0: every aligned chunk of the CSR entry array,
// with the template's own cache pointers (the pass a cache draw runs over the whole graph).
template <int kMode>
__global__ void k_flag_chunks(LayerArgs g, int count, int64_t all_chunks)
{
    extern __shared__ uint4 lds_bitmap16[];
    SampleArgs a = count > 0 ? bind_sample(g, 0) : g.s;
    if (kMode == 1 || kMode == 2) {
        const uint4* src = reinterpret_cast<const uint4*>(kMode == 1 ? a.cache_bitmap : a.coarse_bitmap);
        const int64_t n16 = ((kMode == 1 ? a.bitmap_words : a.coarse_words) + 1) / 2;
        constexpr int kFill = 4;
        for (int64_t base = 0; base < n16; base += (int64_t) blockDim.x * kFill) {
            uint4 v[kFill];
#pragma unroll
            for (int i = 0; i < kFill; ++i) {
                const int64_t q = base + (int64_t) i * blockDim.x + threadIdx.x;
                v[i] = src[q < n16 ? q : n16 - 1];
            }
#pragma unroll
            for (int i = 0; i < kFill; ++i) {
                const int64_t q = base + (int64_t) i * blockDim.x + threadIdx.x;
                if (q < n16) lds_bitmap16[q] = v[i];
            }
        }
        __syncthreads();
    }
    const uint32_t* lds32 = reinterpret_cast<const uint32_t*>(lds_bitmap16);
    if (count == 0) { flag_work_list<kMode>(a, lds32, all_chunks, 0); return; }
    for (int b = 0; b < count; ++b) {
        if (b > 0) a = bind_sample(g, b);
        flag_work_list<kMode>(a, lds32, (int64_t) a.st->plan_chunks, 1);
    }
}

// group-wide helpers for G consecutive lanes (G a power of two)
template <int G>
__device__ __forceinline__ int32_t group_inclusive_scan(int32_t v, int s)
{
#pragma unroll
    for (int d = 1; d < G; d <<= 1) {
        const int32_t up = __shfl_up(v, d, G);
        if (s >= d) v += up;
    }
    return v;
}

constexpr int kHubWords = 4;        // flag words a lane holds per step when the whole wave walks a hub row

// One dst row per group of G consecutive lanes (s = lane within the group): count the row's
// eligible neighbors from its flag words, draw, map the chosen ranks back to CSR positions and
// emit.  A step covers G * W words, lane s holding words s*W .. s*W+W-1 of it,
// so ranks run in lane order.  Every lane of the wave must call it (it exchanges data between
// lanes); `live` says whether this lane's group has a row.
template <int G, int W>
__device__ __forceinline__ void select_row(const SampleArgs& a, int64_t row, bool live, int s, int64_t start,
                                           int64_t end, int32_t vi)
{
    const int k = a.fanout;
    const int32_t nw = live ? chunks_touched(start, end) : 0;     // flag words of this row
    const int64_t g0 = start >> 6;
    const uint64_t head_mask = ~0ull << (start & 63);
    const int tail_bits = (int) (end & 63);
    const uint64_t tail_mask = tail_bits ? ((1ull << tail_bits) - 1ull) : ~0ull;

    auto load_words = [&](int32_t j0, uint64_t* w) -> int32_t {
        int32_t c = 0;
#pragma unroll
        for (int i = 0; i < W; ++i) {
            const int32_t j = j0 + i;
            uint64_t x = 0;
            if (j < nw) {
                x = a.flags[g0 + j];
                if (j == 0) x &= head_mask;
                if (j == nw - 1) x &= tail_mask;
            }
            w[i] = x;
            c += __popcll(x);
        }
        return c;
    };

    // pass 1: N_C(v) = set bits of the row's flag words, trimmed to [start, end)
    uint32_t m = 0;
    uint64_t w_first[W];
    int32_t incl_first = 0;
#pragma unroll
    for (int i = 0; i < W; ++i) w_first[i] = 0;
    for (int32_t it = 0; __any(it * G * W < nw); ++it) {
        uint64_t w[W];
        const int32_t c = load_words((it * G + s) * W, w);
        const int32_t incl = group_inclusive_scan<G>(c, s);
        if (it == 0) {
#pragma unroll
            for (int i = 0; i < W; ++i) w_first[i] = w[i];
            incl_first = incl;
        }
        m += (uint32_t) __shfl(incl, G - 1, G);
    }

    uint32_t val;
    int pos;
    floyd_in_group<G>(m > (uint32_t) k ? m : (uint32_t) k + 1u, k, k, a.st->key0, a.st->key1, a.layer_number,
                      (uint32_t) vi, s, &val, &pos);
    const int cnt = (m > (uint32_t) k) ? k : (int) m;
    if (m <= (uint32_t) k) { val = (uint32_t) s; pos = s; }

    // pass 2: lane s < count finds the lane, then the word, then the bit that holds its rank `want` among
    // the set bits of the row's words (of their complements inside the row when `inverted`)
    auto locate = [&](uint32_t want, int count, bool inverted) -> int64_t {
        int64_t entry = -1;
        uint32_t run = 0;
        for (int32_t it = 0; __any(it * G * W < nw); ++it) {
            uint64_t w[W];
            int32_t incl = incl_first;
#pragma unroll
            for (int i = 0; i < W; ++i) w[i] = w_first[i];
            if (it > 0) incl = group_inclusive_scan<G>(load_words((it * G + s) * W, w), s);   // long rows reload
            if (inverted) {
                // entries of the row that are not flagged: complement inside [start, end)
                int32_t c = 0;
#pragma unroll
                for (int i = 0; i < W; ++i) {
                    const int32_t j = (it * G + s) * W + i;
                    uint64_t valid = (j < nw) ? ~0ull : 0ull;
                    if (j == 0) valid &= head_mask;
                    if (j == nw - 1) valid &= tail_mask;
                    w[i] = ~w[i] & valid;
                    c += __popcll(w[i]);
                }
                incl = group_inclusive_scan<G>(c, s);
            }
            const uint32_t step_total = (uint32_t) __shfl(incl, G - 1, G);
            const bool mine = s < count && entry < 0 && want >= run && want < run + step_total;
            const uint32_t local = want - run;
            // owner = number of lanes whose inclusive count is <= local
            int owner = 0;
            if (G == 64) {
                // the whole wave is one group: one ballot per drawn slot instead of one shuffle per lane
                for (int q = 0; q < k; ++q) {
                    const uint32_t local_q = (uint32_t) __shfl((int) local, q, G);
                    const int below = __popcll(__ballot((uint32_t) incl <= local_q));
                    if (s == q) owner = below;
                }
            } else {
                for (int t = 0; t < G; ++t) owner += ((uint32_t) __shfl(incl, t, G) <= local) ? 1 : 0;
            }
            owner = owner < G ? owner : G - 1;
            uint64_t wo[W];
            int32_t own_total = 0;
#pragma unroll
            for (int i = 0; i < W; ++i) {
                wo[i] = __shfl(w[i], owner, G);
                own_total += __popcll(wo[i]);
            }
            const int32_t incl_owner = __shfl(incl, owner, G);
            if (mine) {
                int32_t rest = (int32_t) local - (incl_owner - own_total);       // rank inside the owner's words
                int which = 0;
                uint64_t word = wo[0];
#pragma unroll
                for (int i = 0; i < W - 1; ++i) {
                    const int32_t c = __popcll(wo[i]);
                    if (which == i && rest >= c) { rest -= c; which = i + 1; word = wo[i + 1]; }
                }
                const int bit = select_bit64(word, rest);
                entry = (g0 + ((int64_t) it * G + owner) * W + which) * 64 + bit;
            }
            run += step_total;
        }
        return entry;
    };

    const int64_t entry = locate(val, cnt, false);
    if (live && s < cnt) {
        const int32_t u = a.indices[entry];
        // Section 3.4: coefficient p^C_u * k / min(k, N_C(v)), weight = 1 / coefficient; p^C_u comes
        // from the table filled when the cache was drawn (u is in the cache); fp32 from here on
        const float inv_pc = a.node_inv_pc[u];
        float wgt;
        if (a.wmode == GNS_W_UNBIASED) wgt = inv_pc * ((float) m / (float) cnt);
        else                           wgt = inv_pc * ((float) cnt / (float) k);
        a.s_w[row * k + pos] = wgt;
        a.s_nbr[row * k + pos] = mark_if_new(a, (uint32_t) u);
    }

    // Section 3.3: a row with fewer than k cached neighbors fills up from its other neighbors, drawn
    // uniformly without replacement with the row's next Philox slots (cnt, cnt + 1, ...).
    int total = cnt;
    if (a.policy == GNS_CACHE_FIRST) {
        const uint32_t others = live ? (uint32_t) (end - start) - m : 0u;        // |N(v) \ C|
        const int room = k - cnt;
        const int fill = (others > (uint32_t) room) ? room : (int) others;
        if (__any(fill > 0)) {
            uint32_t fval;
            int fpos;
            floyd_in_group<G>(others > (uint32_t) room ? others : (uint32_t) room + 1u, room, k, a.st->key0,
                              a.st->key1, a.layer_number, (uint32_t) vi, s, &fval, &fpos, cnt);
            if (others <= (uint32_t) room) { fval = (uint32_t) s; fpos = s; }
            const int64_t fentry = locate(fval, fill, true);
            if (live && s < fill) {
                const int32_t u = a.indices[fentry];
                // fill neighbors: weight 1 (a node-wise sample), or the inverse inclusion probability of a
                // uniform subset of the uncached neighbors in the unbiased mode
                const float wgt = (a.wmode == GNS_W_UNBIASED) ? (float) others / (float) fill : 1.0f;
                a.s_w[row * k + cnt + fpos] = wgt;
                a.s_nbr[row * k + cnt + fpos] = mark_if_new(a, (uint32_t) u);
            }
            total = cnt + fill;
        }
    }
    if (live && s == 0) {
        a.s_cnt[row] = total;
        a.row_eligible[row] = (int32_t) m;
    }
}

// G lanes per dst row, one flag word per lane and step.  Hub rows (listed when their nodes joined
// the batch) would keep the rest of their wave waiting, so for G < 64 the row blocks skip them
// and hub_blocks further blocks give each of them a whole wave (64 * kHubWords words per step).
// Block order: hub blocks, row blocks, relabel blocks of the previous layer.
template <int G>
__global__ void __launch_bounds__(kBlock) k_select_rows(LayerArgs g, int relabel_blocks, int hub_blocks)
{
    const int64_t own_blocks = (int64_t) gridDim.x - relabel_blocks;
    if ((int64_t) blockIdx.x >= own_blocks) {
        relabel_body(bind_finish(g, (int) blockIdx.y, false), (int64_t) blockIdx.x - own_blocks, relabel_blocks);
        return;
    }
    const SampleArgs a = bind_sample(g, (int) blockIdx.y);
    const int wave_in_block = __builtin_amdgcn_readfirstlane((int) (threadIdx.x >> 6));
    if ((int) blockIdx.x < hub_blocks) {
        const int32_t H = a.st->hub_count;
        const int32_t nhw = hub_blocks * (kBlock / kWave);
        for (int32_t h = (int32_t) blockIdx.x * (kBlock / kWave) + wave_in_block; h < H; h += nhw) {
            const int lane = opaque_lane_id();
            const int32_t row = a.hub_rows[h];
            const RowExtent ext = a.row_ext[row];
            const int32_t vi = a.dst_nodes[row];
            select_row<64, kHubWords>(a, row, true, lane, ext.start, ext.end, vi);
        }
        return;
    }
    const int64_t block = (int64_t) blockIdx.x - hub_blocks;
    const int64_t nblocks = own_blocks - hub_blocks;
    const int32_t R = a.st->num_dst[a.layer_index];
    constexpr int kRowsPerWave = kWave / G;
    const int64_t wave_global = block * (kBlock / kWave) + wave_in_block;
    const int64_t num_waves = nblocks * (kBlock / kWave);
    for (int64_t row0 = wave_global * kRowsPerWave; row0 < R; row0 += num_waves * kRowsPerWave) {
        const int lane = opaque_lane_id();
        const int s = lane & (G - 1);
        const int64_t row = row0 + (lane / G);
        bool live = row < R;
        int32_t vi = -1;
        int64_t start = 0, end = 0;
        if (live) {
            const RowExtent ext = a.row_ext[row];
            vi = a.dst_nodes[row];
            start = ext.start;
            end = ext.end;
        }
        if (hub_blocks > 0 && is_hub_extent(start, end)) live = false;      // taken by a hub wave
        select_row<G, 1>(a, row, live, s, start, end, vi);
    }
}

// The cache pointers of the template are those of generation `cache_gen`; kernels that serve mini-batches
// shift them to the generation each batch reads.
static void fill_sample_template_gen(gns_ctx* c, int layer_index, int cache_gen, SampleArgs* out)
{
    const Layout& L = c->lay;
    SampleArgs& a = *out;
    memset(&a, 0, sizeof(a));
    a.layer_index = layer_index;
    a.layer_number = (uint32_t) (c->config.num_layers - layer_index);
    a.fanout = c->config.fanout[layer_index];
    a.wmode = c->config.wmode;
    a.policy = c->config.policy[layer_index];
    a.num_nodes = c->graph.num_nodes;
    a.indptr = c->graph.indptr;
    a.indices = c->graph.indices;
    const int gen = cache_gen;
    a.node_inv_pc = c->uses_cache ? cache_ptr<float>(c, L.node_pc, gen) : nullptr;
    a.cache_bitmap = cache_ptr<uint64_t>(c, L.cache_bitmap, gen);
    a.cache_prefix = cache_ptr<int32_t>(c, L.cache_prefix, gen);
    a.cache_size = c->config.cache_size;
    a.hmask = L.hash_cap - 1;
    a.hshift = 32u - (uint32_t) __builtin_ctz(L.hash_cap);
    a.num_entries = c->graph.num_entries;
    a.flags = c->uses_cache ? cache_ptr<uint64_t>(c, L.edge_flags, gen) : nullptr;
    a.bitmap_words = L.words;
    a.coarse_bitmap = L.coarse_shift ? cache_ptr<uint64_t>(c, L.coarse_bitmap, gen) : nullptr;
    a.coarse_words = L.coarse_words;
    a.coarse_shift = L.coarse_shift;
    const bool induced = c->uses_cache && c->config.flag_mode == GNS_FLAGS_PER_CACHE;
    a.srec = induced ? cache_ptr<ChunkRec>(c, L.srec, gen) : nullptr;
    a.s_nodes = induced ? cache_ptr<int32_t>(c, L.s_nodes, gen) : nullptr;
}

void fill_sample_template(gns_ctx* c, int layer_index, SampleArgs* out)
{
    fill_sample_template_gen(c, layer_index, 0, out);
}

static void launch_flag_kernel(gns_ctx* c, const LayerArgs& a, int count, int64_t all_chunks, hipStream_t s)
{
    const size_t lds_bytes = (size_t) ((c->lay.words + 1) / 2) * 16;
    const size_t coarse_bytes = (size_t) ((c->lay.coarse_words + 1) / 2) * 16;
    if (lds_bytes <= c->lds_bitmap_limit)
        hipLaunchKernelGGL((k_flag_chunks<1>), dim3((unsigned) c->num_cus), dim3(1024), lds_bytes, s, a, count, all_chunks);
    else if (c->lay.coarse_shift > 0 && coarse_bytes <= c->lds_bitmap_limit)
        hipLaunchKernelGGL((k_flag_chunks<2>), dim3((unsigned) c->num_cus), dim3(1024), coarse_bytes, s, a, count, all_chunks);
    else if (c->lay.coarse_shift > 0 && !getenv("GNS_NO_COARSE_L2"))
    {
        const int per_cu = getenv("GNS_FLAG_BLOCKS_PER_CU") ? atoi(getenv("GNS_FLAG_BLOCKS_PER_CU")) : 2;
        hipLaunchKernelGGL((k_flag_chunks<3>), dim3((unsigned) (c->num_cus * per_cu)), dim3(kBlock), 0, s, a, count, all_chunks);
    }
    else
    {
        // every wave keeps 32 x 64 bitmap reads in flight, so a few waves per CU already reach the rate the
        // memory system gives scattered reads; a grid that filled the chip would keep the kernels of other
        // streams out for the whole pass
        const int per_cu = getenv("GNS_FLAG_BLOCKS_PER_CU") ? atoi(getenv("GNS_FLAG_BLOCKS_PER_CU")) : 2;
        hipLaunchKernelGGL((k_flag_chunks<0>), dim3((unsigned) (c->num_cus * per_cu)), dim3(kBlock), 0, s, a, count, all_chunks);
    }
}

// GNS_FLAGS_PER_CACHE: one pass over every aligned chunk of the CSR entry array, for the copy of the cache
// structures a draw is filling.
hipError_t launch_flag_all_entries(gns_ctx* c, int cache_gen, hipStream_t s)
{
    LayerArgs a;
    memset(&a, 0, sizeof(a));
    fill_sample_template_gen(c, 0, cache_gen, &a.s);
    launch_flag_kernel(c, a, 0, (c->graph.num_entries + 63) / 64, s);
    return hipGetLastError();
}

// One layer's sampler launches for a group of mini-batches.  The previous layer's relabel rides in front
// of this layer's first kernel: both only need that layer's phase 3, and they touch disjoint memory
// (sampler scratch alternates by layer).
hipError_t launch_sample_layer(const Group& g, int layer_index, hipStream_t s)
{
    gns_ctx* c = g.ctx[0];
    const Layout& L = c->lay;
    LayerArgs a;
    fill_group_args(g, &a);
    set_group_layer(g, layer_index, &a);
    fill_sample_template(c, layer_index, &a.s);
    int rl = 0;
    if (layer_index > 0) {
        fill_finish_template(c, layer_index - 1, &a.f);
        rl = relabel_grid(c, layer_index - 1);
    }
    const unsigned gy = (unsigned) g.count;

    const int64_t rows_max = L.rows[layer_index];
    const int G = (a.s.fanout <= 8) ? 8 : (a.s.fanout <= 16) ? 16 : 64;
    const int64_t rows_per_block = kBlock / G;
    int64_t row_blocks = (rows_max + rows_per_block - 1) / rows_per_block;
    // One step of rows per wave where that fits: rows differ a lot in cost, and with more blocks
    // than the chip holds the dispatcher hands out new rows as waves finish.
    const int64_t cap = (int64_t) c->num_cus * 64;
    if (row_blocks > cap) row_blocks = cap;
    if (row_blocks < 1) row_blocks = 1;
    const dim3 tb(kBlock);

#define GNS_LAUNCH_BY_G(KERNEL, RL, ...)                                                         \
    do {                                                                                         \
        if (G == 8)       hipLaunchKernelGGL((KERNEL<8>), rb, tb, 0, s, a, (RL), ##__VA_ARGS__);  \
        else if (G == 16) hipLaunchKernelGGL((KERNEL<16>), rb, tb, 0, s, a, (RL), ##__VA_ARGS__); \
        else              hipLaunchKernelGGL((KERNEL<64>), rb, tb, 0, s, a, (RL), ##__VA_ARGS__); \
    } while (0)

    // fan-outs up to 16: one row per lane, for UNIFORM layers and for CACHE_ONLY layers that have the induced subgraph
    const int policy = c->config.policy[layer_index];
    const bool induced = policy == GNS_CACHE_ONLY && c->config.flag_mode == GNS_FLAGS_PER_CACHE;
    // (one row per lane needs many rows to fill the chip: 64 rows make one wave)
    const int64_t lane_rows_min = getenv("GNS_LANE_ROWS_MIN") ? atoll(getenv("GNS_LANE_ROWS_MIN")) : 262144;
    const bool enough_rows = induced || rows_max * g.count >= lane_rows_min;
    if (a.s.fanout <= 16 && (policy == GNS_UNIFORM || induced) && enough_rows && !getenv("GNS_NO_LANE_SAMPLER")) {
        StageTimer t(c, GNS_STAGE_SELECT, s, induced);
        int64_t lane_blocks = (rows_max + kBlock - 1) / kBlock;
        if (lane_blocks > cap) lane_blocks = cap;
        const dim3 lb((unsigned) (lane_blocks + rl), gy);
        if (induced) {
            if (a.s.fanout <= 8) hipLaunchKernelGGL((k_sample_lane<8, true>), lb, tb, 0, s, a, rl);
            else                 hipLaunchKernelGGL((k_sample_lane<16, true>), lb, tb, 0, s, a, rl);
        } else {
            if (a.s.fanout <= 8) hipLaunchKernelGGL((k_sample_lane<8, false>), lb, tb, 0, s, a, rl);
            else                 hipLaunchKernelGGL((k_sample_lane<16, false>), lb, tb, 0, s, a, rl);
        }
        return hipGetLastError();
    }

    if (policy == GNS_UNIFORM) {
        const dim3 rb((unsigned) (row_blocks + rl), gy);
        GNS_LAUNCH_BY_G(k_sample_uniform, rl);
        return hipGetLastError();
    }

    // CACHE_ONLY: (plan -> flag ->) select
    if (c->config.flag_mode == GNS_FLAGS_PER_BATCH) {
        {
            StageTimer t(c, GNS_STAGE_PLAN, s);
            const unsigned plan_blocks = (unsigned) ((rows_max + kPlanTile - 1) / kPlanTile);
            hipLaunchKernelGGL(k_plan_count, dim3(plan_blocks + (unsigned) rl, gy), tb, 0, s, a, rl);
            hipLaunchKernelGGL(k_plan_expand, dim3(plan_blocks, gy), tb, 0, s, a);
        }
        rl = 0;                          // done with the plan kernel
        StageTimer t(c, GNS_STAGE_FLAG, s);
        launch_flag_kernel(c, a, g.count, 0, s);
    }
    StageTimer t(c, GNS_STAGE_SELECT, s);
    // hub rows get dedicated waves (the count lives on the device; the waves stride over the list)
    const int hub_blocks = (G < 64) ? (int) (rows_max / (kBlock / kWave) < (int64_t) c->num_cus * 2
                                                 ? rows_max / (kBlock / kWave) + 1 : (int64_t) c->num_cus * 2) : 0;
    const dim3 rb((unsigned) (row_blocks + rl + hub_blocks), gy);
    GNS_LAUNCH_BY_G(k_select_rows, rl, hub_blocks);
#undef GNS_LAUNCH_BY_G
    return hipGetLastError();
}

}  // namespace gns
