// Layer sampler: for every dst row v independently, N_l(v) <- sample(N(v), C)
// (paper Algorithm 1, top-down loop).
//
//   UNIFORM     Section 2.1: min(k, deg(v)) neighbors uniformly without
//               replacement.  Only the k chosen CSR entries are read.
//   CACHE_ONLY  Sections 3.3 and 4.1: the eligible list is the row's entries
//               whose node is in the cache, in CSR order; min(k, N_C(v)) of
//               them are chosen; each carries the Section 3.4 weight.
//
// The without-replacement choice is Robert Floyd's subset algorithm on ranks
// of the eligible list, driven by k Philox words keyed by (seed, layer, node,
// slot); the chosen ranks are emitted in ascending order.  All decisions are
// integer arithmetic, so the sample does not depend on scheduling.
//
// Output per row r (fixed stride k): s_nbr[r*k + i], s_w[r*k + i] for
// i < s_cnt[r], row_eligible[r]; every emitted id also sets its bit in the
// node-indexed mark bitmap that the frontier stage turns into the src list.
#include "gns_internal.h"
#include "gns_device.hpp"

namespace gns {

struct SampleArgs {
    DeviceState* st;
    int layer_index;
    uint32_t layer_number;     // the paper's l = L - layer_index
    int fanout;
    int wmode;
    uint32_t key0, key1;       // Philox key = (lo32(seed), hi32(seed))
    int64_t num_nodes;
    const void* indptr;
    const int32_t* indices;
    const int32_t* dst_nodes;
    const uint64_t* cache_bitmap;
    const int32_t* cache_prefix;
    const double* cache_inv_pc;
    int32_t* s_nbr;
    float* s_w;
    int32_t* s_cnt;
    int32_t* row_eligible;
    uint64_t* mark;
};

// Floyd's subset draw inside a group of G consecutive lanes (G a power of two
// <= 64, k <= G).  Lane s < k ends up with one chosen rank in *val and that
// rank's position in ascending order in *pos.  Requires m > k.  Every lane of
// the group must call it.
template <int G>
__device__ __forceinline__ void floyd_in_group(uint32_t m, int k, uint32_t key0, uint32_t key1, uint32_t layer,
                                               uint32_t node, int s, uint32_t* val, int* pos)
{
    s = opaque(s);
    // slot s draws t_s uniform in [0, m-k+s]
    const Philox4 r = philox4x32_10(node, (uint32_t) s >> 2, layer, kTagNeighbor, key0, key1);
    const int sel = s & 3;
    const uint32_t word = sel == 0 ? r.w[0] : sel == 1 ? r.w[1] : sel == 2 ? r.w[2] : r.w[3];
    const uint32_t j_own = m - (uint32_t) k + (uint32_t) s;
    const uint32_t t_own = __umulhi(word, j_own + 1u);
    uint32_t chosen = 0xFFFFFFFFu;              // not yet decided
    const int group_base = opaque_lane_id() & ~(G - 1);
    const uint64_t group_mask = (G == 64) ? ~0ull : (((1ull << G) - 1ull) << group_base);
    for (int q = 0; q < k; ++q) {
        const uint32_t t_q = __shfl(t_own, q, G);
        // is t_q already among the ranks decided by slots < q ?
        const uint64_t hit = __ballot(s < q && chosen == t_q) & group_mask;
        if (s == q) chosen = hit ? j_own : t_own;
    }
    int rank = 0;
    for (int q = 0; q < k; ++q) {
        const uint32_t c_q = __shfl(chosen, q, G);
        rank += (c_q < chosen) ? 1 : 0;
    }
    *val = chosen;
    *pos = rank;
}

__device__ __forceinline__ void mark_node(uint64_t* mark, uint32_t u)
{
    atomicOr(reinterpret_cast<unsigned long long*>(&mark[u >> 6]), 1ull << (u & 63u));
}

// ---------------------------------------------------------------------------
// UNIFORM: G lanes per row, rows assigned round-robin to groups.
template <typename OffT, int G>
__global__ void __launch_bounds__(kBlock) k_sample_uniform(SampleArgs a)
{
    const int32_t R = a.st->num_dst[a.layer_index];
    const int k = a.fanout;
    constexpr int kRowsPerWave = kWave / G;
    // The loop bounds live in scalar registers (readfirstlane) so that the whole wave
    // provably iterates together: the draw below exchanges data between lanes.
    const int64_t wave_global = (int64_t) blockIdx.x * (kBlock / kWave) +
                                __builtin_amdgcn_readfirstlane((int) (threadIdx.x >> 6));
    const int64_t num_waves = (int64_t) gridDim.x * (kBlock / kWave);
    for (int64_t row0 = wave_global * kRowsPerWave; row0 < R; row0 += num_waves * kRowsPerWave) {
        const int lane = opaque_lane_id();
        const int s = lane & (G - 1);
        const int64_t row = row0 + (lane / G);
        const bool live = row < R;
        int64_t start = 0;
        uint32_t m = 0;
        uint32_t v = 0;
        if (live) {
            const int32_t vi = a.dst_nodes[row];
            if (vi >= 0 && (int64_t) vi < a.num_nodes) {
                v = (uint32_t) vi;
                start = load_off<OffT>(a.indptr, vi);
                m = (uint32_t) (load_off<OffT>(a.indptr, (int64_t) vi + 1) - start);
            }
        }
        uint32_t val;
        int pos;
        // run the draw with a safe size in every lane, then keep it only where it applies
        floyd_in_group<G>(m > (uint32_t) k ? m : (uint32_t) k + 1u, k, a.key0, a.key1, a.layer_number, v, s, &val, &pos);
        const int cnt = (m > (uint32_t) k) ? k : (int) m;
        if (m <= (uint32_t) k) { val = (uint32_t) s; pos = s; }
        if (live && s < cnt) {
            const int32_t u = a.indices[start + val];
            a.s_nbr[row * k + pos] = u;
            a.s_w[row * k + pos] = 1.0f;
            mark_node(a.mark, (uint32_t) u);
        }
        if (live && s == 0) {
            a.s_cnt[row] = cnt;
            a.row_eligible[row] = (int32_t) m;
        }
    }
}

// ---------------------------------------------------------------------------
// CACHE_ONLY: one wave per row, rows handed out through an atomic queue.
// The row is streamed in chunks of 64 entries (kUnroll chunks in flight); each
// chunk's cache-membership ballot is kept in LDS together with the running
// count, so that after the draw the chosen ranks are mapped back to CSR
// positions without a second pass.  Rows longer than one LDS segment are
// counted first and then resolved segment by segment.
constexpr int kUnroll = 4;
constexpr int kSegChunks = 256;                        // chunks (of 64 entries) per LDS segment
constexpr int kSegEntries = kSegChunks * kWave;        // 16384 entries
constexpr int kWavesPerBlock = kBlock / kWave;

struct RowScan {
    uint64_t* masks;      // LDS, [kSegChunks]
    uint32_t* prefix;     // LDS, [kSegChunks] eligible entries before the chunk, within the segment
};

// Streams `len` entries starting at `idx`; returns the number of cached ones.
// With kStore the chunk ballots and prefixes go to LDS.
template <bool kStore>
__device__ __forceinline__ uint32_t scan_segment(const int32_t* idx, int32_t len, const uint64_t* bitmap,
                                                 const RowScan& rs)
{
    uint32_t running = 0;
    for (int32_t base = 0; base < len; base += kUnroll * kWave) {
        const int lane = opaque_lane_id();
        int32_t u[kUnroll];
        bool in[kUnroll];
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) {
            const int32_t e = base + i * kWave + lane;
            in[i] = e < len;
            u[i] = in[i] ? idx[e] : 0;
        }
        uint64_t ballots[kUnroll];
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) {
            const bool hit = in[i] && bitmap_test(bitmap, (uint32_t) u[i]);
            ballots[i] = __ballot(hit);
        }
        // lane i (< kUnroll) records chunk i: its ballot and the count of eligible entries before it
        uint64_t my_mask = ballots[0];
        uint32_t my_prefix = running;
        uint32_t acc = running;
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) {
            if (lane == i) { my_mask = ballots[i]; my_prefix = acc; }
            acc += (uint32_t) __popcll(ballots[i]);
        }
        if (kStore) {
            if (lane < kUnroll && base + lane * kWave < len) {
                rs.masks[(base >> 6) + lane] = my_mask;
                rs.prefix[(base >> 6) + lane] = my_prefix;
            }
        }
        running = acc;
    }
    return running;
}

// Next row of the work queue, the same value in every lane.  Lane 0 performs the atomic and
// the result is broadcast through a scalar register.  The lane test uses an opaque id so that
// the branch stays inside the caller's loop (see opaque()).
__device__ __forceinline__ int32_t claim_row(int32_t* queue)
{
    int32_t v = 0;
    if (opaque_lane_id() == 0) v = atomicAdd(queue, 1);
    return __builtin_amdgcn_readfirstlane(v);
}

template <typename OffT>
__global__ void __launch_bounds__(kBlock) k_sample_cache_only(SampleArgs a)
{
    __shared__ uint64_t lds_masks[kWavesPerBlock][kSegChunks];
    __shared__ uint32_t lds_prefix[kWavesPerBlock][kSegChunks];
    const int wave = (int) (threadIdx.x >> 6);
    RowScan rs{lds_masks[wave], lds_prefix[wave]};
    const int32_t R = a.st->num_dst[a.layer_index];
    const int k = a.fanout;

    // Rows are dealt round-robin to the waves of the grid.  (A single atomic row counter was
    // measured first: same-address atomics serialise at roughly 12 ns each, which alone cost
    // 1 ms for 85K rows.)  Row index, node and row extent are wave-uniform scalars
    // (readfirstlane): every loop below branches on scalar conditions and the wave stays
    // converged around the ballots and the LDS exchange.
    const int32_t wave_global = (int32_t) blockIdx.x * kWavesPerBlock + __builtin_amdgcn_readfirstlane(wave);
    const int32_t num_waves = (int32_t) gridDim.x * kWavesPerBlock;
    for (int32_t row = wave_global; row < R; row += num_waves) {
        const int lane = opaque_lane_id();

        const int32_t vi = __builtin_amdgcn_readfirstlane(a.dst_nodes[row]);
        int64_t start = 0, deg = 0;
        if (vi >= 0 && (int64_t) vi < a.num_nodes) {
            const int64_t b = load_off<OffT>(a.indptr, vi);
            const int64_t e = load_off<OffT>(a.indptr, (int64_t) vi + 1);
            start = ((int64_t) __builtin_amdgcn_readfirstlane((int) (b >> 32)) << 32) |
                    (uint32_t) __builtin_amdgcn_readfirstlane((int) (uint32_t) b);
            deg = (int64_t) __builtin_amdgcn_readfirstlane((int) (e - b));
        }
        const int32_t* row_idx = a.indices + start;
        const int64_t num_seg = (deg + kSegEntries - 1) / kSegEntries;

        uint32_t m = 0;                                        // N_C(v)
        if (num_seg > 1) {
            for (int64_t sg = 0; sg < num_seg; ++sg) {
                const int64_t off = sg * kSegEntries;
                const int32_t len = (int32_t) ((deg - off < kSegEntries) ? (deg - off) : kSegEntries);
                m += scan_segment<false>(row_idx + off, len, a.cache_bitmap, rs);
            }
        }

        uint32_t val = 0;
        int pos = 0;
        int cnt = 0;
        bool drawn = false;
        uint32_t seen = 0;                                     // eligible entries in earlier segments
        for (int64_t sg = 0; sg < num_seg; ++sg) {
            const int64_t off = sg * kSegEntries;
            const int32_t len = (int32_t) ((deg - off < kSegEntries) ? (deg - off) : kSegEntries);
            const uint32_t here = scan_segment<true>(row_idx + off, len, a.cache_bitmap, rs);
            if (num_seg == 1) m = here;
            if (!drawn) {
                drawn = true;
                floyd_in_group<kWave>(m > (uint32_t) k ? m : (uint32_t) k + 1u, k, a.key0, a.key1, a.layer_number,
                                      (uint32_t) vi, lane, &val, &pos);
                cnt = (m > (uint32_t) k) ? k : (int) m;
                if (m <= (uint32_t) k) { val = (uint32_t) lane; pos = lane; }
            }
            // make the LDS writes of this wave visible to all of its lanes
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (opaque_lane_id() < cnt && val >= seen && val < seen + here) {
                const uint32_t local = val - seen;
                // last chunk whose prefix is <= local
                const int chunks = (len + kWave - 1) / kWave;
                int lo = 0, hi = chunks;                       // answer in [lo, hi)
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (rs.prefix[mid] <= local) lo = mid; else hi = mid;
                }
                const int bit = select_bit64(rs.masks[lo], (int) (local - rs.prefix[lo]));
                const int32_t u = row_idx[off + (int64_t) lo * kWave + bit];
                const int32_t slot = bitmap_rank(a.cache_bitmap, a.cache_prefix, (uint32_t) u);
                const double inv_pc = a.cache_inv_pc[slot];
                double w;
                if (a.wmode == GNS_W_UNBIASED) w = inv_pc * (double) m / (double) cnt;
                else                           w = inv_pc * (double) cnt / (double) k;
                a.s_nbr[(int64_t) row * k + pos] = u;
                a.s_w[(int64_t) row * k + pos] = (float) w;
                mark_node(a.mark, (uint32_t) u);
            }
            seen += here;
            // the next segment overwrites the LDS arrays: wait until every lane has read them
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        if (lane == 0) {
            a.s_cnt[row] = (m > (uint32_t) k) ? k : (int32_t) m;
            a.row_eligible[row] = (int32_t) m;
        }
    }
}

hipError_t launch_sample_layer(gns_ctx* c, int layer_index, uint64_t seed, const int32_t* dst_nodes,
                               int32_t* row_eligible, hipStream_t s)
{
    const Layout& L = c->lay;
    SampleArgs a;
    a.st = c->d_state;
    a.layer_index = layer_index;
    a.layer_number = (uint32_t) (c->config.num_layers - layer_index);
    a.fanout = c->config.fanout[layer_index];
    a.wmode = c->config.wmode;
    a.key0 = (uint32_t) seed;
    a.key1 = (uint32_t) (seed >> 32);
    a.num_nodes = c->graph.num_nodes;
    a.indptr = c->graph.indptr;
    a.indices = c->graph.indices;
    a.dst_nodes = dst_nodes;
    a.cache_bitmap = ws_ptr<uint64_t>(c, L.cache_bitmap);
    a.cache_prefix = ws_ptr<int32_t>(c, L.cache_prefix);
    a.cache_inv_pc = ws_ptr<double>(c, L.cache_inv_pc);
    a.s_nbr = ws_ptr<int32_t>(c, L.s_nbr);
    a.s_w = ws_ptr<float>(c, L.s_w);
    a.s_cnt = ws_ptr<int32_t>(c, L.s_cnt);
    a.row_eligible = row_eligible;
    a.mark = ws_ptr<uint64_t>(c, L.mark_bitmap);

    const int64_t rows_max = L.rows[layer_index];
    const bool i64 = c->graph.indptr_is_i64 != 0;
    if (c->config.policy[layer_index] == GNS_UNIFORM) {
        const int G = (a.fanout <= 16) ? 16 : 64;
        const int64_t groups_per_block = kBlock / G;
        int64_t blocks = (rows_max + groups_per_block - 1) / groups_per_block;
        const int64_t cap = (int64_t) c->num_cus * 8;
        if (blocks > cap) blocks = cap;
        if (blocks < 1) blocks = 1;
        if (G == 16) {
            if (i64) hipLaunchKernelGGL((k_sample_uniform<int64_t, 16>), dim3((unsigned) blocks), dim3(kBlock), 0, s, a);
            else     hipLaunchKernelGGL((k_sample_uniform<int32_t, 16>), dim3((unsigned) blocks), dim3(kBlock), 0, s, a);
        } else {
            if (i64) hipLaunchKernelGGL((k_sample_uniform<int64_t, 64>), dim3((unsigned) blocks), dim3(kBlock), 0, s, a);
            else     hipLaunchKernelGGL((k_sample_uniform<int32_t, 64>), dim3((unsigned) blocks), dim3(kBlock), 0, s, a);
        }
    } else {
        int64_t blocks = (rows_max + kWavesPerBlock - 1) / kWavesPerBlock;
        const int64_t cap = (int64_t) c->num_cus * 8;
        if (blocks > cap) blocks = cap;
        if (blocks < 1) blocks = 1;
        if (i64) hipLaunchKernelGGL((k_sample_cache_only<int64_t>), dim3((unsigned) blocks), dim3(kBlock), 0, s, a);
        else     hipLaunchKernelGGL((k_sample_cache_only<int32_t>), dim3((unsigned) blocks), dim3(kBlock), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace gns
