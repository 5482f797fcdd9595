// Feature gather (paper Section 2.2 steps 2-3: slice the input nodes' rows;
// cached rows are already device resident, Section 3.2) and the weighted mean
// aggregation of one layer (Algorithm 1 bottom-up loop with Section 3.4's
// rescaling).  Both are pure data movement / fp32 FMA streams: a group of
// lanes owns one row and moves it with 128-bit accesses.
#include "gns_internal.h"
#include "gns_device.hpp"
#include <string.h>
#include <stdlib.h>

namespace gns {

// Output rows are written once and not read again by the writing kernel: a non-temporal store keeps
// them from displacing the rows other waves still want from L2.
__device__ __forceinline__ void store_streaming(float4* p, const float4& v)
{
    __builtin_nontemporal_store(v.x, &p->x);
    __builtin_nontemporal_store(v.y, &p->y);
    __builtin_nontemporal_store(v.z, &p->z);
    __builtin_nontemporal_store(v.w, &p->w);
}

// One launch serves a group of mini-batches: blockIdx.y picks the batch.
struct GatherBatch {
    const int32_t* nodes;
    const int32_t* num_nodes_dev;   // if not null the count is read here (num_nodes is then the worst case)
    float* out;
    int32_t num_nodes;
    int32_t pad;
};

struct GatherArgs {
    GatherBatch b[GNS_MAX_GROUP];
    int64_t n;
    int32_t feat_dim;
    int32_t use_cache;
    const uint64_t* cache_bitmap;
    const int32_t* cache_prefix;
    const float* cache_feat;
    const float* store;          // device store or device-visible pinned host store
};

// kLanes lanes per row; kVec: rows are moved as float4 (feat_dim % 4 == 0, 16-byte aligned bases)
template <int kLanes, bool kVec>
__global__ void __launch_bounds__(kBlock) k_gather(GatherArgs a)
{
    const int lane = (int) (threadIdx.x % kLanes);
    const int64_t groups_per_block = kBlock / kLanes;
    const int64_t group = (int64_t) blockIdx.x * groups_per_block + threadIdx.x / kLanes;
    const int64_t num_groups = (int64_t) gridDim.x * groups_per_block;
    const int64_t F = a.feat_dim;
    const GatherBatch q = a.b[blockIdx.y];
    const int64_t count = q.num_nodes_dev ? (int64_t) *q.num_nodes_dev : (int64_t) q.num_nodes;
    for (int64_t row = group; row < count; row += num_groups) {
        const int32_t u = q.nodes[row];
        const bool valid = u >= 0 && (int64_t) u < a.n;
        const float* src = nullptr;
        if (valid) {
            if (a.use_cache && bitmap_test(a.cache_bitmap, (uint32_t) u))
                src = a.cache_feat + (int64_t) bitmap_rank(a.cache_bitmap, a.cache_prefix, (uint32_t) u) * F;
            else
                src = a.store + (int64_t) u * F;
        }
        float* dst = q.out + row * F;
        if (kVec) {
            const float4* s4 = reinterpret_cast<const float4*>(src);
            float4* d4 = reinterpret_cast<float4*>(dst);
            for (int i = lane; i < (int) (F >> 2); i += kLanes)
                store_streaming(d4 + i, valid ? s4[i] : make_float4(0.f, 0.f, 0.f, 0.f));
        } else {
            for (int i = lane; i < (int) F; i += kLanes) dst[i] = valid ? src[i] : 0.f;
        }
    }
}

static inline int lanes_for(int64_t units)
{
    int l = 4;
    while (l < 64 && l < units) l <<= 1;
    return l;
}

template <bool kVec>
static void gather_dispatch(int lanes, dim3 blocks, hipStream_t s, const GatherArgs& a)
{
    switch (lanes) {
        case 4:  hipLaunchKernelGGL((k_gather<4, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        case 8:  hipLaunchKernelGGL((k_gather<8, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        case 16: hipLaunchKernelGGL((k_gather<16, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        case 32: hipLaunchKernelGGL((k_gather<32, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        default: hipLaunchKernelGGL((k_gather<64, kVec>), blocks, dim3(kBlock), 0, s, a); break;
    }
}

// count mini-batches (contexts ctxs[0..count) of one family) in one launch.  num_nodes[b] < 0: the input
// nodes of the last batch sampled on ctxs[b], counted on the device.
hipError_t launch_gather(gns_ctx* const* ctxs, int count, const int32_t* const* nodes, const int32_t* num_nodes,
                         float* const* out, int use_cache_gen, hipStream_t s)
{
    gns_ctx* c = ctxs[0];
    const Layout& L = c->lay;
    GatherArgs a;
    memset(&a, 0, sizeof(a));
    int64_t most = 0;
    bool aligned = true;
    for (int b = 0; b < count; ++b) {
        GatherBatch& q = a.b[b];
        q.nodes = nodes[b];
        q.out = out[b];
        q.num_nodes = num_nodes[b];
        if (num_nodes[b] < 0) {
            q.num_nodes_dev = &ctxs[b]->d_state->num_dst[c->config.num_layers];
            q.num_nodes = (int32_t) L.rows[c->config.num_layers];
        }
        if (q.num_nodes > most) most = q.num_nodes;
        aligned = aligned && (reinterpret_cast<uintptr_t>(out[b]) & 15u) == 0;
    }
    if (most == 0) return hipSuccess;
    a.n = c->graph.num_nodes;
    a.feat_dim = c->graph.feat_dim;
    const int gen = use_cache_gen < 0 ? 0 : use_cache_gen;
    a.use_cache = (use_cache_gen >= 0 && c->uses_cache && c->root->cache_valid) ? 1 : 0;
    a.cache_bitmap = cache_ptr<uint64_t>(c, L.cache_bitmap, gen);
    a.cache_prefix = cache_ptr<int32_t>(c, L.cache_prefix, gen);
    a.cache_feat = cache_ptr<float>(c, L.cache_feat, gen);
    a.store = c->graph.feat_dev ? c->graph.feat_dev : c->graph.feat_host_pinned;
    const int64_t F = a.feat_dim;
    const bool vec = (F % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.store) & 15u) == 0) && aligned;
    const int lanes = lanes_for(vec ? F / 4 : F);
    const int64_t groups_per_block = kBlock / lanes;
    int64_t blocks = (most + groups_per_block - 1) / groups_per_block;
    const int64_t cap = (int64_t) c->num_cus * 8;        // what is resident together; beyond that a group copies several rows
    if (blocks > cap) blocks = cap;
    const dim3 grid((unsigned) blocks, (unsigned) count);
    if (vec) gather_dispatch<true>(lanes, grid, s, a);
    else     gather_dispatch<false>(lanes, grid, s, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
struct AggBatch {
    const int32_t* indptr;
    const int32_t* indices;
    const float* weights;
    const float* x_src;
    float* out;
    const int32_t* num_dst_dev;     // if not null the row count is read here
    const int32_t* num_src_dev;
    int32_t num_dst;
    int32_t num_src;                // rows of x_src; an edge whose index lies outside is skipped
};

struct AggGroup {
    AggBatch b[GNS_MAX_GROUP];
    int32_t feat_dim;
};

// the view of one batch the kernel body works on
struct AggArgs : AggBatch {
    int32_t feat_dim;
};

// Rows of at most kLanes float4 columns, one column per lane: the plain form of the loop below, for widths whose
// rows do not start on cache-line boundaries or do not fill several columns per lane.  Branch-free inner loop:
// the first kSlots lanes of a row's group read one edge each (index and weight, one coalesced read), every lane
// then takes edge t from lane t of its group, so the reads of up to kSlots source rows are issued back to back;
// in a slot past its row's end a lane group stands aside (weight 0 on zeros), rows with more than kSlots edges
// take further rounds.  All lanes of the wave stay converged: trip counts are wave-uniform (the shuffles need
// every source lane).
template <int kLanes>
__device__ __forceinline__ void aggregate_rows_one_column(const AggArgs& a, int64_t group, int64_t num_groups, int64_t count,
                                                          uint32_t num_src)
{
    constexpr int kSlots = kLanes < 8 ? kLanes : 8;
    const int lane = (int) (threadIdx.x % kLanes);
    const int64_t F = a.feat_dim;
    const int64_t F4 = F >> 2;
    const int col = lane < (int) F4 ? lane : (int) F4 - 1;       // idle lanes repeat the last column
    const bool has = lane < (int) F4;
    const float4* x4 = reinterpret_cast<const float4*>(a.x_src) + col;
    // row j of x_src starts at float4 index j * F4: a shift when F4 is a power of two and the product fits
    // 32 bits (integer multiplies run at a quarter of the rate of other vector instructions)
    const bool by_shift = (F4 & (F4 - 1)) == 0 && (uint64_t) num_src * (uint64_t) F4 < ((uint64_t) 1 << 32);
    const uint32_t f4_shift = (uint32_t) __builtin_ctzll((unsigned long long) F4);
    const int64_t trips = (count + num_groups - 1) / num_groups;                 // the same for every group
    for (int64_t it = 0; it < trips; ++it) {
        const int64_t row = group + it * num_groups;
        const bool live = row < count;
        int32_t b = 0, e = 0;
        if (live) { b = a.indptr[row]; e = a.indptr[row + 1]; }
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int32_t q0 = b; __any(q0 < e); q0 += kSlots) {
            const int32_t here = e - q0 < kSlots ? (e - q0 > 0 ? e - q0 : 0) : kSlots;   // edges of this round
            const bool mine = lane < here;
            uint32_t my_j = mine ? (uint32_t) a.indices[q0 + lane] : 0u;
            float my_w = mine ? a.weights[q0 + lane] : 0.f;
            const bool bad = my_j >= num_src;                    // an index outside [0, num_src) is skipped
            if (bad) { my_j = 0u; my_w = 0.f; }
            const bool any_bad = __any(bad && mine);
            float4 x[kSlots];
            float w[kSlots];
#pragma unroll
            for (int t = 0; t < kSlots; ++t) {
                w[t] = 0.f;
                x[t] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (t < 4 || __any(t < here)) {                  // slots no row of this wave needs are skipped
                    const uint32_t j = (uint32_t) __shfl((int) my_j, t, kLanes);
                    const float wt = __shfl(my_w, t, kLanes);
                    if (t < here) {                              // a row without an edge in this slot stands aside
                        w[t] = wt;
                        x[t] = by_shift ? x4[j << f4_shift] : x4[(int64_t) j * F4];
                    }
                }
            }
            if (any_bad) {
                // rare: a skipped edge must not contribute even a NaN of the row it was redirected to
#pragma unroll
                for (int t = 0; t < kSlots; ++t)
                    if (__shfl((int) (bad && mine), t, kLanes)) x[t] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int t = 0; t < kSlots; ++t) {                    // edge order, one fma per term
                if (t < 4 || __any(t < here)) {
                    acc.x = fmaf(w[t], x[t].x, acc.x);
                    acc.y = fmaf(w[t], x[t].y, acc.y);
                    acc.z = fmaf(w[t], x[t].z, acc.z);
                    acc.w = fmaf(w[t], x[t].w, acc.w);
                }
            }
        }
        if (e > b) {                                              // (a row without edges has read nothing: 0)
            const float inv_n = 1.0f / (float) (e - b);           // one division per row, then four products
            acc.x *= inv_n; acc.y *= inv_n; acc.z *= inv_n; acc.w *= inv_n;
        }
        if (live && has) store_streaming(reinterpret_cast<float4*>(a.out + row * F) + lane, acc);
    }
}

// Rows whose features are float4-aligned and fit kLanes * kPer float4 columns: a group of kLanes lanes owns a
// dst row, lane l accumulates columns l, l + kLanes, ... (kPer of them).  Branch-free inner loop: the first
// kSlots lanes of the group hold one edge each (index and weight, one coalesced read), every lane then takes
// edge t from lane t of its group, so the reads of the source rows are issued back to back; in a slot past its
// row's end a lane group stands aside (weight 0 on zeros: the texture addressers only work for lanes that take
// part in a read), rows with more than kSlots edges take further rounds.  All lanes of the wave stay converged: trip counts are wave-uniform (the shuffles need
// every source lane).
// A row is a chain of dependent accesses (row extent -> edges -> source rows -> store); it is software-pipelined
// over the rows a group visits: while the source rows of row i are in flight, the edges of row i+1 and the
// extent of row i+2 are being read.  (What bounds the kernel on 128-float rows is the rate at which the L2s
// deliver scattered 512-byte rows next to the stream of output rows: a loop with no bookkeeping at all -- hashed
// source rows, constant weights -- is within 15 % of it, and lane layout, pipelining and grid size each move it by
// a few percent only.)
// The hardware counts outstanding vector memory operations in order, and the compiler can only leave the
// younger ones in flight across a use of an older one if it knows how many there are: a read or store inside
// a branch makes it wait for everything.  Hence every access of the steady state is unconditional -- reads
// of rows or edges that do not exist go to a valid address (the first extent) and their value is replaced,
// lanes past the last column repeat it, and the last trip, in which some groups have no row, stands apart -- and
// only rare cases (a row with more than kSlots edges, slots beyond the fourth) sit in branches.
// kOff32: every byte offset into x_src fits 32 bits and row index and row size fit 24 bits, so an address is
// the uniform base plus one 32-bit vector offset (one multiply-add per load).
template <int kLanes, int kPer, bool kOff32>
__device__ __forceinline__ void aggregate_rows(const AggArgs& a, uint32_t group, uint32_t num_groups, uint32_t count,
                                               uint32_t num_src)
{
    constexpr int kSlots = kLanes < 8 ? kLanes : 8;                      // edges a round covers (one per lane)
    constexpr int kFlight = (kPer >= 4 && kSlots > 4) ? 5 : kSlots;     // source rows read together
    const int lane = (int) (threadIdx.x % kLanes);
    const uint32_t F = (uint32_t) a.feat_dim;
    const uint32_t F4 = F >> 2;
    const uint32_t row_bytes = F * 4u;
    uint32_t col_bytes[kPer];                   // lanes past the last column repeat it
#pragma unroll
    for (int p = 0; p < kPer; ++p) {
        const uint32_t cidx = (uint32_t) lane + (uint32_t) p * kLanes;
        col_bytes[p] = (cidx < F4 ? cidx : F4 - 1u) * 16u;
    }
    const char* x_bytes = reinterpret_cast<const char*>(a.x_src);
    const uint32_t trips = (count + num_groups - 1u) / num_groups;       // the same for every group (count > 0)

    // extent of the row this group visits in trip `it` (empty past the end)
    auto extent = [&](uint32_t it, int32_t& b, int32_t& e) {
        const uint32_t row = group + it * num_groups;
        const bool ok = it < trips && row < count;
        const uint32_t r = ok ? row : 0u;
        struct __attribute__((packed, aligned(4))) Pair { int32_t lo, hi; };       // one 8-byte read, 4-byte aligned
        const Pair pr = *reinterpret_cast<const Pair*>(a.indptr + r);
        b = pr.lo;
        e = ok ? pr.hi : pr.lo;
    };
    // the edge this lane holds in the round that starts at entry q0 of a row ending at e
    auto edge = [&](int32_t q0, int32_t e, uint32_t& j, float& w) {
        const bool mine = q0 + lane < e && lane < kSlots;
        const int32_t* pj = mine ? a.indices + (q0 + lane) : a.indptr;
        const float* pw = mine ? a.weights + (q0 + lane) : reinterpret_cast<const float*>(a.indptr);
        const uint32_t jv = (uint32_t) *pj;
        const float wv = *pw;
        j = mine ? jv : 0u;
        w = mine ? wv : 0.f;
    };
    // one round: the edges (my_j, my_w) the group's lanes hold for entries [q0, e) of the row, slots [kFirst, kSlots)
    auto round = [&](int32_t q0, int32_t e, uint32_t my_j, float my_w, float4 (&acc)[kPer], auto&& between) {
        const int32_t here = e - q0 < kSlots ? (e - q0 > 0 ? e - q0 : 0) : kSlots;   // edges of this round
        const bool bad = lane < here && my_j >= num_src;         // an index outside [0, num_src) is skipped
        if (bad) { my_j = 0u; my_w = 0.f; }
        const bool any_bad = __any(bad);
#pragma unroll
        for (int t0 = 0; t0 < kSlots; t0 += kFlight) {
            if (t0 > 0 && !__any(t0 < here)) break;              // no row of this wave has that many edges
            float4 x[kFlight][kPer];
            float w[kFlight];
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                const int t = t0 + u;
                w[u] = 0.f;
#pragma unroll
                for (int p = 0; p < kPer; ++p) x[u][p] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (t >= kSlots || (t >= 4 && !__any(t < here))) continue;       // a slot no row of this wave needs
                const uint32_t j = (uint32_t) __shfl((int) my_j, t, kLanes);
                const float wt = __shfl(my_w, t, kLanes);
                // Lanes of rows that have no edge in this slot stand aside: the texture addressers, which bound this
                // kernel, only work for the lanes that take part in a read.
                if (t < here) {
                    w[u] = wt;
#pragma unroll
                    for (int p = 0; p < kPer; ++p) {
                        if (kOff32) {
                            const uint32_t off = __umul24(j, row_bytes) + col_bytes[p];     // both factors < 2^24
                            x[u][p] = *reinterpret_cast<const float4*>(x_bytes + off);
                        } else {
                            const uint64_t off = (uint64_t) j * row_bytes + col_bytes[p];
                            x[u][p] = *reinterpret_cast<const float4*>(x_bytes + off);
                        }
                    }
                }
            }
            if (t0 == 0) between();                              // reads for the rows ahead, behind this row's first reads
            if (any_bad) {
                // rare: a skipped edge must not contribute even a NaN of the row it was redirected to
#pragma unroll
                for (int u = 0; u < kFlight; ++u) {
                    const int t = t0 + u;
                    if (t >= kSlots) continue;
                    if (__shfl((int) bad, t, kLanes)) {
#pragma unroll
                        for (int p = 0; p < kPer; ++p) x[u][p] = make_float4(0.f, 0.f, 0.f, 0.f);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {                  // edge order, one fma per term
                if (t0 + u >= kSlots || (t0 + u >= 4 && !__any(t0 + u < here))) continue;
#pragma unroll
                for (int p = 0; p < kPer; ++p) {
                    acc[p].x = fmaf(w[u], x[u][p].x, acc[p].x);
                    acc[p].y = fmaf(w[u], x[u][p].y, acc[p].y);
                    acc[p].z = fmaf(w[u], x[u][p].z, acc[p].z);
                    acc[p].w = fmaf(w[u], x[u][p].w, acc[p].w);
                }
            }
        }
    };

    // one row: its first round with the reads for the rows ahead slipped in, further rounds if it has more than
    // kSlots edges, scaling, store
    auto visit = [&](uint32_t row, int32_t b, int32_t e, uint32_t j, float w, auto&& between, auto&& store) {
        float4 acc[kPer];
#pragma unroll
        for (int p = 0; p < kPer; ++p) acc[p] = make_float4(0.f, 0.f, 0.f, 0.f);
        round(b, e, j, w, acc, between);
        if (__any(e - b > kSlots)) {            // read on the spot
            for (int32_t q0 = b + kSlots; __any(q0 < e); q0 += kSlots) {
                uint32_t my_j;
                float my_w;
                edge(q0, e, my_j, my_w);
                round(q0, e, my_j, my_w, acc, []() {});
            }
        }
        const bool some = e > b;                                           // (a row without edges has read nothing: 0)
        const float inv_n = some ? 1.0f / (float) (e - b) : 0.f;           // one division per row, then the products
        float4* o4 = reinterpret_cast<float4*>(a.out + (int64_t) row * F);
#pragma unroll
        for (int p = 0; p < kPer; ++p) {
            const float4 r = make_float4(acc[p].x * inv_n, acc[p].y * inv_n, acc[p].z * inv_n, acc[p].w * inv_n);
            // a lane past the last column has computed the last column once more: it stores the same value there
            store(o4 + (col_bytes[p] >> 4), r);
        }
    };

    int32_t b0, e0, b1, e1;
    uint32_t j0;
    float w0;
    extent(0, b0, e0);
    extent(1, b1, e1);
    edge(b0, e0, j0, w0);
    // every group has a row in all trips but the last: nothing conditional there
    for (uint32_t it = 0; it + 1 < trips; ++it) {
        int32_t b2 = 0, e2 = 0;
        uint32_t j1 = 0;
        float w1 = 0.f;
        visit(group + it * num_groups, b0, e0, j0, w0,
              [&]() {
                  extent(it + 2, b2, e2);       // two rows ahead
                  edge(b1, e1, j1, w1);         // one row ahead
              },
              [](float4* dst, const float4& r) { store_streaming(dst, r); });
        b0 = b1; e0 = e1; b1 = b2; e1 = e2; j0 = j1; w0 = w1;
    }
    const uint32_t row = group + (trips - 1u) * num_groups;
    const bool live = row < count;
    visit(row, b0, e0, j0, w0, []() {}, [&](float4* dst, const float4& r) { if (live) store_streaming(dst, r); });
}

template <int kLanes, int kPer, bool kVec>
__global__ void __launch_bounds__(kBlock) k_aggregate(AggGroup g)
{
    AggArgs a;
    static_cast<AggBatch&>(a) = g.b[blockIdx.y];
    a.feat_dim = g.feat_dim;
    const int lane = (int) (threadIdx.x % kLanes);
    const int64_t groups_per_block = kBlock / kLanes;
    const int64_t group = (int64_t) blockIdx.x * groups_per_block + threadIdx.x / kLanes;
    const int64_t num_groups = (int64_t) gridDim.x * groups_per_block;
    const int64_t F = a.feat_dim;
    const int64_t count = a.num_dst_dev ? (int64_t) *a.num_dst_dev : (int64_t) a.num_dst;
    const uint32_t num_src = (uint32_t) (a.num_src_dev ? *a.num_src_dev : a.num_src);
    constexpr int kEdges = 8;       // edges whose rows are in flight together
    if (count <= 0) return;
    if (num_src == 0) {             // no source row to read (and none may be touched): every edge is skipped
        for (int64_t row = group; row < count; row += num_groups)
            for (int i = lane; i < (int) F; i += kLanes) a.out[row * F + i] = 0.f;
        return;
    }
    if (kVec && kPer == 1 && F <= 4 * kLanes) {
        aggregate_rows_one_column<kLanes>(a, group, num_groups, count, num_src);
        return;
    }
    if (kVec && F <= 4 * kLanes * kPer) {
        if ((uint64_t) num_src * (uint64_t) F * 4u < ((uint64_t) 1 << 32) && num_src < (1u << 24) && F < (1 << 22))
            aggregate_rows<kLanes, kPer, true>(a, (uint32_t) group, (uint32_t) num_groups, (uint32_t) count, num_src);
        else
            aggregate_rows<kLanes, kPer, false>(a, (uint32_t) group, (uint32_t) num_groups, (uint32_t) count, num_src);
        return;
    }
    for (int64_t row = group; row < count; row += num_groups) {
        const int32_t b = a.indptr[row], e = a.indptr[row + 1];
        const float n_v = (float) (e - b);
        if (kVec) {
            const float4* x4 = reinterpret_cast<const float4*>(a.x_src);
            float4* o4 = reinterpret_cast<float4*>(a.out + row * F);
            const int64_t F4 = F >> 2;
            for (int i = lane; i < (int) F4; i += kLanes) {
                float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
                for (int32_t q0 = b; q0 < e; q0 += kEdges) {
                    float w[kEdges];
                    float4 x[kEdges];
#pragma unroll
                    for (int t = 0; t < kEdges; ++t) {
                        const int32_t q = q0 + t;
                        const uint32_t j = (q < e) ? (uint32_t) a.indices[q] : 0xFFFFFFFFu;
                        const bool ok = j < num_src;
                        w[t] = ok ? a.weights[q] : 0.f;
                        x[t] = x4[(int64_t) (ok ? j : 0u) * F4 + i];
                        if (!ok) x[t] = make_float4(0.f, 0.f, 0.f, 0.f);
                    }
#pragma unroll
                    for (int t = 0; t < kEdges; ++t) {       // edge order, one fma per term
                        if (q0 + t < e) {
                            acc.x = fmaf(w[t], x[t].x, acc.x);
                            acc.y = fmaf(w[t], x[t].y, acc.y);
                            acc.z = fmaf(w[t], x[t].z, acc.z);
                            acc.w = fmaf(w[t], x[t].w, acc.w);
                        }
                    }
                }
                if (e > b) { acc.x /= n_v; acc.y /= n_v; acc.z /= n_v; acc.w /= n_v; }
                o4[i] = acc;
            }
        } else {
            for (int i = lane; i < (int) F; i += kLanes) {
                float acc = 0.f;
                for (int32_t q = b; q < e; ++q) {
                    const uint32_t j = (uint32_t) a.indices[q];
                    if (j < num_src) acc = fmaf(a.weights[q], a.x_src[(int64_t) j * F + i], acc);
                }
                if (e > b) acc /= n_v;
                a.out[row * F + i] = acc;
            }
        }
    }
}

template <int kPer, bool kVec>
static void aggregate_dispatch(int lanes, dim3 blocks, hipStream_t s, const AggGroup& a)
{
    switch (lanes) {
        case 4:  hipLaunchKernelGGL((k_aggregate<4, kPer, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        case 8:  hipLaunchKernelGGL((k_aggregate<8, kPer, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        case 16: hipLaunchKernelGGL((k_aggregate<16, kPer, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        case 32: hipLaunchKernelGGL((k_aggregate<32, kPer, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        default: hipLaunchKernelGGL((k_aggregate<64, kPer, kVec>), blocks, dim3(kBlock), 0, s, a); break;
    }
}

hipError_t launch_aggregate(gns_ctx* const* ctxs, int count, const gns_block* const* blks, const float* const* x_src,
                            int32_t feat_dim, float* const* out, hipStream_t s)
{
    gns_ctx* c = ctxs[0];
    if (feat_dim == 0) return hipSuccess;
    AggGroup a;
    memset(&a, 0, sizeof(a));
    int64_t most = 0;
    bool aligned = true;
    for (int b = 0; b < count; ++b) {
        const gns_block* blk = blks[b];
        AggBatch& q = a.b[b];
        int32_t rows = blk->num_dst;
        q.num_src = blk->num_src;
        if (rows < 0) {                 // GNS_DEVICE_COUNTS(layer): rows counted on the device
            const int layer = -1 - rows;
            q.num_dst_dev = &ctxs[b]->d_state->num_dst[layer];
            q.num_src_dev = &ctxs[b]->d_state->num_dst[layer + 1];
            rows = (int32_t) c->lay.rows[layer];
        }
        q.indptr = blk->indptr;
        q.indices = blk->indices;
        q.weights = blk->weights;
        q.x_src = x_src[b];
        q.out = out[b];
        q.num_dst = rows;
        if (rows > most) most = rows;
        aligned = aligned && ((reinterpret_cast<uintptr_t>(x_src[b]) | reinterpret_cast<uintptr_t>(out[b])) & 15u) == 0;
    }
    if (most == 0) return hipSuccess;
    a.feat_dim = feat_dim;
    const int64_t F = feat_dim;
    const bool vec = (F % 4 == 0) && aligned;
    // float4 columns per lane.  Rows that start on cache-line boundaries and are at least two lines long are spread
    // over few lanes with several columns each, which keeps the per-edge bookkeeping small (on 128-float rows 8 lanes
    // x 4 columns is ahead of 16 x 2 and 32 x 1 once other kernels share the chip); other widths take one column per
    // lane, so that a row is read as one contiguous piece.
    const int64_t F4 = F / 4;
    const int per = (vec && F4 % 8 == 0) ? (F4 >= 32 ? 4 : (F4 >= 16 ? 2 : 1)) : 1;
    const int lanes = lanes_for(vec ? (F4 + per - 1) / per : F);
    const int64_t groups_per_block = kBlock / lanes;
    int64_t blocks = (most + groups_per_block - 1) / groups_per_block;
    // Several columns per lane: about the blocks that are resident together (beyond that a group visits several
    // rows, which its pipeline wants anyway); a larger grid is no faster alone and 7 % slower next to another
    // stream's kernels.
    const int64_t cap = (int64_t) c->num_cus * (per > 1 ? 4 : 16);
    if (blocks > cap) blocks = cap;
    const dim3 grid((unsigned) blocks, (unsigned) count);
    if (!vec) aggregate_dispatch<1, false>(lanes, grid, s, a);
    else if (per == 4) aggregate_dispatch<4, true>(lanes, grid, s, a);
    else if (per == 2) aggregate_dispatch<2, true>(lanes, grid, s, a);
    else aggregate_dispatch<1, true>(lanes, grid, s, a);
    return hipGetLastError();
}

}  // namespace gns
