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
    const int64_t cap = (int64_t) c->num_cus * 16;
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
    // Column slices: the chip's 8 XCDs have an L2 each and workgroups go to them round robin, so block
    // x of a launch runs on XCD x % 8.  With `slices` > 1 a block works on float4 columns
    // [slice * kLanes, (slice + 1) * kLanes) of its rows only, slice = (x % 8) % slices: each XCD's L2 then
    // holds one slice of the few thousand hot source rows instead of all of them.
    int32_t slices;
    int32_t fold;       // XCDs that share a slice (8 / slices when that divides, else 1: surplus XCDs' blocks stand down)
};

// the view of one batch the kernel body works on
struct AggArgs : AggBatch {
    int32_t feat_dim;
};

template <int kLanes, bool kVec>
__global__ void __launch_bounds__(kBlock) k_aggregate(AggGroup g)
{
    AggArgs a;
    static_cast<AggBatch&>(a) = g.b[blockIdx.y];
    a.feat_dim = g.feat_dim;
    const int lane = (int) (threadIdx.x % kLanes);
    const int64_t groups_per_block = kBlock / kLanes;
    int64_t group = (int64_t) blockIdx.x * groups_per_block + threadIdx.x / kLanes;
    int64_t num_groups = (int64_t) gridDim.x * groups_per_block;
    const int64_t F = a.feat_dim;
    int col0 = 0;                   // first float4 column of this block's slice
    if (g.slices > 1) {
        const int xcd = (int) (blockIdx.x & 7u);
        const int slice = g.fold > 1 ? xcd % g.slices : xcd;
        if (slice >= g.slices) return;
        const int64_t row_block = g.fold > 1 ? (int64_t) (blockIdx.x >> 3) * g.fold + xcd / g.slices : (int64_t) (blockIdx.x >> 3);
        group = row_block * groups_per_block + threadIdx.x / kLanes;
        num_groups = (int64_t) (gridDim.x >> 3) * g.fold * groups_per_block;
        col0 = slice * kLanes;
    }
    const int64_t count = a.num_dst_dev ? (int64_t) *a.num_dst_dev : (int64_t) a.num_dst;
    const uint32_t num_src = (uint32_t) (a.num_src_dev ? *a.num_src_dev : a.num_src);
    constexpr int kEdges = 8;       // edges whose rows are in flight together
    if (kVec && (g.slices > 1 || F <= 4 * kLanes)) {
        // One float4 per lane covers a row (or the row's column slice).  Branch-free inner loop: the first
        // kSlots lanes of a row's group read one edge each (index and weight, one coalesced read), every lane
        // then takes edge t from lane t of its group, so the reads of up to kSlots source rows are issued back
        // to back; slots past the row's end repeat its last edge with weight 0 (adds an exact 0), rows with
        // more than kSlots edges take further rounds.  All lanes of the wave stay converged: trip counts are
        // wave-uniform (the shuffles need every source lane).
        constexpr int kSlots = kLanes < 8 ? kLanes : 8;
        const int64_t F4 = F >> 2;
        const int col = col0 + lane < (int) F4 ? col0 + lane : (int) F4 - 1;       // idle lanes repeat the last column
        const bool has = col0 + lane < (int) F4;
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
                        const int from = t < here ? t : (here > 0 ? here - 1 : 0);
                        const uint32_t j = (uint32_t) __shfl((int) my_j, from, kLanes);
                        const float wt = __shfl(my_w, from, kLanes);
                        w[t] = t < here ? wt : 0.f;
                        x[t] = by_shift ? x4[j << f4_shift] : x4[(int64_t) j * F4];
                    }
                }
                if (any_bad) {
                    // rare: a skipped edge must not contribute even a NaN of the row it was redirected to
#pragma unroll
                    for (int t = 0; t < kSlots; ++t) {
                        const int from = t < here ? t : (here > 0 ? here - 1 : 0);
                        if (__shfl((int) (bad && mine), from, kLanes)) x[t] = make_float4(0.f, 0.f, 0.f, 0.f);
                    }
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
            if (e > b) {
                const float inv_n = 1.0f / (float) (e - b);           // one division per row, then four products
                acc.x *= inv_n; acc.y *= inv_n; acc.z *= inv_n; acc.w *= inv_n;
            }
            if (live && has) store_streaming(reinterpret_cast<float4*>(a.out + row * F) + col0 + lane, acc);
        }
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

template <bool kVec>
static void aggregate_dispatch(int lanes, dim3 blocks, hipStream_t s, const AggGroup& a)
{
    switch (lanes) {
        case 4:  hipLaunchKernelGGL((k_aggregate<4, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        case 8:  hipLaunchKernelGGL((k_aggregate<8, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        case 16: hipLaunchKernelGGL((k_aggregate<16, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        case 32: hipLaunchKernelGGL((k_aggregate<32, kVec>), blocks, dim3(kBlock), 0, s, a); break;
        default: hipLaunchKernelGGL((k_aggregate<64, kVec>), blocks, dim3(kBlock), 0, s, a); break;
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
    int lanes = lanes_for(vec ? F / 4 : F);
    a.slices = 1;
    a.fold = 1;
    if (vec && F / 4 >= 16 && getenv("GNS_AGG_SLICES")) {
        // at least 8 lanes (128 bytes, one cache line) of a row per slice, at most 8 slices
        lanes = 8;
        if (const char* e = getenv("GNS_AGG_SLICE_LANES")) lanes = atoi(e) >= 4 ? atoi(e) : 8;
        while (lanes * 8 < F / 4) lanes <<= 1;
        a.slices = (int32_t) ((F / 4 + lanes - 1) / lanes);
        a.fold = (8 % a.slices == 0) ? 8 / a.slices : 1;
    }
    const int64_t groups_per_block = kBlock / lanes;
    int64_t blocks = (most + groups_per_block - 1) / groups_per_block;
    const int64_t cap = (int64_t) c->num_cus * 16;
    if (a.slices > 1) {
        // row blocks per (8 / fold) ... every group of 8 consecutive blocks covers `fold` row blocks in all slices
        int64_t row_blocks = (blocks + a.fold - 1) / a.fold;
        if (row_blocks * 8 > cap * 2) row_blocks = cap * 2 / 8;
        if (row_blocks < 1) row_blocks = 1;
        blocks = row_blocks * 8;
    } else if (blocks > cap) {
        blocks = cap;
    }
    const dim3 grid((unsigned) blocks, (unsigned) count);
    if (vec) aggregate_dispatch<true>(lanes, grid, s, a);
    else     aggregate_dispatch<false>(lanes, grid, s, a);
    return hipGetLastError();
}

}  // namespace gns
