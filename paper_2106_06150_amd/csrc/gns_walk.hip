// Random-walk cache probability (paper Section 3.2, second approach):
//   P^0 = uniform on the training nodes,  P^l = (D_l A + I) P^(l-1),  D_l = diag(min(k_l, deg)/deg),
// kept in integer units (2^scale per training node, every step rounded down) so that the result
// is independent of the order of the additions; then its exclusive prefix sum, which takes the
// place of the CSR offsets in the cache draw (a uniform integer below the total picks the node
// whose prefix interval holds it) and in Section 3.4's p_u.
#include "gns_internal.h"
#include "gns_device.hpp"

namespace gns {

constexpr unsigned long long kWalkLimit = 1ull << 62;     // sums, products and the total stay below this
constexpr int kWalkLanes = 16;                             // lanes per row in a step

__global__ void __launch_bounds__(kBlock) k_walk_seed(const int32_t* train, int64_t num_train, int64_t n,
                                                      unsigned long long unit, unsigned long long* cur, DeviceState* st)
{
    const int64_t t = (int64_t) blockIdx.x * kBlock + threadIdx.x;
    if (t >= num_train) return;
    const int32_t v = train[t];
    if (v < 0 || (int64_t) v >= n) { st->walk_error = 1; return; }
    cur[v] = unit;
}

// Addition that sticks at kWalkLimit.  Operands are at most kWalkLimit, so the plain sum fits in
// 64 bits; min(limit, a + b) is associative and commutative, so sums and scans may be taken in any
// order, are exact whenever the true result is below the limit, and equal the limit otherwise.
__device__ __forceinline__ unsigned long long sat_add(unsigned long long a, unsigned long long b)
{
    const unsigned long long s = a + b;
    return s < kWalkLimit ? s : kWalkLimit;
}

// One step: nxt[i] = cur[i] + floor(min(k, deg_i) * sum_{j in N(i)} cur[j] / deg_i).
template <typename OffT>
__global__ void __launch_bounds__(kBlock) k_walk_step(const void* indptr, const int32_t* indices, int64_t n, int32_t k,
                                                      const unsigned long long* cur, unsigned long long* nxt,
                                                      DeviceState* st)
{
    constexpr int G = kWalkLanes;
    const int64_t group = ((int64_t) blockIdx.x * kBlock + threadIdx.x) / G;
    const int64_t num_groups = (int64_t) gridDim.x * kBlock / G;
    for (int64_t i = group; i < n; i += num_groups) {
        const int lane = opaque_lane_id() & (G - 1);             // see opaque(): the loop exchanges data between lanes
        const int64_t b = load_off<OffT>(indptr, i), e = load_off<OffT>(indptr, i + 1);
        unsigned long long sum = 0;
        for (int64_t q = b + lane; q < e; q += G) sum = sat_add(sum, cur[indices[q]]);
#pragma unroll
        for (int d = G / 2; d > 0; d >>= 1) sum = sat_add(sum, __shfl_xor(sum, d, G));
        if (lane == 0) {
            const unsigned long long deg = (unsigned long long) (e - b);
            bool bad = sum >= kWalkLimit;
            unsigned long long out = cur[i];
            if (deg > 0 && !bad) {
                const unsigned long long kk = (unsigned long long) k < deg ? (unsigned long long) k : deg;
                const unsigned long long quo = sum / deg, rem = sum % deg;
                bad = quo >= kWalkLimit / 64;                  // kk <= 64: the product below stays under the limit
                if (!bad) out = sat_add(out, kk * quo + (kk * rem) / deg);
            }
            bad |= out >= kWalkLimit;
            nxt[i] = bad ? 0ull : out;
            if (bad) st->walk_error = 2;
        }
    }
}

// Exclusive prefix sum of n 64-bit values in three phases (tile sums, one block over the tile
// sums, per-tile scan) with the saturating addition above, plus the number of non-zero values.
__device__ __forceinline__ unsigned long long wave_inclusive_sat_scan(unsigned long long v)
{
    const int lane = opaque_lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const unsigned long long up = __shfl_up(v, d, kWave);
        if (lane >= d) v = sat_add(v, up);
    }
    return v;
}

// exclusive scan over the block; *total = block sum.  smem: kBlock / kWave + 1 values
__device__ __forceinline__ unsigned long long block_exclusive_sat_scan(unsigned long long v, unsigned long long* smem,
                                                                        unsigned long long* total)
{
    const int lane = opaque_lane_id();
    const int wave = opaque((int) (threadIdx.x >> 6));
    constexpr int kWaves = kBlock / kWave;
    const unsigned long long incl = wave_inclusive_sat_scan(v);
    const unsigned long long before_in_wave = __shfl_up(incl, 1, kWave);
    __syncthreads();
    if (lane == kWave - 1) smem[wave] = incl;
    __syncthreads();
    unsigned long long base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const unsigned long long s = smem[w];
        if (w < wave) base = sat_add(base, s);
        sum = sat_add(sum, s);
    }
    *total = sum;
    return lane == 0 ? base : sat_add(base, before_in_wave);
}

__global__ void __launch_bounds__(kBlock) k_walk_scan_phase1(const unsigned long long* w, int64_t n,
                                                             unsigned long long* tile_sums, int32_t* tile_nonzero)
{
    __shared__ unsigned long long smem[kBlock / kWave + 1];
    __shared__ int32_t smem32[kBlock / kWave + 1];
    const int64_t base = (int64_t) blockIdx.x * kTile + (int64_t) threadIdx.x * kItems;
    unsigned long long sum = 0;
    int32_t nz = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const unsigned long long x = (base + i < n) ? w[base + i] : 0ull;
        sum = sat_add(sum, x);
        nz += x ? 1 : 0;
    }
    unsigned long long total;
    (void) block_exclusive_sat_scan(sum, smem, &total);
    const int32_t nzt = block_sum(nz, smem32);
    if (threadIdx.x == 0) {
        tile_sums[blockIdx.x] = total;
        tile_nonzero[blockIdx.x] = nzt;
    }
}

__global__ void __launch_bounds__(kBlock) k_walk_scan_phase2(unsigned long long* tile_sums, const int32_t* tile_nonzero,
                                                             int64_t tiles, DeviceState* st)
{
    __shared__ unsigned long long smem[kBlock / kWave + 1];
    __shared__ int32_t smem32[kBlock / kWave + 1];
    unsigned long long carry = 0;
    int32_t nz = 0;
    for (int64_t base = 0; base < tiles; base += kBlock) {
        const int64_t i = base + threadIdx.x;
        const unsigned long long v = (i < tiles) ? tile_sums[i] : 0ull;
        unsigned long long total;
        const unsigned long long ex = block_exclusive_sat_scan(v, smem, &total);
        if (i < tiles) tile_sums[i] = sat_add(carry, ex);
        carry = sat_add(carry, total);
        nz += block_sum((i < tiles) ? tile_nonzero[i] : 0, smem32);
    }
    if (threadIdx.x == 0) {
        st->walk_total = carry;
        st->walk_support = nz;
        if (carry >= kWalkLimit) st->walk_error = 2;
    }
}

__global__ void __launch_bounds__(kBlock) k_walk_scan_phase3(const unsigned long long* w, int64_t n,
                                                             const unsigned long long* tile_offsets,
                                                             long long* prefix, const DeviceState* st)
{
    __shared__ unsigned long long smem[kBlock / kWave + 1];
    const int64_t base = (int64_t) blockIdx.x * kTile + (int64_t) threadIdx.x * kItems;
    unsigned long long x[kItems];
    unsigned long long sum = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        x[i] = (base + i < n) ? w[base + i] : 0ull;
        sum = sat_add(sum, x[i]);
    }
    unsigned long long total;
    unsigned long long off = sat_add(tile_offsets[blockIdx.x], block_exclusive_sat_scan(sum, smem, &total));
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        if (base + i < n) prefix[base + i] = (long long) off;
        off = sat_add(off, x[i]);
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) prefix[n] = (long long) st->walk_total;
}

gns_status run_walk_probability(gns_ctx* c, const int32_t* train_nodes, int64_t num_train, int32_t scale_log2,
                                hipStream_t s)
{
    const Layout& L = c->lay;
    const int64_t n = c->graph.num_nodes;
    gns_ctx* root = c->root;
    root->prob_valid = false;
    unsigned long long* cur = ws_ptr<unsigned long long>(c, L.walk_a);
    unsigned long long* nxt = ws_ptr<unsigned long long>(c, L.walk_b);
    long long* prefix = ws_ptr<long long>(c, L.prob_prefix);
    unsigned long long* tile_sums = ws_ptr<unsigned long long>(c, L.walk_tiles);
    int32_t* tile_nz = ws_ptr<int32_t>(c, L.walk_tiles_nz);

    hipError_t e = launch_fill_u64(cur, (size_t) n, 0ull, s);
    if (e == hipSuccess) e = launch_fill_u32(reinterpret_cast<uint32_t*>(&c->d_state->walk_error), 1, 0u, s);
    if (e != hipSuccess) return ctx_fail(c, GNS_EHIP, "walk init", e);
    hipLaunchKernelGGL(k_walk_seed, dim3((unsigned) ((num_train + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, train_nodes,
                       num_train, n, 1ull << scale_log2, cur, c->d_state);
    const bool i64 = c->graph.indptr_is_i64 != 0;
    int64_t blocks = (n * kWalkLanes + kBlock - 1) / kBlock;
    const int64_t cap = (int64_t) c->num_cus * 64;
    if (blocks > cap) blocks = cap;
    for (int l = 0; l < c->config.num_layers; ++l) {
        const int32_t k = c->config.fanout[l];
        if (i64) hipLaunchKernelGGL((k_walk_step<int64_t>), dim3((unsigned) blocks), dim3(kBlock), 0, s, c->graph.indptr,
                                    c->graph.indices, n, k, cur, nxt, c->d_state);
        else     hipLaunchKernelGGL((k_walk_step<int32_t>), dim3((unsigned) blocks), dim3(kBlock), 0, s, c->graph.indptr,
                                    c->graph.indices, n, k, cur, nxt, c->d_state);
        unsigned long long* t = cur; cur = nxt; nxt = t;
    }
    const int64_t tiles = (n + kTile - 1) / kTile;
    hipLaunchKernelGGL(k_walk_scan_phase1, dim3((unsigned) tiles), dim3(kBlock), 0, s, cur, n, tile_sums, tile_nz);
    hipLaunchKernelGGL(k_walk_scan_phase2, dim3(1), dim3(kBlock), 0, s, tile_sums, tile_nz, tiles, c->d_state);
    hipLaunchKernelGGL(k_walk_scan_phase3, dim3((unsigned) tiles), dim3(kBlock), 0, s, cur, n, tile_sums, prefix, c->d_state);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(c->h_state, c->d_state, sizeof(DeviceState), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return ctx_fail(c, GNS_EHIP, "walk probability", e);
    if (c->h_state->walk_error == 1) return ctx_fail(c, GNS_EINVAL, "a training node id lies outside [0, num_nodes)");
    if (c->h_state->walk_error) return ctx_fail(c, GNS_ECAPACITY, "the walk probability does not fit in 62 bits: lower scale_log2");
    if (c->h_state->walk_total == 0) return ctx_fail(c, GNS_EINVAL, "the walk probability is zero everywhere");
    root->prob_weights = cur;
    root->prob_total = c->h_state->walk_total;
    root->prob_support = c->h_state->walk_support;
    root->prob_valid = true;
    return GNS_OK;
}

}  // namespace gns
