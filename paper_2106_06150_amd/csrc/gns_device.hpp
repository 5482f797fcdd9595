// Device-side building blocks shared by the GNS kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gns {

constexpr int kWave = 64;
constexpr int kBlock = 256;                 // threads per block for the scan-style kernels
constexpr int kItems = 8;                   // items per thread in a scan tile
constexpr int kTile = kBlock * kItems;      // 2048 items per scan tile
constexpr int kMarkTileMin = 64;             // frontier mark bitmap: words per tile, a power of two chosen per graph
constexpr int kMarkTileMax = 32 * kBlock;    //   so that the tiles number about a hundred (at most 32 words per thread)
constexpr int kMarkCap = 1024;               // marked words of a tile the union step keeps in LDS at a time

constexpr uint32_t kTagCache = 0x43414348u;     // 'CACH'
constexpr uint32_t kTagNeighbor = 0x4E424853u;  // 'NBHS'

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  One call yields four 32-bit words.
struct Philox4 {
    uint32_t w[4];
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1)
{
    constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
    constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t a_hi = __umulhi(kMulA, c0), a_lo = kMulA * c0;
        const uint32_t b_hi = __umulhi(kMulB, c2), b_lo = kMulB * c2;
        c0 = b_hi ^ c1 ^ k0;
        c1 = b_lo;
        c2 = a_hi ^ c3 ^ k1;
        c3 = a_lo;
        k0 += kWeylA;
        k1 += kWeylB;
    }
    Philox4 out;
    out.w[0] = c0; out.w[1] = c1; out.w[2] = c2; out.w[3] = c3;
    return out;
}

// ---------------------------------------------------------------------------
// CSR offsets may be int32 or int64.
template <typename OffT>
__device__ __forceinline__ int64_t load_off(const void* indptr, int64_t i)
{
    return (int64_t) reinterpret_cast<const OffT*>(indptr)[i];
}

// Same with the offset width chosen at run time (kernels that touch offsets only in passing).
__device__ __forceinline__ int64_t load_off_rt(const void* indptr, int is_i64, int64_t i)
{
    return is_i64 ? load_off<int64_t>(indptr, i) : load_off<int32_t>(indptr, i);
}

// CSR extent [start, end) of one dst row's node, kept per row of the batch's node list.
struct alignas(16) RowExtent {
    int64_t start, end;
};

// ---------------------------------------------------------------------------
// Open-addressing hash map node id -> local id, one 64-bit slot per entry
// (low word = key, high word = value), linear probing, load factor <= 1/2.
constexpr uint64_t kEmptySlot = 0xFFFFFFFFFFFFFFFFull;

__device__ __forceinline__ uint32_t hash_start(uint32_t key, uint32_t shift)
{
    return (key * 0x9E3779B1u) >> shift;    // shift = 32 - log2(capacity)
}

// returns the slot the entry went into, or -1 if the key was already present (or the table is full)
__device__ __forceinline__ int64_t hash_insert(unsigned long long* slots, uint32_t mask, uint32_t shift,
                                               uint32_t key, uint32_t val)
{
    const unsigned long long entry = ((unsigned long long) val << 32) | key;
    uint32_t h = hash_start(key, shift);
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        const unsigned long long old = atomicCAS(&slots[h], (unsigned long long) kEmptySlot, entry);
        if (old == kEmptySlot) return (int64_t) h;
        if ((uint32_t) old == key) return -1;
        h = (h + 1) & mask;
    }
    return -1;
}

// local id of `key`, or -1 if absent
__device__ __forceinline__ int32_t hash_lookup(const unsigned long long* slots, uint32_t mask, uint32_t shift,
                                               uint32_t key)
{
    uint32_t h = hash_start(key, shift);
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        const unsigned long long s = slots[h];
        if ((uint32_t) s == key && s != kEmptySlot) return (int32_t) (s >> 32);
        if (s == kEmptySlot) return -1;
        h = (h + 1) & mask;
    }
    return -1;
}

// ---------------------------------------------------------------------------
// Wave and block scans (wave64).
__device__ __forceinline__ int lane_id() { return (int) (threadIdx.x & (kWave - 1)); }

// Lane / thread ids the optimiser cannot prove loop-invariant.  A branch on a lane id inside
// a loop that also exchanges data between lanes (shuffles, ballots, readfirstlane, barriers)
// must use these: if the optimiser hoists such a branch out of the loop, the wave is split
// into per-lane-class copies of the loop and the cross-lane operations no longer see all of
// their lanes (observed as lanes spinning forever on a stale row index).
__device__ __forceinline__ int opaque(int x)
{
    asm volatile("" : "+v"(x));
    return x;
}
__device__ __forceinline__ int opaque_lane_id() { return opaque(lane_id()); }

__device__ __forceinline__ int32_t wave_inclusive_scan(int32_t v)
{
    const int lane = opaque_lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int32_t up = __shfl_up(v, d, kWave);
        if (lane >= d) v += up;
    }
    return v;
}

__device__ __forceinline__ int32_t wave_sum(int32_t v)
{
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

// Exclusive scan over the kBlock threads of a block; *total receives the block
// sum in every thread.  `smem` must hold kBlock / kWave + 1 ints.
__device__ __forceinline__ int32_t block_exclusive_scan(int32_t v, int32_t* smem, int32_t* total)
{
    const int lane = opaque_lane_id();
    const int wave = opaque((int) (threadIdx.x >> 6));
    constexpr int kWaves = kBlock / kWave;
    const int32_t incl = wave_inclusive_scan(v);
    __syncthreads();                         // smem may still be read from a previous call
    if (lane == kWave - 1) smem[wave] = incl;
    __syncthreads();
    int32_t base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int32_t s = smem[w];
        if (w < wave) base += s;
        sum += s;
    }
    *total = sum;
    return base + incl - v;
}

__device__ __forceinline__ int32_t block_sum(int32_t v, int32_t* smem)
{
    const int lane = opaque_lane_id();
    const int wave = opaque((int) (threadIdx.x >> 6));
    constexpr int kWaves = kBlock / kWave;
    const int32_t s = wave_sum(v);
    __syncthreads();
    if (lane == 0) smem[wave] = s;
    __syncthreads();
    int32_t sum = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) sum += smem[w];
    return sum;
}

// index of the n-th (0-based) set bit of a 64-bit mask that has more than n bits set
__device__ __forceinline__ int select_bit64(uint64_t mask, int n)
{
    int pos = 0;
#pragma unroll
    for (int width = 32; width >= 1; width >>= 1) {
        const uint64_t low = mask & ((1ull << width) - 1ull);
        const int c = __popcll(low);
        if (n >= c) { n -= c; mask >>= width; pos += width; }
        else        { mask = low; }
    }
    return pos;
}

// rank of node u among the set bits of a bitmap with a per-word exclusive prefix
__device__ __forceinline__ int32_t bitmap_rank(const uint64_t* bitmap, const int32_t* word_prefix, uint32_t u)
{
    const uint64_t word = bitmap[u >> 6];
    return word_prefix[u >> 6] + __popcll(word & ((1ull << (u & 63u)) - 1ull));
}

__device__ __forceinline__ bool bitmap_test(const uint64_t* bitmap, uint32_t u)
{
    const uint32_t* words32 = reinterpret_cast<const uint32_t*>(bitmap);
    return (words32[u >> 5] >> (u & 31u)) & 1u;
}

}  // namespace gns
