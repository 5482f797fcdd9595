// The update step of one layer (paper Algorithm 1, h_u = g(W . (h_u, h_N(u))), GraphSAGE form of
// Section 2.1), forward only:  out = g([h_self | h_neigh] . W + bias).  This is the one dense
// contraction of the path, so it runs on the matrix cores: fp32 MFMA 32x32x2, fp32 accumulate.
//
// Tiling: a block of 256 threads (4 waves, 2 x 2) owns a 128 x 128 tile of the output and walks K in
// steps of 32.  The A (activations, concatenated on the fly from the two inputs) and B (weights)
// tiles of a step are staged in LDS k-major; lane l feeds A[m = l % 32][k = l / 32] and
// B[k = l / 32][n = l % 32] of a 32 x 32 product.  Inside an LDS row the 128 columns are permuted so
// that the two 32 x 32 tiles a wave needs sit side by side (column c = 64*w + 32*t + i is stored at
// 64*w + 2*i + t): one 8-byte LDS read then brings a lane's operands for both tiles, and every read of
// the K loop is the same base address plus a constant.  The tiles of the next step are fetched into
// registers while the current step multiplies.  Each wave keeps
// 2 x 2 accumulator tiles of 32 x 32 (64 VGPRs); element v of lane l is row 8*(v/4) + 4*(l/32) + v%4,
// column l % 32 of its tile.
#include "gns_internal.h"
#include "gns_device.hpp"

namespace gns {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kDM = 128, kDN = 128, kDK = 32;
constexpr int kDFetch = kDM * kDK / 4 / kBlock;  // float4 per thread and operand tile
constexpr int kDPad = 4;                      // keeps 16-byte alignment of LDS rows, spreads the transposed writes

// position of tile column c (0..127) inside an LDS row
__device__ __forceinline__ int dense_slot(int c) { return (c & 64) | ((c & 31) << 1) | ((c >> 5) & 1); }

struct DenseArgs {
    const float* a1;
    const float* a2;
    const float* w;
    const float* bias;
    float* out;
    int32_t f1, f2, hdim, relu;
    int32_t rows;
    const int32_t* rows_dev;                  // if not null the row count is read here (rows is then the worst case)
};

// at least two blocks per CU: one block's fetch, staging and epilogue run under another's products
__global__ void __launch_bounds__(kBlock, 2) k_sage_dense(DenseArgs a)
{
    __shared__ float As[kDK][kDM + kDPad];
    __shared__ float Bs[kDK][kDN + kDPad];
    const int32_t rows = a.rows_dev ? *a.rows_dev : a.rows;
    const int32_t m0 = (int32_t) blockIdx.x * kDM, n0 = (int32_t) blockIdx.y * kDN;
    if (m0 >= rows) return;
    const int32_t K = a.f1 + a.f2;
    const int tid = (int) threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    float4 ra[kDFetch], rb[kDFetch];
    constexpr int kA4 = kDK / 4;                     // float4 per A-tile row
    auto fetch = [&](int32_t k0) {
#pragma unroll
        for (int j = 0; j < kDFetch; ++j) {
            const int idx = tid + j * kBlock;
            {   // A: 128 rows x kDK / 4 float4
                const int row = idx / kA4, k = k0 + (idx % kA4) * 4;
                const int64_t gr = (int64_t) m0 + row;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (gr < rows && k < K) {
                    const float* p = (k < a.f1) ? a.a1 + gr * a.f1 + k : a.a2 + gr * a.f2 + (k - a.f1);
                    v = *reinterpret_cast<const float4*>(p);
                }
                ra[j] = v;
            }
            {   // B: kDK k-rows x 32 float4
                const int kr = idx >> 5, n = n0 + (idx & 31) * 4, k = k0 + kr;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < K && n < a.hdim) v = *reinterpret_cast<const float4*>(a.w + (int64_t) k * a.hdim + n);
                rb[j] = v;
            }
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int j = 0; j < kDFetch; ++j) {
            const int idx = tid + j * kBlock;
            const int row = dense_slot(idx / kA4), kc = (idx % kA4) * 4;
            As[kc + 0][row] = ra[j].x;
            As[kc + 1][row] = ra[j].y;
            As[kc + 2][row] = ra[j].z;
            As[kc + 3][row] = ra[j].w;
            const int kr = idx >> 5, nc = (idx & 31) * 4;
            Bs[kr][dense_slot(nc + 0)] = rb[j].x;
            Bs[kr][dense_slot(nc + 1)] = rb[j].y;
            Bs[kr][dense_slot(nc + 2)] = rb[j].z;
            Bs[kr][dense_slot(nc + 3)] = rb[j].w;
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][nt][v] = 0.f;

    fetch(0);
    stage();
    __syncthreads();
    const int kh = lane >> 5, l32 = lane & 31;
    for (int32_t k0 = 0; k0 < K; k0 += kDK) {
        const bool more = k0 + kDK < K;
        if (more) fetch(k0 + kDK);
        // a lane's operands of both tiles in one 8-byte read; the reads of step kk + 2 are issued before
        // the products of step kk
        const float2* arow = reinterpret_cast<const float2*>(&As[kh][wm * 64 + l32 * 2]);
        const float2* brow = reinterpret_cast<const float2*>(&Bs[kh][wn * 64 + l32 * 2]);
        constexpr int kRow2 = (kDM + kDPad) / 2;                       // LDS row stride in float2
        float2 af[2], bf[2];
        af[0] = arow[0];
        bf[0] = brow[0];
#pragma unroll
        for (int kk = 0; kk < kDK; kk += 2) {
            const int cur = (kk >> 1) & 1;
            if (kk + 2 < kDK) {
                af[cur ^ 1] = arow[(kk + 2) * kRow2];
                bf[cur ^ 1] = brow[(kk + 2) * kRow2];
            }
            __builtin_amdgcn_sched_barrier(0);          // the reads above stay ahead of the products below
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur].x, bf[cur].x, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur].x, bf[cur].y, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur].y, bf[cur].x, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur].y, bf[cur].y, acc[1][1], 0, 0, 0);
        }
        __syncthreads();
        if (more) {
            stage();
            __syncthreads();
        }
    }

#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int32_t col = n0 + wn * 64 + nt * 32 + l32;
            const float b = (a.bias && col < a.hdim) ? a.bias[col] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = (int64_t) m0 + wm * 64 + mt * 32 + 8 * (v >> 2) + 4 * kh + (v & 3);
                if (row < rows && col < a.hdim) {
                    float x = acc[mt][nt][v] + b;
                    if (a.relu) x = fmaxf(x, 0.f);
                    a.out[row * a.hdim + col] = x;
                }
            }
        }
    }
}

hipError_t launch_sage_dense(gns_ctx* c, const float* h_self, int32_t f1, const float* h_neigh, int32_t f2,
                             const float* w, const float* bias, int32_t hdim, int32_t relu, float* out,
                             int32_t num_rows, hipStream_t s)
{
    if (num_rows == 0) return hipSuccess;
    DenseArgs a;
    a.a1 = h_self; a.a2 = h_neigh; a.w = w; a.bias = bias; a.out = out;
    a.f1 = f1; a.f2 = f2; a.hdim = hdim; a.relu = relu;
    a.rows_dev = nullptr;
    int32_t rows = num_rows;
    if (rows < 0) {                 // GNS_DEVICE_COUNTS(layer): rows counted on the device
        const int layer = -1 - rows;
        a.rows_dev = &c->d_state->num_dst[layer];
        rows = (int32_t) c->lay.rows[layer];
    }
    a.rows = rows;
    const dim3 grid((unsigned) ((rows + kDM - 1) / kDM), (unsigned) ((hdim + kDN - 1) / kDN));
    hipLaunchKernelGGL(k_sage_dense, grid, dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

}  // namespace gns
